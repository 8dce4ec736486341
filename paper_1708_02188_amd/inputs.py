"""Seeded synthetic inputs: binding of libddlgen plus the workload shapes.

This module serves both the tests' oracle side (host arrays) and the HIP side (device
fills) and contains none of the allreduce's arithmetic.  The paper's workloads are
ImageNet training runs of ResNet-50 (about 100 MB of gradients, Sec. 5.1) and of
ResNet-101 with a 22K-class head (about 350 MB, Sec. 4.3 / 5.2); buffers of those sizes
filled from a counter-based generator stand in for the gradients.
"""
import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))

DDLGEN_INT8, DDLGEN_UNIFORM, DDLGEN_NORMAL = 0, 1, 2
DIST = {"int8": DDLGEN_INT8, "uniform": DDLGEN_UNIFORM, "normal": DDLGEN_NORMAL}

BASE_SEED = 170802188


def library_path():
    return os.environ.get("DDLGEN_LIBRARY") or os.path.join(_PKG, "libddlgen.so")


def _load():
    try:
        import torch  # noqa: F401  (its bundled HIP runtime must be the process's only one)
    except ImportError:
        pass
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_1708_02188_amd.build`")
    lib = ctypes.CDLL(path)
    lib.ddlgen_fill_host.restype = ctypes.c_int
    lib.ddlgen_fill_host.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64,
                                     ctypes.c_uint32, ctypes.c_size_t, ctypes.c_int]
    lib.ddlgen_fill_device.restype = ctypes.c_int
    lib.ddlgen_fill_device.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64,
                                       ctypes.c_uint32, ctypes.c_size_t, ctypes.c_int,
                                       ctypes.c_void_p]
    return lib


_lib = _load()


def fill_host(n, seed, learner, dist, first=0):
    """fp32 numpy array with elements first..first+n-1 of `learner`'s buffer."""
    out = np.empty(n, dtype=np.float32)
    rc = _lib.ddlgen_fill_host(out.ctypes.data, n, seed, learner, first, DIST.get(dist, dist))
    if rc != 0:
        raise ValueError(f"ddlgen_fill_host failed ({rc})")
    return out


def fill_device(tensor, seed, learner, dist, first=0, stream=None):
    """Fill a contiguous fp32 device tensor in place with the same values."""
    assert tensor.is_contiguous() and tensor.element_size() == 4 and tensor.is_cuda
    s = getattr(stream, "cuda_stream", stream)
    rc = _lib.ddlgen_fill_device(tensor.data_ptr(), tensor.numel(), seed, learner, first,
                                 DIST.get(dist, dist), s)
    if rc != 0:
        raise RuntimeError(f"ddlgen_fill_device failed ({rc})")
    return tensor


# ---------------------------------------------------------------------------------------
# Workload shapes
# ---------------------------------------------------------------------------------------
def resnet_shapes(blocks, num_classes):
    """Parameter tensor shapes of a bottleneck ResNet in definition order.

    Stem 7x7 convolution with 64 filters + batch norm; four stages of bottleneck blocks of
    widths 64/128/256/512 (1x1, 3x3, 1x1 to four times the width, each followed by a batch
    norm's weight and bias), a 1x1 projection + batch norm on the first block of every
    stage; a fully connected head.  Convolutions carry no bias.
    """
    shapes = [(64, 3, 7, 7), (64,), (64,)]
    inplanes = 64
    for stage, nblocks in enumerate(blocks):
        width = 64 * 2 ** stage
        for b in range(nblocks):
            shapes += [(width, inplanes, 1, 1), (width,), (width,),
                       (width, width, 3, 3), (width,), (width,),
                       (4 * width, width, 1, 1), (4 * width,), (4 * width,)]
            if b == 0:
                shapes += [(4 * width, inplanes, 1, 1), (4 * width,), (4 * width,)]
            inplanes = 4 * width
    shapes += [(num_classes, inplanes), (num_classes,)]
    return shapes


def numel(shapes):
    return int(sum(int(np.prod(s)) for s in shapes))


def tensor_segments(shapes):
    """(offsets, counts) of the tensors laid end to end in definition order."""
    offs, cnts, pos = [], [], 0
    for shp in shapes:
        n = int(np.prod(shp))
        offs.append(pos)
        cnts.append(n)
        pos += n
    return offs, cnts


def resnet50_shapes():
    return resnet_shapes([3, 4, 6, 3], 1000)


def resnet101_22k_shapes():
    return resnet_shapes([3, 4, 23, 3], 21841)


RESNET50_COUNT = 25557032
RESNET101_22K_COUNT = 87252369

# The five configurations: P learners, box dims, elements per learner, value distribution.
CONFIGS = [
    dict(name="c1_ring4_int", P=4, dims=[4], count=1 << 20, dist="int8", seed=BASE_SEED + 1),
    dict(name="c2_box4x4_resnet50", P=16, dims=[4, 4], count=RESNET50_COUNT, dist="uniform",
         seed=BASE_SEED + 2),
    dict(name="c3_box4x16_resnet50_layers", P=64, dims=[4, 16], count=RESNET50_COUNT,
         dist="normal", seed=BASE_SEED + 3),
    dict(name="c4_box4x8x8_resnet50", P=256, dims=[4, 8, 8], count=RESNET50_COUNT,
         dist="uniform", seed=BASE_SEED + 4),
    dict(name="c5_box4x8x8_resnet101_22k", P=256, dims=[4, 8, 8], count=RESNET101_22K_COUNT,
         dist="normal", seed=BASE_SEED + 5),
]
