"""Compile the in-tree HIP libraries for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_1708_02188_amd.build        # builds libddlsim.so and libddlgen.so

Extra -D options (kernel tuning knobs of csrc/kernels.hip) can be given via the
environment variable DDLSIM_CXXFLAGS, and another output directory via DDLSIM_OUT.
"""
import os
import shlex
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")

COMMON = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-Wall",
    # packed fp32 instructions are kept out of every kernel (one rounding per scalar add)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off",
]

SIM_SOURCES = ["plan.cpp", "api.cpp", "kernels.hip"]
LIBS = {
    "libddlsim.so": (SIM_SOURCES, []),
    "libddlgen.so": (["ddlgen.hip"], []),
    # The same library with tiny launch limits, so that inputs of test size run the paths
    # that only huge inputs reach otherwise: the kernels' stride over the tiles a capped grid
    # leaves, and the split of a several-tensor phase into more than one launch.  Loaded by
    # the GPU tests through DDLSIM_LIBRARY; never by the product.
    "libddlsim_smallgrid.so": (SIM_SOURCES, ["-DDDL_MAX_GRID_THREADS=65536", "-DDDL_LIST_PER_LAUNCH=1000"]),
}


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build_all(out_dir=None, extra_flags=None, verbose=True):
    out_dir = out_dir or os.environ.get("DDLSIM_OUT") or PKG
    extra = list(extra_flags or []) + shlex.split(os.environ.get("DDLSIM_CXXFLAGS", ""))
    os.makedirs(out_dir, exist_ok=True)
    def one(item):
        lib, (sources, flags) = item
        out = os.path.join(out_dir, lib)
        cmd = [hipcc()] + COMMON + flags + extra + ["-o", out] + [os.path.join(CSRC, s) for s in sources]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return out

    # the libraries are independent: compile them side by side
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(len(LIBS)) as pool:
        return list(pool.map(one, LIBS.items()))


if __name__ == "__main__":
    build_all()
    sys.exit(0)
