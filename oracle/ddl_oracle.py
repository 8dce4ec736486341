"""Plain CPU oracle of the multi-dimensional ring ("multi-ring") allreduce.

TEST INFRASTRUCTURE ONLY.  Single-threaded numpy, written for a reader who wants
to check it against the paper by eye; nothing here is blocked, fused or tuned.
It shares no code with the HIP library and must never import it; only tests, the
smoke check and the benchmark's CPU-baseline leg may import this module.

What the paper fixes (Sec. 4.3, "Topology aware communication"):
  * the result: R = sum_{j=1..N} V_j, delivered to every learner;
  * a ring over N nodes reduces in N-1 phases, each phase being N concurrent
    transfers of an N-th of the data each, and the result then has to be copied to all
    learners with the same amount of traffic;
  * the multi-dimensional variant places the N learners in an m-dimensional box
    with N = d_1 * d_2 * ... * d_m, dimension 1 riding the fastest links;
  * the cost estimate T ~ sum_{j=1}^{N-1} (S / (N * B_min) + L) of one ring pass.
What the paper names as operations (Sec. 4.1): assignment (copy), ReduceScatter
and AllGather over a set of objects, one per learner.

What the paper does NOT fix, and this oracle therefore takes as a stated reading:
rank <-> box-coordinate numbering, ring direction, which chunk travels first, how
a buffer whose length does not divide evenly is chunked, and that the gather
runs through the dimensions in reverse.  Those readings are the functions
`coords`, `neighbour`, `split`, `schedule` below.

PIN STATUS
  * value of the result (the element-wise sum on every learner): pinned by brute
    force against integer arithmetic, by an fp64 sum with the rounding-error
    bound of the schedule, and by special cases that collapse to numpy routines.
  * fp32 association order (which of the many valid summation orders): the paper
    prescribes none, so this is "parity unpinned" by the paper.  It is fixed by
    the reading above and cross-checked by two independently written forms (the
    message-passing simulator `allreduce_steps` and the per-element nested fold
    `allreduce_fold`), a hand-worked cancellation example, and the all-dims-2
    case, which must equal a pairwise (binary tree) summation.
  * `multiring_time_model`, `choose_dims_bruteforce`: parity unpinned (the paper
    prints the formula for one ring only and says only that the dimensions are
    adjusted to the links; the multi-dimensional estimate and the exhaustive
    search over it are readings).  `ring_time_model` is the printed sum, pinned
    to its closed form and to the figures the paper states.
  * `allreduce_tensors` / `schedule_tensors` (several tensors per buffer): the
    definition is the single-tensor oracle applied tensor by tensor; the batched
    phase list is pinned to that definition and to integer sums.
  * `bf16_add`, `f32_to_bf16`, `bf16_to_f32`: pinned to torch's CPU bfloat16
    conversion and addition; fp16 uses numpy's own half arithmetic.
  * Two hand-worked fp32 examples (tests/golden): one ring of four (order inside
    a ring) and a 2 x 2 box (which learners share a ring of dimension 1).
"""
from __future__ import annotations

import itertools
from math import prod

import numpy as np


# --------------------------------------------------------------------------------------
# Box geometry (Sec. 4.3: the learners form a box of m dimensions, N = d_1 * ... * d_m)
# --------------------------------------------------------------------------------------
def coords(r: int, dims) -> tuple:
    """Box coordinates (c_1..c_m) of learner rank r; c_1 varies fastest.

    Reading: dimension 1 is the fastest link (the GPUs of one node, Sec. 4.3 and
    Sec. 5), so consecutive ranks are neighbours in dimension 1.
    """
    c = []
    for d in dims:
        c.append(r % d)
        r //= d
    return tuple(c)


def rank_of(c, dims) -> int:
    """Inverse of `coords`."""
    r = 0
    for ct, d in zip(reversed(c), reversed(dims)):
        r = r * d + ct
    return r


def neighbour(r: int, dims, t: int) -> int:
    """The learner one position further along the ring of dimension t (0-based)."""
    c = list(coords(r, dims))
    c[t] = (c[t] + 1) % dims[t]
    return rank_of(c, dims)


# --------------------------------------------------------------------------------------
# Chunking (Sec. 4.3: every transfer of a phase carries an N-th of the data; uneven sizes: a reading)
# --------------------------------------------------------------------------------------
def granule(dtype) -> int:
    """Elements per 16-byte granule; chunk boundaries fall on granule multiples."""
    return 16 // np.dtype(dtype).itemsize


def split(lo: int, hi: int, d: int, k: int, G: int) -> tuple:
    """Part k of d of the element range [lo, hi).

    The range is cut into ceil(n/G) granules of G elements (the last one possibly
    short); part k receives granules floor(k*ng/d) .. floor((k+1)*ng/d)-1.  Parts
    tile the range, differ by at most one granule, and may be empty.
    """
    n = hi - lo
    ng = -(-n // G)
    a = lo + min(n, (k * ng // d) * G)
    b = lo + min(n, ((k + 1) * ng // d) * G)
    return a, b


def level_segment(r: int, dims, t: int, count: int, G: int) -> tuple:
    """The range learner r still works on when dimension t (0-based) starts.

    Dimension 0 works on the whole buffer; after the reduce-scatter of dimension u
    a learner keeps only part c_u of what it had (Sec. 4.3: the box is processed
    one dimension after the other).
    """
    c = coords(r, dims)
    lo, hi = 0, count
    for u in range(t):
        lo, hi = split(lo, hi, dims[u], c[u], G)
    return lo, hi


def fine_chunks(dims, count: int, G: int) -> list:
    """All P finest chunks as (k, a, b): chunk index k = (k_1..k_m), range [a, b).

    The finest chunk k is what learner with coordinates k owns after the
    reduce-scatter has run through every dimension.
    """
    out = []
    for r in range(prod(dims)):
        a, b = level_segment(r, dims, len(dims), count, G)
        out.append((coords(r, dims), a, b))
    return out


# --------------------------------------------------------------------------------------
# The schedule (Sec. 4.3: N-1 phases per ring, N concurrent transfers per phase)
# --------------------------------------------------------------------------------------
def schedule(dims, count: int, G: int) -> list:
    """Every phase of the allreduce as (kind, t, ops), ops = [(src, dst, a, b)].

    Reduce-scatter, dimensions in order 1..m, d_t - 1 phases each: in phase s the
    learner at ring position c sends part (c - s - 1) mod d_t of its level
    segment to its +1 neighbour, which adds it to its own copy.  After the last
    phase position c holds the completed part c.
    All-gather, dimensions in order m..1, d_t - 1 phases each: in phase s position
    c forwards part (c - s) mod d_t, which the neighbour stores over its copy.
    """
    P = prod(dims)
    m = len(dims)
    steps = []
    for t in range(m):
        d = dims[t]
        for s in range(d - 1):
            ops = []
            for r in range(P):
                k = (coords(r, dims)[t] - s - 1) % d
                lo, hi = level_segment(r, dims, t, count, G)
                a, b = split(lo, hi, d, k, G)
                ops.append((r, neighbour(r, dims, t), a, b))
            steps.append(("RS", t, ops))
    for t in reversed(range(m)):
        d = dims[t]
        for s in range(d - 1):
            ops = []
            for r in range(P):
                k = (coords(r, dims)[t] - s) % d
                lo, hi = level_segment(r, dims, t, count, G)
                a, b = split(lo, hi, d, k, G)
                ops.append((r, neighbour(r, dims, t), a, b))
            steps.append(("AG", t, ops))
    return steps


def schedule_bytes(dims, count: int, itemsize: int) -> int:
    """Bytes the schedule itself moves through memory.

    A reduce phase reads the sent chunk, reads the receiver's copy and writes it
    back (3 accesses per element); a gather phase reads and writes (2).
    """
    total = 0
    for kind, _, ops in schedule(dims, count, 16 // itemsize):
        per_elem = 3 if kind == "RS" else 2
        total += sum(b - a for _, _, a, b in ops) * per_elem * itemsize
    return total


def _check_inputs(V, dims):
    P = prod(dims)
    if len(dims) < 1 or any(d < 1 for d in dims):
        raise ValueError("every dimension of the box must be >= 1")
    if len(V) != P:
        raise ValueError("number of learners must equal the product of the dimensions")
    count = len(V[0])
    if any(len(v) != count or v.dtype != V[0].dtype for v in V):
        raise ValueError("all learner buffers must have one length and dtype")
    return P, count


def _plain_add(x, y):
    return x + y


def _run(bufs, steps, add=None):
    add = add or _plain_add
    for kind, _, ops in steps:
        # A phase is N concurrent transfers: every message leaves its sender
        # before any message is applied at a receiver.
        messages = [bufs[src][a:b].copy() for src, _, a, b in ops]
        for (_, dst, a, b), msg in zip(ops, messages):
            if kind == "RS":
                bufs[dst][a:b] = add(bufs[dst][a:b], msg)  # one rounding per element
            else:
                bufs[dst][a:b] = msg
    return bufs


def allreduce_steps(V, dims, add=None) -> list:
    """Form (i): simulate every phase on in-memory copies of the P buffers.

    Returns the P buffers after reduce-scatter and all-gather (Sec. 4.1, 4.3);
    each must hold R = sum_j V_j.  `add(x, y)` replaces numpy's `+` for element
    types numpy cannot add itself (see `bf16_add`).
    """
    _, count = _check_inputs(V, dims)
    bufs = [np.array(v, copy=True) for v in V]
    return _run(bufs, schedule(dims, count, granule(bufs[0].dtype)), add)


def reduce_scatter_steps(V, dims, add=None) -> list:
    """Only the reduce-scatter half (Sec. 4.1 ReduceScatter): afterwards learner
    with coordinates k holds the completed finest chunk k; the rest of each buffer
    holds partial sums."""
    _, count = _check_inputs(V, dims)
    bufs = [np.array(v, copy=True) for v in V]
    steps = [s for s in schedule(dims, count, granule(bufs[0].dtype)) if s[0] == "RS"]
    return _run(bufs, steps, add)


def allgather_steps(V, dims) -> list:
    """Only the all-gather half (Sec. 4.1 AllGather): finest chunk k of learner k
    is copied into every learner."""
    _, count = _check_inputs(V, dims)
    bufs = [np.array(v, copy=True) for v in V]
    steps = [s for s in schedule(dims, count, granule(bufs[0].dtype)) if s[0] == "AG"]
    return _run(bufs, steps)


def allreduce_fold_range(get, dims, count: int, lo: int, hi: int, dtype, add=None) -> np.ndarray:
    """Form (ii): the result on elements [lo, hi) only, element by element, without
    simulating phases.  `get(r, a, b)` returns elements [a, b) of learner r's input.

    For an element of finest chunk k = (k_1..k_m), the ring of dimension t adds the
    d_t partial results in the order of ring positions k_t+1, k_t+2, ..., k_t+d_t
    (mod d_t), left to right: the partial sum starts at the position after the
    chunk's owner and travels once round the ring until it reaches the owner.
    Dimension 1 is folded first, then dimension 2 over those results, and so on.
    """
    add = add or _plain_add
    m = len(dims)
    out = np.empty(hi - lo, dtype=dtype)
    for k, ca, cb in fine_chunks(dims, count, granule(dtype)):
        a, b = max(ca, lo), min(cb, hi)
        if a >= b:
            continue
        # A maps the not-yet-folded coordinates (c_t..c_m) to a partial result
        A = {c: get(rank_of(c, dims), a, b) for c in itertools.product(*[range(d) for d in dims])}
        for t in range(m):
            d = dims[t]
            nxt = {}
            for rest in itertools.product(*[range(dd) for dd in dims[t + 1:]]):
                acc = A[((k[t] + 1) % d,) + rest]
                for i in range(2, d + 1):
                    acc = add(acc, A[((k[t] + i) % d,) + rest])
                nxt[rest] = acc
            A = nxt
        out[a - lo:b - lo] = A[()]
    return out


def allreduce_fold(V, dims, add=None) -> np.ndarray:
    """Form (ii) over whole in-memory buffers: the single vector every learner ends with."""
    _, count = _check_inputs(V, dims)
    return allreduce_fold_range(lambda r, a, b: V[r][a:b], dims, count, 0, count, V[0].dtype, add)


# --------------------------------------------------------------------------------------
# bfloat16, which numpy has no type for: stored as uint16 = the upper half of a float32
# --------------------------------------------------------------------------------------
def bf16_to_f32(x: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32: exact."""
    return (x.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16(f: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 bit pattern, ties to the even mantissa."""
    w = np.ascontiguousarray(f, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (w >> np.uint64(16)) & np.uint64(1)
    rounded = ((w + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)
    nan = (w & np.uint64(0x7FFFFFFF)) > np.uint64(0x7F800000)
    return np.where(nan, ((w >> np.uint64(16)) | np.uint64(0x40)).astype(np.uint16), rounded)


def bf16_add(x: np.ndarray, y: np.ndarray) -> np.ndarray:
    """x + y in bfloat16 (uint16 bit patterns): added in float32, rounded once to
    bfloat16.  float32 keeps 24 >= 2*8 + 2 significand bits, so the two roundings equal
    one correctly rounded bfloat16 addition."""
    return f32_to_bf16(bf16_to_f32(x) + bf16_to_f32(y))


# --------------------------------------------------------------------------------------
# Several tensors per learner, each reduced on its own (the gradients of a network are a
# list of per-layer tensors; Sec. 4.1: the library's objects are such tensors plus metadata)
# --------------------------------------------------------------------------------------
def schedule_tensors(dims, segments, G: int) -> list:
    """Phases when every tensor (off, n) of `segments` is chunked and reduced by itself but
    the transfers of one phase are issued together: ops of all tensors, tensor-major,
    with offsets relative to the whole buffer."""
    per_tensor = [schedule(dims, n, G) for _, n in segments]
    steps = []
    for i in range(2 * sum(d - 1 for d in dims)):
        kind, t = ("RS", 0), None
        ops = []
        for (off, _), sched in zip(segments, per_tensor):
            kind, t, tensor_ops = sched[i]
            ops += [(src, dst, off + a, off + b) for src, dst, a, b in tensor_ops]
        steps.append((kind, t, ops))
    return steps


def allreduce_tensors(V, dims, segments, add=None) -> list:
    """The plain definition of the per-tensor mode: run the single-tensor allreduce on
    every tensor's slice; elements outside all tensors are left alone."""
    _check_inputs(V, dims)
    out = [np.array(v, copy=True) for v in V]
    for off, n in segments:
        part = allreduce_steps([v[off:off + n] for v in V], dims, add)
        for o, p in zip(out, part):
            o[off:off + n] = p
    return out


def sum_fp64(V) -> np.ndarray:
    """Form (iii): R = sum_j V_j in double precision, learners in rank order."""
    acc = np.zeros(len(V[0]), dtype=np.float64)
    for v in V:
        acc = acc + v.astype(np.float64)
    return acc


# --------------------------------------------------------------------------------------
# Cost estimate (Sec. 4.3)
# --------------------------------------------------------------------------------------
def ring_time_model(S: float, N: int, B_min: float, L: float) -> float:
    """T ~ sum_{j=1}^{N-1} (S / (N * B_min) + L): one pass round a ring of N nodes
    over S bytes, slowest link B_min bytes/s, per-phase latency L seconds."""
    T = 0.0
    for _ in range(1, N):
        T += S / (N * B_min) + L
    return T


def multiring_time_model(S: float, dims, B, L) -> float:
    """Reduction plus distribution over the m-dimensional box (a reading).

    Dimension t runs a ring of d_t nodes over the S / (d_1 ... d_{t-1}) bytes that
    are left at that level, at that dimension's bandwidth B[t] and latency L[t];
    the ring formula is charged once for the reduction and once for the
    distribution, which carries the same traffic.
    """
    T = 0.0
    S_t = float(S)
    for d, Bt, Lt in zip(dims, B, L):
        T += 2.0 * ring_time_model(S_t, d, Bt, Lt)
        S_t /= d
    return T


def choose_dims_bruteforce(P: int, S: float, B, L, max_dim=None):
    """Every box (d_1..d_m), d_t >= 1, product P, within the caps, scored with
    `multiring_time_model`; returns (best time, list of all boxes within 1e-12 of it).

    Sec. 4.3 says only that the dimensions are adjusted to link bandwidths, topology and
    latency; exhaustive search over the estimate is this build's reading (parity unpinned).
    """
    m = len(B)

    def boxes(remaining, t):
        """All (d_t..d_m) with product `remaining`."""
        if t == m - 1:
            yield (remaining,)
            return
        for d in range(1, remaining + 1):
            if remaining % d == 0:
                for rest in boxes(remaining // d, t + 1):
                    yield (d,) + rest

    scored = []
    for dims in boxes(P, 0):
        if max_dim is not None and any(c and d > c for d, c in zip(dims, max_dim)):
            continue
        scored.append((multiring_time_model(S, dims, B, L), dims))
    if not scored:
        return None, []
    best = min(t for t, _ in scored)
    return best, [list(d) for t, d in scored if t <= best * (1 + 1e-12)]
