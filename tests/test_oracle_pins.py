"""Pins of the CPU oracle to things other than itself (no GPU, no HIP library).

Each pin is a plain function so that the mutation tests at the bottom can re-run
it against an oracle with a planted mistake and see it fail.
"""
import itertools
from math import prod

import numpy as np
import pytest

import oracle.ddl_oracle as O
from conftest import read_golden_kv, read_golden_ring_example


# ---------------------------------------------------------------------------------------
# helpers
# ---------------------------------------------------------------------------------------
def ordered_factorizations(P, allow_one=False):
    """All tuples of integers >= 2 (optionally >= 1, at most one 1) whose product is P."""
    if P == 1:
        return [(1,)]
    out = []

    def rec(rem, acc):
        if rem == 1:
            out.append(tuple(acc))
            return
        for d in range(2, rem + 1):
            if rem % d == 0:
                rec(rem // d, acc + [d])

    rec(P, [])
    if allow_one:
        out += [f[:i] + (1,) + f[i:] for f in list(out) for i in range(len(f) + 1)]
    return out


def int_inputs(rng, P, count, lo=-8, hi=8):
    return [rng.integers(lo, hi + 1, size=count).astype(np.float32) for _ in range(P)]


def wide_fp32_inputs(rng, P, count):
    """Random signs, mantissas and exponents spread over 1e-3 .. 1e3."""
    return [
        (rng.uniform(-1, 1, count) * 10.0 ** rng.uniform(-3, 3, count)).astype(np.float32)
        for _ in range(P)
    ]


COUNTS = [0, 1, 3, 4, 5, 15, 16, 17, 31, 63, 64, 65, 100, 255, 256, 257]


# ---------------------------------------------------------------------------------------
# T1: the plain definition R = sum_j V_j (Sec. 4.3), brute force in integers
# ---------------------------------------------------------------------------------------
def pin_bruteforce_integer_sum(Ps=range(1, 17), counts=COUNTS):
    rng = np.random.default_rng(1)
    for P in Ps:
        for dims in ordered_factorizations(P, allow_one=(P <= 6)):
            for count in counts:
                V = int_inputs(rng, P, count)
                want = np.zeros(count, dtype=np.int64)
                for v in V:
                    want += v.astype(np.int64)
                got = O.allreduce_steps(V, list(dims))
                assert len(got) == P
                for j in range(P):
                    assert got[j].dtype == np.float32
                    assert np.array_equal(got[j].astype(np.int64), want), (dims, count, j)
                assert np.array_equal(O.allreduce_fold(V, list(dims)).astype(np.int64), want), (dims, count)


def test_bruteforce_integer_sum():
    pin_bruteforce_integer_sum()


def test_inputs_are_not_modified():
    rng = np.random.default_rng(2)
    V = int_inputs(rng, 6, 50)
    keep = [v.copy() for v in V]
    O.allreduce_steps(V, [2, 3])
    O.allreduce_fold(V, [2, 3])
    assert all(np.array_equal(a, b) for a, b in zip(V, keep))


# ---------------------------------------------------------------------------------------
# T2 + T3: all learners identical; simulator == nested fold, bit for bit
# ---------------------------------------------------------------------------------------
DIMS_FP32 = [[1], [2], [3], [4], [5], [7], [2, 2], [2, 3], [3, 2], [4, 4], [3, 1, 2], [2, 2, 2],
             [4, 2, 2], [2, 3, 4], [1, 1], [4, 1], [1, 4], [16], [4, 2, 3]]


def pin_steps_equal_fold(dims_list=DIMS_FP32, counts=(0, 1, 7, 64, 257, 1000, 4099)):
    rng = np.random.default_rng(3)
    for dims in dims_list:
        for count in counts:
            V = wide_fp32_inputs(rng, prod(dims), count)
            got = O.allreduce_steps(V, dims)
            fold = O.allreduce_fold(V, dims)
            for j, g in enumerate(got):
                assert g.tobytes() == fold.tobytes(), (dims, count, j)


def test_steps_equal_fold_bitwise():
    pin_steps_equal_fold()


# ---------------------------------------------------------------------------------------
# T4: the hand-worked example
# ---------------------------------------------------------------------------------------
def pin_hand_worked_example():
    for name in ("ring4_cancellation.txt", "box2x2_dimension_order.txt"):
        ex = read_golden_ring_example(name)
        n = len(ex["expected"])
        V = [np.full(n, v, dtype=np.float32) for v in ex["inputs"]]
        want = np.array(ex["expected"], dtype=np.float32)
        for g in O.allreduce_steps(V, ex["dims"]):
            assert np.array_equal(g, want), (name, g)
        assert np.array_equal(O.allreduce_fold(V, ex["dims"]), want), name


def test_hand_worked_example():
    pin_hand_worked_example()


# ---------------------------------------------------------------------------------------
# T5: special cases that collapse to numpy routines / textbook forms
# ---------------------------------------------------------------------------------------
def pin_two_learners_is_numpy_add():
    rng = np.random.default_rng(5)
    V = wide_fp32_inputs(rng, 2, 1001)
    want = np.add(V[0], V[1])
    for dims in ([2], [2, 1], [1, 2], [1, 2, 1]):
        for g in O.allreduce_steps(V, dims):
            assert g.tobytes() == want.tobytes()
        assert O.allreduce_fold(V, dims).tobytes() == want.tobytes()


def pin_all_twos_is_pairwise_tree():
    """With every d_t = 2 each ring adds two operands, so the order inside a ring is
    immaterial (IEEE addition commutes) and the result must equal the binary-tree
    sum that pairs adjacent ranks first: dimension 1 = fastest-varying coordinate."""
    rng = np.random.default_rng(6)
    for m in (2, 3, 4):
        V = wide_fp32_inputs(rng, 2 ** m, 515)
        level = list(V)
        while len(level) > 1:
            level = [np.add(level[i], level[i + 1]) for i in range(0, len(level), 2)]
        for g in O.allreduce_steps(V, [2] * m):
            assert g.tobytes() == level[0].tobytes(), m
        assert O.allreduce_fold(V, [2] * m).tobytes() == level[0].tobytes()


def pin_unit_dims_are_transparent():
    rng = np.random.default_rng(7)
    V = wide_fp32_inputs(rng, 1, 77)
    for dims in ([1], [1, 1], [1, 1, 1]):
        assert O.allreduce_steps(V, dims)[0].tobytes() == V[0].tobytes()
    V = wide_fp32_inputs(rng, 5, 333)
    base = O.allreduce_steps(V, [5])[0]
    for dims in ([5, 1], [1, 5], [1, 5, 1]):
        assert O.allreduce_steps(V, dims)[0].tobytes() == base.tobytes()


def pin_constant_learners():
    # learner j filled with j+1 on a ring of 4 -> 10 everywhere
    V = [np.full(40, j + 1, dtype=np.float32) for j in range(4)]
    for g in O.allreduce_steps(V, [4]):
        assert np.array_equal(g, np.full(40, 10, dtype=np.float32))


def pin_two_level_ring_is_ring_of_rings():
    """dims = [a, b]: the result must equal summing each group of `a` consecutive
    ranks with a one-dimensional ring, then summing the b group results with a
    one-dimensional ring, PROVIDED both use the chunk the element falls in.  With
    one element per granule-sized buffer there is a single non-empty chunk, so the
    composition can be formed with the one-dimensional oracle alone."""
    rng = np.random.default_rng(8)
    a, b = 3, 4
    G = O.granule(np.float32)
    V = wide_fp32_inputs(rng, a * b, G)  # one granule: exactly one non-empty chunk per level
    got = O.allreduce_steps(V, [a, b])[0]
    # level 1: the single granule is part k1 where split is non-empty
    k1 = [k for k in range(a) if O.split(0, G, a, k, G)[1] > O.split(0, G, a, k, G)[0]]
    assert len(k1) == 1
    # one-dimensional ring over the a members of each group, as plain left folds
    groups = []
    for c2 in range(b):
        acc = V[(k1[0] + 1) % a + a * c2]
        for i in range(2, a + 1):
            acc = np.add(acc, V[(k1[0] + i) % a + a * c2])
        groups.append(acc)
    assert O.allreduce_steps(V[0:a], [a])[0].tobytes() == groups[0].tobytes()
    want = O.allreduce_steps(groups, [b])[0]
    assert got.tobytes() == want.tobytes()


def test_special_cases():
    pin_two_learners_is_numpy_add()
    pin_all_twos_is_pairwise_tree()
    pin_unit_dims_are_transparent()
    pin_constant_learners()
    pin_two_level_ring_is_ring_of_rings()


# ---------------------------------------------------------------------------------------
# T6: phase counts, transfers per phase, bytes (Sec. 4.3: N-1 phases, N transfers of 1/N)
# ---------------------------------------------------------------------------------------
def pin_schedule_counts():
    for dims in DIMS_FP32 + [[4, 8, 8], [4, 16]]:
        P = prod(dims)
        for count in (0, 5, 4 * P, 4 * P * 3, 1000):
            steps = O.schedule(dims, count, 4)
            assert len(steps) == 2 * sum(d - 1 for d in dims)
            kinds = [k for k, _, _ in steps]
            half = len(steps) // 2
            assert kinds == ["RS"] * half + ["AG"] * half
            # reduce visits the dimensions 1..m, gather m..1
            rs_dims = [t for k, t, _ in steps if k == "RS"]
            assert rs_dims == sorted(rs_dims)
            assert [t for k, t, _ in steps if k == "AG"] == rs_dims[::-1]
            for _, t, ops in steps:
                assert len(ops) == P
                assert sorted(src for src, _, _, _ in ops) == list(range(P))
                assert sorted(dst for _, dst, _, _ in ops) == list(range(P))
                for src, dst, a, b in ops:
                    cs, cd = O.coords(src, dims), O.coords(dst, dims)
                    assert all(cs[u] == cd[u] for u in range(len(dims)) if u != t)
                    assert cd[t] == (cs[t] + 1) % dims[t]
                    assert 0 <= a <= b <= count
            if count % (4 * P) == 0:
                # every transfer of a ring of d carries exactly 1/d of the level's data
                for _, t, ops in steps:
                    level = count // prod(dims[:t])
                    assert all(b - a == level // dims[t] for _, _, a, b in ops)
                assert O.schedule_bytes(dims, count, 4) == 20 * count * (P - 1)


def test_schedule_counts():
    pin_schedule_counts()


def test_flat_ring_needs_more_phases_than_box():
    # Sec. 4.3: the ring's latency term grows with N; the box replaces N-1 by sum(d_t-1)
    assert len(O.schedule([256], 1024, 4)) == 2 * 255
    assert len(O.schedule([4, 8, 8], 1024, 4)) == 2 * (3 + 7 + 7)


# ---------------------------------------------------------------------------------------
# T7: closeness to the fp64 sum, within the rounding-error bound of the schedule
# ---------------------------------------------------------------------------------------
def pin_fp64_closeness():
    rng = np.random.default_rng(9)
    u = 2.0 ** -24
    for dims in ([4, 4], [2, 3, 4], [16], [4, 8, 8]):
        P = prod(dims)
        count = 2048 + 3
        for V in (
            [rng.uniform(-1, 1, count).astype(np.float32) for _ in range(P)],
            [(rng.standard_normal(count) * 1e-2).astype(np.float32) for _ in range(P)],
        ):
            ref = O.sum_fp64(V)
            absum = np.zeros(count)
            for v in V:
                absum += np.abs(v.astype(np.float64))
            got = O.allreduce_steps(V, dims)[0].astype(np.float64)
            depth = sum(d - 1 for d in dims)  # additions any one element passes through
            bound = depth * u / (1 - depth * u) * absum
            assert np.all(np.abs(got - ref) <= bound)
            assert np.all(np.abs(got - ref) <= 1e-5 * absum)
            assert np.max(np.abs(got - ref)) <= 1e-5 * np.max(np.abs(ref))


def test_fp64_closeness():
    pin_fp64_closeness()


def test_sum_fp64_is_numpy_sum():
    rng = np.random.default_rng(10)
    V = [rng.integers(-1000, 1000, 99).astype(np.float32) for _ in range(7)]
    assert np.array_equal(O.sum_fp64(V), np.sum(np.stack(V).astype(np.float64), axis=0))


# ---------------------------------------------------------------------------------------
# T8: invariants of chunking and schedule
# ---------------------------------------------------------------------------------------
def test_split_hand_values():
    # 37 elements, granule 4 -> 10 granules over 4 parts: 2,3,2,3 granules, last one short
    assert [O.split(0, 37, 4, k, 4) for k in range(4)] == [(0, 8), (8, 20), (20, 28), (28, 37)]
    # ResNet-50-sized buffer: 25557032 = 4 * 6389258; cuts at floor(k*6389258/4)*4
    assert [O.split(0, 25557032, 4, k, 4) for k in range(4)] == [
        (0, 6389256), (6389256, 12778516), (12778516, 19167772), (19167772, 25557032)]
    # ResNet-101/22K-sized buffer: 87252369 -> 21813093 granules, last holds one element
    assert [O.split(0, 87252369, 4, k, 4) for k in range(4)] == [
        (0, 21813092), (21813092, 43626184), (43626184, 65439276), (65439276, 87252369)]
    # fewer granules than parts -> empty parts
    assert [O.split(0, 5, 4, k, 4) for k in range(4)] == [(0, 0), (0, 4), (4, 4), (4, 5)]
    assert [O.split(8, 8, 3, k, 4) for k in range(3)] == [(8, 8)] * 3


def pin_chunk_invariants():
    for G in (2, 4, 8):
        for dims in DIMS_FP32:
            P = prod(dims)
            for count in (0, 1, G, G + 1, 5 * G * P + 3, 1000):
                # I1: parts tile their segment, start on granule multiples, sizes within one granule
                for r in range(P):
                    for t in range(len(dims)):
                        lo, hi = O.level_segment(r, dims, t, count, G)
                        parts = [O.split(lo, hi, dims[t], k, G) for k in range(dims[t])]
                        assert parts[0][0] == lo and parts[-1][1] == hi
                        assert all(parts[i][1] == parts[i + 1][0] for i in range(len(parts) - 1))
                        assert all(a % G == 0 for a, b in parts if b > a)
                        full = [b - a for a, b in parts if b != count]
                        assert all(x % G == 0 for x in full)
                        sizes = [-(-(b - a) // G) for a, b in parts]
                        assert max(sizes) - min(sizes) <= 1
                # I4: the finest chunks tile the buffer, in rank order of their owners
                fc = O.fine_chunks(dims, count, G)
                assert len(fc) == P
                covered = np.zeros(count, dtype=np.int32)
                for k, a, b in fc:
                    covered[a:b] += 1
                assert np.all(covered == 1)
                # I5: a ring only links learners that work on the same segment
                for t in range(len(dims)):
                    for r in range(P):
                        assert O.level_segment(r, dims, t, count, G) == \
                            O.level_segment(O.neighbour(r, dims, t), dims, t, count, G)
                # I3: within one phase, what a learner sends is disjoint from what it receives
                for _, _, ops in O.schedule(dims, count, G):
                    recv = {dst: (a, b) for _, dst, a, b in ops}
                    for src, _, a, b in ops:
                        ra, rb = recv[src]
                        assert b <= ra or rb <= a or a == b or ra == rb


def test_chunk_invariants():
    pin_chunk_invariants()


def test_coords_roundtrip_and_order():
    dims = [4, 8, 8]
    assert O.coords(0, dims) == (0, 0, 0)
    assert O.coords(1, dims) == (1, 0, 0)        # dimension 1 varies fastest
    assert O.coords(4, dims) == (0, 1, 0)
    assert O.coords(32, dims) == (0, 0, 1)
    for r in range(256):
        assert O.rank_of(O.coords(r, dims), dims) == r
    assert O.neighbour(3, dims, 0) == 0 and O.neighbour(28, dims, 1) == 0 and O.neighbour(224, dims, 2) == 0


def test_reduce_scatter_then_allgather_is_allreduce():
    """Sec. 4.1 names ReduceScatter and AllGather as the two operations."""
    rng = np.random.default_rng(11)
    for dims in ([4], [2, 3], [4, 2, 2]):
        V = wide_fp32_inputs(rng, prod(dims), 301)
        rs = O.reduce_scatter_steps(V, dims)
        fold = O.allreduce_fold(V, dims)
        for k, a, b in O.fine_chunks(dims, 301, 4):
            assert rs[O.rank_of(k, dims)][a:b].tobytes() == fold[a:b].tobytes()
        ag = O.allgather_steps(rs, dims)
        for g in ag:
            assert g.tobytes() == fold.tobytes()


def test_rejects_bad_arguments():
    V = [np.zeros(4, np.float32)] * 4
    with pytest.raises(ValueError):
        O.allreduce_steps(V, [2, 3])
    with pytest.raises(ValueError):
        O.allreduce_steps(V, [4, 0])
    with pytest.raises(ValueError):
        O.allreduce_steps([np.zeros(4, np.float32), np.zeros(5, np.float32)], [2])


# ---------------------------------------------------------------------------------------
# Cost estimate (Sec. 4.3) against the paper's figures
# ---------------------------------------------------------------------------------------
def test_ring_time_model_closed_form_and_paper_figures():
    fig = read_golden_kv("paper_figures.txt")
    # the printed sum has N-1 identical terms
    for N, S, B, L in [(4, 1e8, 2e10, 0.0), (256, 3.5e8, 9.5e9, 1e-5), (2, 8.0, 1.0, 0.5), (1, 1e9, 1.0, 1.0)]:
        assert O.ring_time_model(S, N, B, L) == pytest.approx((N - 1) * (S / (N * B) + L), rel=1e-12)
    # strawman of Sec. 4.3: all learners' data into one server at the quoted rate
    assert fig["all_learners_bytes"] / fig["param_server_rate"] == pytest.approx(fig["param_server_time"])
    assert fig["learners"] * fig["resnet101_22k_bytes"] == pytest.approx(fig["all_learners_bytes"], rel=0.01)
    # reduction + distribution of 350 MB over 256 learners stays below the quoted 100 ms
    # both as a flat ring at the slowest link and as the 3-dimensional box at zero latency
    S, N = fig["resnet101_22k_bytes"], int(fig["learners"])
    flat = 2 * O.ring_time_model(S, N, fig["bw_dim3"], 0.0)
    box = O.multiring_time_model(S, [4, 8, 8], [fig["bw_dim1"], fig["bw_dim2"], fig["bw_dim3"]], [0.0] * 3)
    assert box < flat < fig["allreduce_time_max"]
    # with a per-phase latency the box wins by the phase count (Sec. 4.3: latency term ~ N)
    lat = 1e-4
    assert O.multiring_time_model(S, [4, 8, 8], [fig["bw_dim3"]] * 3, [lat] * 3) < \
        2 * O.ring_time_model(S, N, fig["bw_dim3"], lat) - 2 * (255 - 17) * lat * 0.99
    assert O.multiring_time_model(S, [N], [fig["bw_dim3"]], [lat]) == \
        pytest.approx(2 * O.ring_time_model(S, N, fig["bw_dim3"], lat))


# ---------------------------------------------------------------------------------------
# Mutation tests: a planted mistake in the oracle must trip at least one pin
# ---------------------------------------------------------------------------------------
def _expect_some_pin_fails(pins):
    failed = 0
    for pin in pins:
        try:
            pin()
        except (AssertionError, IndexError, KeyError, ValueError):
            failed += 1
    assert failed >= 1, "planted mistake went unnoticed"


SMALL = dict(Ps=(4, 6, 8), counts=(16, 65))


def test_mutation_transposed_coordinates(monkeypatch):
    def coords_slowest_first(r, dims):
        c = []
        for d in reversed(dims):
            c.append(r % d)
            r //= d
        return tuple(reversed(c))

    def rank_slowest_first(c, dims):
        r = 0
        for ct, d in zip(c, dims):
            r = r * d + ct
        return r

    monkeypatch.setattr(O, "coords", coords_slowest_first)
    monkeypatch.setattr(O, "rank_of", rank_slowest_first)
    # still a valid allreduce (so brute force passes) but pairs the wrong ranks first
    pin_bruteforce_integer_sum(**SMALL)
    with pytest.raises(AssertionError):
        pin_all_twos_is_pairwise_tree()
    with pytest.raises(AssertionError):
        pin_hand_worked_example()


def test_mutation_wrong_direction_only_in_neighbour(monkeypatch):
    def backwards(r, dims, t):
        c = list(O.coords(r, dims))
        c[t] = (c[t] - 1) % dims[t]
        return O.rank_of(c, dims)

    monkeypatch.setattr(O, "neighbour", backwards)
    with pytest.raises(AssertionError):
        pin_bruteforce_integer_sum(**SMALL)


def test_mutation_mirrored_ring_is_caught_by_hand_example(monkeypatch):
    """A ring run consistently the other way round is still an allreduce; only the
    hand-worked example tells it from this build's reading."""
    real_schedule = O.schedule

    def mirrored(dims, count, G):
        flipped = []
        for kind, t, ops in real_schedule(dims, count, G):
            d = dims[t]
            new_ops = []
            for src, dst, a, b in ops:
                # reflect ring positions: c -> (d - c) % d, which reverses the direction
                cs = list(O.coords(src, dims)); cs[t] = (d - cs[t]) % d
                cd = list(O.coords(dst, dims)); cd[t] = (d - cd[t]) % d
                new_ops.append((O.rank_of(cs, dims), O.rank_of(cd, dims), a, b))
            flipped.append((kind, t, new_ops))
        return flipped

    monkeypatch.setattr(O, "schedule", mirrored)
    # 1-D only: reflection keeps the level segments consistent there
    rng = np.random.default_rng(12)
    V = int_inputs(rng, 4, 64)
    want = sum(v.astype(np.int64) for v in V)
    assert np.array_equal(O.allreduce_steps(V, [4])[0].astype(np.int64), want)
    ex = read_golden_ring_example("ring4_cancellation.txt")
    Vc = [np.full(16, v, dtype=np.float32) for v in ex["inputs"]]
    assert not np.array_equal(O.allreduce_steps(Vc, [4])[0], np.array(ex["expected"], dtype=np.float32))


def test_mutation_dropped_phase(monkeypatch):
    real_schedule = O.schedule

    def one_short(dims, count, G):
        steps = real_schedule(dims, count, G)
        return steps[:-1]

    monkeypatch.setattr(O, "schedule", one_short)
    with pytest.raises(AssertionError):
        pin_bruteforce_integer_sum(**SMALL)


def test_mutation_copy_instead_of_add(monkeypatch):
    def run_copy_only(bufs, steps, add=None):
        for _, _, ops in steps:
            msgs = [bufs[src][a:b].copy() for src, _, a, b in ops]
            for (_, dst, a, b), msg in zip(ops, msgs):
                bufs[dst][a:b] = msg
        return bufs

    monkeypatch.setattr(O, "_run", run_copy_only)
    with pytest.raises(AssertionError):
        pin_bruteforce_integer_sum(**SMALL)


def test_mutation_split_off_by_one_granule(monkeypatch):
    def bad_split(lo, hi, d, k, G):
        n = hi - lo
        ng = n // G  # drops the short last granule
        return lo + min(n, (k * ng // d) * G), lo + min(n, ((k + 1) * ng // d) * G)

    monkeypatch.setattr(O, "split", bad_split)
    _expect_some_pin_fails([lambda: pin_bruteforce_integer_sum(**SMALL), pin_chunk_invariants])
    with pytest.raises(AssertionError):
        pin_bruteforce_integer_sum(Ps=(4,), counts=(17,))


def test_mutation_fold_wrong_start(monkeypatch):
    """The nested fold starting at the owner instead of the position after it."""
    def fold_from_owner(V, dims):
        count = len(V[0])
        out = np.empty(count, dtype=V[0].dtype)
        for k, a, b in O.fine_chunks(dims, count, O.granule(V[0].dtype)):
            A = {c: V[O.rank_of(c, dims)][a:b] for c in itertools.product(*[range(d) for d in dims])}
            for t in range(len(dims)):
                d = dims[t]
                nxt = {}
                for rest in itertools.product(*[range(dd) for dd in dims[t + 1:]]):
                    acc = A[(k[t] % d,) + rest]
                    for i in range(1, d):
                        acc = acc + A[((k[t] + i) % d,) + rest]
                    nxt[rest] = acc
                A = nxt
            out[a:b] = A[()]
        return out

    monkeypatch.setattr(O, "allreduce_fold", fold_from_owner)  # replaces the whole-buffer entry
    with pytest.raises(AssertionError):
        pin_steps_equal_fold(dims_list=[[4], [3, 2]], counts=(257,))


def test_fold_range_equals_whole_fold():
    rng = np.random.default_rng(13)
    dims, count = [3, 2, 2], 1003
    V = wide_fp32_inputs(rng, 12, count)
    whole = O.allreduce_fold(V, dims)
    for lo, hi in [(0, 0), (0, 1), (5, 900), (998, 1003), (83, 84), (0, 1003)]:
        part = O.allreduce_fold_range(lambda r, a, b: V[r][a:b], dims, count, lo, hi, np.float32)
        assert part.tobytes() == whole[lo:hi].tobytes()


def test_choose_dims_bruteforce_special_cases():
    S = 349e6
    # no latency, one bandwidth: every box moves the same bytes -> all tie at 2 S (1 - 1/P) / B
    t, boxes = O.choose_dims_bruteforce(64, S, [1e10] * 3, [0.0] * 3)
    assert t == pytest.approx(2 * S * (1 - 1 / 64) / 1e10, rel=1e-12)
    assert [4, 4, 4] in boxes and [64, 1, 1] in boxes and [1, 8, 8] in boxes and len(boxes) == 28
    # one level: only the flat ring
    assert O.choose_dims_bruteforce(12, S, [1e10], [1e-5])[1] == [[12]]
    # latency dominates: the box with the fewest phases, sum(d_t - 1) minimal
    t, boxes = O.choose_dims_bruteforce(256, 1.0, [1e10] * 3, [1.0] * 3)
    assert sorted(boxes) == [[4, 8, 8], [8, 4, 8], [8, 8, 4]]
    assert t == pytest.approx(2 * 17 * 1.0, rel=1e-6)
    assert O.choose_dims_bruteforce(256, 1.0, [1e10] * 8, [1.0] * 8)[1] == [[2] * 8]
    # bandwidth only, faster first level: everything rides the fastest links (Sec. 4.3)
    fig = read_golden_kv("paper_figures.txt")
    bw = [fig["bw_dim1"], fig["bw_dim2"], fig["bw_dim3"]]
    assert O.choose_dims_bruteforce(256, S, bw, [0.0] * 3)[1] == [[256, 1, 1]]
    # the paper's cluster: 4 GPUs per node, 16 nodes per rack, 4 racks leave one box
    assert O.choose_dims_bruteforce(256, S, bw, [0.0] * 3, [4, 16, 4])[1] == [[4, 16, 4]]
    assert O.choose_dims_bruteforce(256, S, bw, [0.0] * 3, [4, 4, 4]) == (None, [])


# ---------------------------------------------------------------------------------------
# 16-bit element types
# ---------------------------------------------------------------------------------------
def test_bf16_helpers_against_torch_cpu():
    import torch
    rng = np.random.default_rng(14)
    f = np.concatenate([
        (rng.uniform(-1, 1, 20000) * 10.0 ** rng.uniform(-30, 30, 20000)).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, np.inf, -np.inf], np.float32),
    ])
    bits = O.f32_to_bf16(f)
    want = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    back = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    assert O.bf16_to_f32(bits).tobytes() == back.tobytes()
    x, y = bits[:10000], bits[10000:20000]
    tsum = (torch.from_numpy(x.view(np.int16)).view(torch.bfloat16) +
            torch.from_numpy(y.view(np.int16)).view(torch.bfloat16)).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(O.bf16_add(x, y), tsum)
    # ties go to the even mantissa: 1 + 2^-8 lies between 1 and 1 + 2^-7
    assert O.f32_to_bf16(np.array([1.00390625], np.float32))[0] == 0x3F80
    assert O.f32_to_bf16(np.array([1.01171875], np.float32))[0] == 0x3F82
    assert np.isnan(O.bf16_to_f32(O.f32_to_bf16(np.array([np.nan], np.float32))))[0]


def test_sixteen_bit_types_bruteforce_and_forms_agree():
    rng = np.random.default_rng(15)
    for dims in ([4], [2, 3], [4, 2, 2]):
        P = prod(dims)
        for count in (0, 7, 8, 9, 100, 1001):
            # small integers are exact in both 16-bit types -> plain integer sum
            ints = [rng.integers(-8, 9, count) for _ in range(P)]
            want = sum(ints) if count else np.zeros(0)
            h = O.allreduce_steps([v.astype(np.float16) for v in ints], dims)
            b = O.allreduce_steps([O.f32_to_bf16(v.astype(np.float32)) for v in ints], dims, add=O.bf16_add)
            for j in range(P):
                assert np.array_equal(h[j].astype(np.int64), want)
                assert np.array_equal(O.bf16_to_f32(b[j]).astype(np.int64), want)
            # general values: simulator == fold, in each type's own arithmetic
            V = wide_fp32_inputs(rng, P, count)
            Vh = [v.astype(np.float16) for v in V]
            Vb = [O.f32_to_bf16(v) for v in V]
            for g in O.allreduce_steps(Vh, dims):
                assert g.tobytes() == O.allreduce_fold(Vh, dims).tobytes()
            for g in O.allreduce_steps(Vb, dims, add=O.bf16_add):
                assert g.tobytes() == O.allreduce_fold(Vb, dims, add=O.bf16_add).tobytes()
    # chunks are cut on 16-byte granules = 8 elements
    assert O.granule(np.float16) == 8 and O.granule(np.uint16) == 8


# ---------------------------------------------------------------------------------------
# per-tensor mode
# ---------------------------------------------------------------------------------------
def test_per_tensor_mode_definition_and_batched_schedule_agree():
    rng = np.random.default_rng(16)
    segments = [(0, 64), (64, 4), (68, 0), (72, 1000), (1072, 8), (1100, 37)]  # gaps allowed
    count = 1140
    for dims in ([4], [2, 3], [4, 2, 2]):
        P = prod(dims)
        # integers: every tensor ends as the plain sum, the gaps are untouched
        Vi = int_inputs(rng, P, count)
        got = O.allreduce_tensors(Vi, dims, segments)
        total = sum(v.astype(np.int64) for v in Vi)
        covered = np.zeros(count, bool)
        for off, n in segments:
            covered[off:off + n] = True
        for j in range(P):
            assert np.array_equal(got[j][covered].astype(np.int64), total[covered])
            assert np.array_equal(got[j][~covered], Vi[j][~covered])
        # running the batched phase list gives the same bits as tensor-by-tensor
        V = wide_fp32_inputs(rng, P, count)
        want = O.allreduce_tensors(V, dims, segments)
        bufs = O._run([v.copy() for v in V], O.schedule_tensors(dims, segments, 4))
        for j in range(P):
            assert bufs[j].tobytes() == want[j].tobytes()
        # one tensor covering everything is the ordinary allreduce
        one = O.allreduce_tensors(V, dims, [(0, count)])
        for a, b in zip(one, O.allreduce_steps(V, dims)):
            assert a.tobytes() == b.tobytes()
        # phases: same count, P transfers per tensor and phase
        steps = O.schedule_tensors(dims, segments, 4)
        assert len(steps) == 2 * sum(d - 1 for d in dims)
        assert all(len(ops) == P * len(segments) for _, _, ops in steps)
