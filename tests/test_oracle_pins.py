"""Pins for the CPU oracle: nothing here retypes the oracle's numpy formulas.

Each oracle function is checked against something fixed by the paper or by
mathematics: pure-Python brute force on tiny inputs (sorted(), dict, Fraction),
closed forms, invariants, special cases that reduce to a library routine, and
the numbers the paper prints in its Introduction.
"""
import math
import os
import struct
from fractions import Fraction

import numpy as np
import pytest

from oracle import okt_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f32(x: float) -> float:
    """Round a Python float (double) to the nearest fp32, ties to even."""
    return struct.unpack("f", struct.pack("f", x))[0]


def bits(x) -> int:
    return struct.unpack("I", struct.pack("f", float(x)))[0]


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            key, value = line.split()
            out[key] = value
    return out


def rand_f32(rng, size, scale=1e-3):
    return (rng.laplace(0, scale, size)).astype(np.float32)


# ------------------------------------------------------------------ accumulate
def test_accumulate_matches_double_then_round():
    # fp32 a*b is exact in double (48-bit product); double rounding of an fp32
    # sum through double is innocuous (53 >= 2*24+2), so Python floats give the
    # correctly rounded two-step fp32 result without using numpy arithmetic.
    rng = np.random.default_rng(11)
    g = rand_f32(rng, 500)
    e = rand_f32(rng, 500, 3e-3)
    for lr in (1.0, 0.1, 0.0, 3.7e-4, -2.5):
        lr32 = f32(lr)
        got = orc.residual_accumulate(g, e, lr)
        for i in range(g.size):
            want = f32(float(e[i]) + f32(lr32 * float(g[i])))
            assert bits(got[i]) == bits(want), (lr, i)


def test_accumulate_special_cases():
    rng = np.random.default_rng(12)
    g = rand_f32(rng, 1000)
    e = rand_f32(rng, 1000)
    zero = np.zeros_like(g)
    # eps_0 = 0 and lr = 1 (Algorithm 2, line 2): acc is the gradient, bit for bit
    nz = g != 0
    assert np.array_equal(orc.residual_accumulate(g, zero, 1.0).view(np.uint32)[nz],
                          g.view(np.uint32)[nz])
    # lr = 0: acc is the residual
    assert np.array_equal(orc.residual_accumulate(g, e, 0.0), e)
    # linear in lr for exactly representable data
    gi = np.arange(-50, 50, dtype=np.float32)
    ei = np.arange(100, dtype=np.float32) * 0.25
    assert np.array_equal(orc.residual_accumulate(gi, ei, 0.5), ei + gi / 2)


def test_accumulate_is_not_fused():
    # lr*g = 1 + 2^-11 + 2^-24 exactly: the product rounds (tie to even) to
    # 1 + 2^-11, so the two-rounding result is 0; a fused multiply-add would
    # leave 2^-24.
    lr = 1.0 + 2.0 ** -12
    g = np.array([1.0 + 2.0 ** -12], dtype=np.float32)
    e = np.array([-(1.0 + 2.0 ** -11)], dtype=np.float32)
    exact = Fraction(lr) * Fraction(float(g[0])) + Fraction(float(e[0]))
    assert exact == Fraction(1, 2 ** 24)
    assert orc.residual_accumulate(g, e, lr)[0] == 0.0


# ------------------------------------------------------------------- threshold
def brute_threshold(values, k):
    mags = sorted((abs(float(v)) for v in values), reverse=True)
    th = mags[k - 1]
    return th, sum(1 for m in mags if m >= th)


@pytest.mark.parametrize("n,k", [(1, 1), (7, 3), (64, 1), (64, 64), (1000, 10), (4096, 41)])
def test_threshold_vs_python_sort(n, k):
    rng = np.random.default_rng(100 + n + k)
    acc = rand_f32(rng, n)
    th, cnt = orc.topk_threshold_exact(acc, k)
    bth, bcnt = brute_threshold(acc, k)
    assert th >= 0 and bits(th) == bits(bth)
    assert cnt == bcnt
    th2, cnt2 = orc.topk_threshold_exact(acc, k, method="partition")
    assert bits(th2) == bits(th) and cnt2 == cnt


def test_threshold_special_cases():
    rng = np.random.default_rng(5)
    acc = rand_f32(rng, 2000)
    assert orc.topk_threshold_exact(acc, 1)[0] == np.abs(acc).max()
    th, cnt = orc.topk_threshold_exact(acc, acc.size)
    assert th == np.abs(acc).min() and cnt == acc.size
    same = np.full(100, -0.125, dtype=np.float32)
    th, cnt = orc.topk_threshold_exact(same, 17)
    assert th == 0.125 and cnt == 100
    # the sign never matters
    th_a, cnt_a = orc.topk_threshold_exact(np.abs(acc), 20)
    th_b, cnt_b = orc.topk_threshold_exact(-np.abs(acc), 20)
    assert (th_a, cnt_a) == (th_b, cnt_b) == orc.topk_threshold_exact(acc, 20)


def test_threshold_ties_straddling_rank_k():
    # 5 values above, then 4 copies of the tied value, then smaller ones; any k
    # in 6..9 must return the tied value and count all its copies.
    acc = np.array([9, -8, 7, -6, 5, 3, -3, 3, -3, 2, 1, 0, -0.5], dtype=np.float32)
    for k in range(6, 10):
        th, cnt = orc.topk_threshold_exact(acc, k)
        assert th == 3.0 and cnt == 9
    assert orc.topk_threshold_exact(acc, 5) == (5.0, 5)
    assert orc.topk_threshold_exact(acc, 10) == (2.0, 10)


def test_threshold_matches_torch_topk():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(77)
    acc = rand_f32(rng, 50_000)
    k = 500
    th, cnt = orc.topk_threshold_exact(acc, k)
    want = torch.topk(torch.from_numpy(acc).abs(), k).values[-1].item()
    assert bits(th) == bits(want)
    # two-sided invariant: fewer than k strictly above, at least k at or above
    mags = np.abs(acc)
    assert (mags > th).sum() < k <= (mags >= th).sum() == cnt


def test_threshold_key_order_subnormal_zero_inf():
    acc = np.array([0.0, -0.0, 1e-45, -1e-40, 1.0, np.inf, -3.0], dtype=np.float32)
    order = [np.inf, 3.0, 1.0, 1e-40, 1e-45, 0.0, 0.0]
    for k, want in enumerate(order, start=1):
        th, _ = orc.topk_threshold_exact(acc, k)
        assert bits(th) == bits(np.float32(want))


def test_k_from_density_paper_numbers():
    gold = read_golden("intro_fillin.txt")
    assert orc.k_from_density(int(gold["n"]), int(gold["density_num"]),
                              int(gold["density_den"])) == int(gold["k"])
    assert orc.k_from_density(1_048_576, 1, 100) == 10_486      # ceil, not floor
    assert orc.k_from_density(336_000_000, 1, 1000) == 336_000


# ---------------------------------------------------------------------- select
@pytest.mark.parametrize("n,k", [(1, 1), (33, 5), (1000, 10), (5000, 50)])
def test_select_vs_python_filter(n, k):
    rng = np.random.default_rng(300 + n)
    acc = rand_f32(rng, n)
    th, cnt = brute_threshold(acc, k)
    idx, val, res, total = orc.threshold_select(acc, np.float32(th))
    want = [i for i in range(n) if abs(float(acc[i])) >= th]
    assert idx.dtype == np.uint32 and list(idx) == want
    assert total == cnt == len(want) >= k
    assert [bits(v) for v in val] == [bits(acc[i]) for i in want]
    chosen = set(want)
    for i in range(n):
        assert bits(res[i]) == (0 if i in chosen else bits(acc[i]))


def test_select_exactly_k_when_values_distinct():
    rng = np.random.default_rng(31)
    acc = rng.permutation(np.arange(1, 2001)).astype(np.float32) * np.float32(1e-3)
    acc[::2] *= -1
    for k in (1, 20, 1999, 2000):
        th, cnt = orc.topk_threshold_exact(acc, k)
        idx, val, res, total = orc.threshold_select(acc, th)
        assert cnt == total == idx.size == k
        # the selected set is the brute-force top-k set
        want = sorted(sorted(range(acc.size), key=lambda i: -abs(float(acc[i])))[:k])
        assert list(idx) == want


def test_select_residual_plus_selected_is_acc():
    rng = np.random.default_rng(32)
    acc = rand_f32(rng, 20_000)
    th, _ = orc.topk_threshold_exact(acc, 200)
    idx, val, res, _ = orc.threshold_select(acc, th)
    assert np.all(np.diff(idx.astype(np.int64)) > 0)
    back = res.copy()
    assert np.all(back[idx] == 0) and not np.signbit(back[idx]).any()
    back[idx] = val
    assert np.array_equal(back.view(np.uint32), acc.view(np.uint32))


def test_select_degenerate_thresholds_and_capacity():
    rng = np.random.default_rng(33)
    acc = rand_f32(rng, 3000)
    idx, val, res, total = orc.threshold_select(acc, np.float32(np.inf))
    assert total == 0 and idx.size == 0 and np.array_equal(res.view(np.uint32), acc.view(np.uint32))
    idx, val, res, total = orc.threshold_select(acc, np.float32(0.0))
    assert total == acc.size and np.array_equal(idx, np.arange(acc.size))
    assert not res.any() and np.array_equal(val.view(np.uint32), acc.view(np.uint32))
    # a negative threshold means its magnitude
    a = orc.threshold_select(acc, np.float32(-1e-3))
    b = orc.threshold_select(acc, np.float32(1e-3))
    assert np.array_equal(a[0], b[0]) and a[3] == b[3]
    # truncation: first `capacity` members in index order, the rest stay behind
    full_idx, _, _, total = b
    assert total > 10
    idx, val, res, total_c = orc.threshold_select(acc, np.float32(1e-3), capacity=10)
    assert total_c == total and list(idx) == list(full_idx[:10])
    assert np.all(res[full_idx[:10]] == 0)
    assert np.array_equal(res[full_idx[10:]], acc[full_idx[10:]])


# ------------------------------------------------------------------- partition
def test_partition_counts_balanced():
    rng = np.random.default_rng(41)
    n = 100_000
    for nnz, R in [(1000, 4), (1001, 16), (999, 64), (5, 8), (64, 64), (1, 1), (7, 1)]:
        idx = np.sort(rng.choice(n, nnz, replace=False)).astype(np.uint32)
        b, off = orc.region_partition(idx, n, R)
        assert b.dtype == np.uint32 and b[0] == 0 and b[R] == n
        assert np.all(np.diff(b.astype(np.int64)) >= 0)
        assert off[0] == 0 and off[R] == nnz
        counts = np.diff(off.astype(np.int64))
        assert set(counts) <= {nnz // R, -(-nnz // R)}
        # off is consistent with b: region r holds exactly the entries in [b[r], b[r+1])
        for r in range(R):
            inside = [int(i) for i in idx if b[r] <= i < b[r + 1]]
            assert inside == [int(i) for i in idx[int(off[r]):int(off[r + 1])]]


def test_partition_worked_by_hand():
    # the reading written out on lists short enough to do by hand: boundary r is
    # the entry at list position floor(r * nnz / R); region r takes the entries
    # from there up to the next boundary
    idx = np.array([10, 20, 30, 40, 50], dtype=np.uint32)             # nnz = 5
    b, off = orc.region_partition(idx, 100, 2)                         # floor(5/2) = 2 -> idx[2]
    assert b.tolist() == [0, 30, 100] and off.tolist() == [0, 2, 5]
    b, off = orc.region_partition(idx, 100, 3)                         # floor(5/3) = 1, floor(10/3) = 3
    assert b.tolist() == [0, 20, 40, 100] and off.tolist() == [0, 1, 3, 5]
    b, off = orc.region_partition(idx, 100, 4)                         # positions 1, 2, 3
    assert b.tolist() == [0, 20, 30, 40, 100] and off.tolist() == [0, 1, 2, 3, 5]
    idx = np.array([7, 8], dtype=np.uint32)                            # fewer entries than regions
    b, off = orc.region_partition(idx, 64, 4)                          # positions 0, 1, 1
    assert b.tolist() == [0, 7, 8, 8, 64] and off.tolist() == [0, 0, 1, 1, 2]


def test_partition_extreme_case_from_the_paper():
    gold = read_golden("split_extreme.txt")
    P, k, n = 8, 4000, 1 << 20
    # all local top-k entries inside the first naive region [0, n/P)
    rng = np.random.default_rng(42)
    idx = np.sort(rng.choice(n // P, k, replace=False)).astype(np.uint32)
    naive_b = [(r * n) // P for r in range(P + 1)]
    naive_counts = [int(((idx >= naive_b[r]) & (idx < naive_b[r + 1])).sum()) for r in range(P)]
    # P-1 peers each send all their k (index, value) pairs to worker 0
    env = {"P": P, "k": k}
    assert 2 * (P - 1) * naive_counts[0] == eval(gold["naive_received_by_worker0_elements"], env)
    assert sum(naive_counts[1:]) == eval(gold["naive_received_by_other_workers_elements"], env)
    b, off = orc.region_partition(idx, n, P)
    counts = np.diff(off.astype(np.int64))
    assert np.all(2 * counts == eval(gold["balanced_received_from_each_peer_elements"], env))


def test_partition_without_entries_is_the_equal_split():
    b, off = orc.region_partition(np.zeros(0, np.uint32), 1000, 8)
    assert list(b) == [0, 125, 250, 375, 500, 625, 750, 875, 1000]
    assert not off.any()
    b, off = orc.region_partition(np.zeros(0, np.uint32), 10, 4)
    assert list(b) == [0, 2, 5, 7, 10]


# ---------------------------------------------------------------------- reduce
def dict_reduce(chunks, lo, hi):
    acc = {}
    for idx, val in chunks:
        for i, v in zip(idx, val):
            if lo <= int(i) < hi:
                acc[int(i)] = acc.get(int(i), Fraction(0)) + Fraction(float(v))
    return dict(sorted(acc.items()))


def cat(chunks):
    off = np.zeros(len(chunks) + 1, dtype=np.uint64)
    off[1:] = np.cumsum([len(c[0]) for c in chunks])
    return (np.concatenate([c[0] for c in chunks]).astype(np.uint32),
            np.concatenate([c[1] for c in chunks]).astype(np.float32), off)


def make_chunks(rng, P, m, n, dyadic=True):
    chunks = []
    for _ in range(P):
        idx = np.sort(rng.choice(n, m, replace=False)).astype(np.uint32)
        if dyadic:       # multiples of 2^-8, |v| < 64: every partial sum is exact
            val = (rng.integers(-16000, 16000, m) / 256.0).astype(np.float32)
        else:
            val = rand_f32(rng, m)
        chunks.append((idx, val))
    return chunks


@pytest.mark.parametrize("P,m,n,lo,hi", [(1, 50, 400, 0, 400), (4, 60, 300, 0, 300),
                                         (4, 60, 300, 75, 150), (16, 40, 200, 10, 190),
                                         (70, 30, 64, 0, 64)])
def test_reduce_vs_dict_exact_values(P, m, n, lo, hi):
    rng = np.random.default_rng(500 + P)
    chunks = make_chunks(rng, P, m, n)
    out = orc.sparse_reduce(*cat(chunks), lo, hi)
    want = dict_reduce(chunks, lo, hi)
    assert list(out["idx"]) == list(want.keys())
    assert [Fraction(float(v)) for v in out["val"]] == list(want.values())
    dense = np.zeros(hi - lo, dtype=np.float32)
    for i, v in want.items():
        dense[i - lo] = float(v)
    assert np.array_equal(out["dense"], dense)
    hits = {}
    for idx, _ in chunks:
        for i in idx:
            if lo <= i < hi:
                hits[int(i)] = hits.get(int(i), 0) + 1
    assert list(out["hits"]) == [hits[i] for i in want]


def test_reduce_rounding_of_general_values():
    # general fp32 values: the exact rational sum rounded once to fp32 may differ
    # from a float64 running sum by at most a few double ulps before rounding
    rng = np.random.default_rng(51)
    chunks = make_chunks(rng, 32, 200, 500, dyadic=False)
    out = orc.sparse_reduce(*cat(chunks), 0, 500)
    want = dict_reduce(chunks, 0, 500)
    for i, v, a in zip(out["idx"], out["val"], out["abs_sum"]):
        exact = want[int(i)]
        assert abs(Fraction(float(v)) - exact) <= Fraction(float(a)) * Fraction(2, 2 ** 24)
    # abs_sum is the sum of magnitudes
    mags = {}
    for idx, val in chunks:
        for i, v in zip(idx, val):
            mags[int(i)] = mags.get(int(i), 0.0) + abs(float(v))
    assert np.allclose(out["abs_sum"], [mags[int(i)] for i in out["idx"]], rtol=1e-12)


def test_reduce_special_cases():
    rng = np.random.default_rng(52)
    n = 1000
    (idx, val), = make_chunks(rng, 1, 100, n, dyadic=False)
    # P = 1: the output is the input slice, bit for bit
    out = orc.sparse_reduce(idx, val, np.array([0, 100], np.uint64), 200, 700)
    inside = (idx >= 200) & (idx < 700)
    assert np.array_equal(out["idx"], idx[inside])
    assert np.array_equal(out["val"].view(np.uint32), val[inside].view(np.uint32))
    # identical index sets: U = len, values add
    out = orc.sparse_reduce(*cat([(idx, val), (idx, val), (idx, val)]), 0, n)
    assert np.array_equal(out["idx"], idx)
    assert np.array_equal(out["val"], (3.0 * val.astype(np.float64)).astype(np.float32))
    # a chunk and its negation: structural zeros are kept
    out = orc.sparse_reduce(*cat([(idx, val), (idx, -val)]), 0, n)
    assert np.array_equal(out["idx"], idx) and not out["val"].any()
    # no 1/P inside the reduction (the average belongs to the model update)
    out = orc.sparse_reduce(*cat([(idx, np.ones(100, np.float32))] * 4), 0, n)
    assert np.all(out["val"] == 4.0)
    # empty region / no entries inside
    out = orc.sparse_reduce(idx, val, np.array([0, 100], np.uint64), n, n + 10)
    assert out["idx"].size == 0 and out["dense"].size == 10 and not out["dense"].any()


def test_reduce_fill_in_numbers_from_the_introduction():
    gold = read_golden("intro_fillin.txt")
    n, k = int(gold["n"]), int(gold["k"])
    rng = np.random.default_rng(53)
    perm = rng.permutation(n)

    def union_of(nchunks):
        chunks = []
        for p in range(nchunks):   # non-overlapping indexes, k per contribution
            idx = np.sort(perm[p * k:(p + 1) * k]).astype(np.uint32)
            chunks.append((idx, np.ones(k, np.float32)))
        out = orc.sparse_reduce(*cat(chunks), 0, n)
        assert np.all(out["val"] == 1.0)
        return out["idx"].size

    assert union_of(2) == int(gold["values_entering_stage_2"])
    assert union_of(4) == int(gold["values_entering_stage_3"])
    stages = int(gold["stages"])
    assert union_of(2 ** (stages - 1)) == int(gold["values_after_last_stage"])


def test_reduce_equals_dense_sum_of_densified_inputs():
    rng = np.random.default_rng(54)
    n, P = 5000, 12
    chunks = make_chunks(rng, P, 700, n, dyadic=False)
    dense = np.zeros(n, dtype=np.float64)
    for idx, val in chunks:
        d = np.zeros(n, dtype=np.float64)
        d[idx] = val
        dense += d
    out = orc.sparse_reduce(*cat(chunks), 1000, 4000)
    assert np.allclose(out["dense"], dense[1000:4000], rtol=1e-6, atol=0)
    assert math.isclose(float(out["val"].astype(np.float64).sum()),
                        float(dense[1000:4000].sum()), rel_tol=1e-4)


# ------------------------------------------- global select, indexes, residual
def test_coo_select_vs_python_filter_and_dense_select():
    rng = np.random.default_rng(71)
    n = 5000
    idx = np.sort(rng.choice(n, 700, replace=False)).astype(np.uint32)
    val = rand_f32(rng, idx.size)
    val[::50] = 0.0
    val[7] = -val[8]                               # a tie in magnitude
    for th in (abs(float(val[8])), 1e-3, 0.0, 1e9, float(np.abs(val).max())):
        gi, gv, total = orc.coo_threshold_select(idx, val, th)
        th_key = bits(f32(th)) & 0x7FFFFFFF
        want = [(int(i), float(v)) for i, v in zip(idx, val) if (bits(v) & 0x7FFFFFFF) >= th_key]
        assert total == len(want)
        assert [(int(i), float(v)) for i, v in zip(gi, gv)] == want
        if th > 0:
            # absent entries are zeros, below any positive threshold: the dense
            # select of the densified region sees the same set
            dense = np.zeros(n, dtype=np.float32)
            dense[idx] = val
            di, dv, _, dtotal = orc.threshold_select(dense, th)
            assert dtotal == total and np.array_equal(di, gi)
            assert np.array_equal(dv.view(np.uint32), gv.view(np.uint32))
    gi, gv, total = orc.coo_threshold_select(idx, val, 1e-3, capacity=5)
    full_i, full_v, full_total = orc.coo_threshold_select(idx, val, 1e-3)
    assert total == full_total and np.array_equal(gi, full_i[:5]) and np.array_equal(gv, full_v[:5])
    ei, ev, et = orc.coo_threshold_select(idx[:0], val[:0], 1e-3)
    assert ei.size == 0 and ev.size == 0 and et == 0


def test_index_intersection_vs_python_sets():
    rng = np.random.default_rng(72)
    for na, nb in ((0, 0), (0, 9), (9, 0), (40, 40), (300, 57), (57, 300)):
        a = np.sort(rng.choice(500, na, replace=False)).astype(np.uint32)
        b = np.sort(rng.choice(500, nb, replace=False)).astype(np.uint32)
        got = orc.index_intersection(a, b)
        assert got.dtype == np.uint32
        assert [int(x) for x in got] == sorted(set(map(int, a)) & set(map(int, b)))
    a = np.arange(0, 100, 2, dtype=np.uint32)
    assert orc.index_intersection(a, a + 1).size == 0          # disjoint
    assert np.array_equal(orc.index_intersection(a, a), a)     # identical
    assert np.array_equal(orc.index_intersection(a, np.arange(100, dtype=np.uint32)), a)


def test_residual_update_keeps_everything_but_indexes():
    rng = np.random.default_rng(73)
    acc = rand_f32(rng, 2000)
    acc[5] = -0.0
    indexes = np.sort(rng.choice(acc.size, 100, replace=False)).astype(np.uint32)
    eps = orc.residual_update(acc, indexes)
    marked = set(map(int, indexes))
    for i in range(acc.size):
        assert bits(eps[i]) == (0 if i in marked else bits(acc[i])), i
    # all locally selected entries reach the global top-k (one worker, or a
    # global threshold at or below the local one): the update is the plain
    # "zero what was selected" of the local select
    th, _ = orc.topk_threshold_exact(acc, 150)
    li, _, res, _ = orc.threshold_select(acc, th)
    assert np.array_equal(orc.residual_update(acc, orc.index_intersection(li, li)).view(np.uint32),
                          res.view(np.uint32))


def test_what_leaves_the_residuals_is_what_is_applied():
    # Algorithm 1 + Algorithm 2 line 6 over P simulated workers with dyadic
    # values, so every sum is exact: u_t = Topk(sum_i Topk(acc_i)) densified must
    # equal sum_i (acc_i - eps_i) element by element, and a locally selected
    # entry that did not reach the global top-k must still be in its residual.
    rng = np.random.default_rng(74)
    n, P, k = 3000, 4, 90
    accs = [(rng.integers(-2000, 2001, n) / 64.0).astype(np.float32) for _ in range(P)]
    local, chunks_i, chunks_v, off = [], [], [], [0]
    for acc in accs:
        th, _ = orc.topk_threshold_exact(acc, k)
        li, lv, _, _ = orc.threshold_select(acc, th)
        local.append(li)
        chunks_i.append(li)
        chunks_v.append(lv)
        off.append(off[-1] + li.size)
    red = orc.sparse_reduce(np.concatenate(chunks_i), np.concatenate(chunks_v),
                            np.array(off, dtype=np.uint64), 0, n)
    gth, _ = orc.topk_threshold_exact(red["val"], k)
    gi, gv, _ = orc.coo_threshold_select(red["idx"], red["val"], gth)
    assert k <= gi.size < red["idx"].size           # something is filtered out
    u = [Fraction(0)] * n
    for i, v in zip(gi, gv):
        u[int(i)] = Fraction(float(v))
    left = [Fraction(0)] * n
    kept_back = 0
    gset = set(map(int, gi))
    for acc, li in zip(accs, local):
        eps = orc.residual_update(acc, orc.index_intersection(li, gi))
        for i in range(n):
            left[i] += Fraction(float(acc[i])) - Fraction(float(eps[i]))
        for i in map(int, li):
            if i not in gset:
                kept_back += 1
                assert bits(eps[i]) == bits(acc[i])
    assert left == u
    assert kept_back > 0


def test_bucketed_reduce_equals_one_shot_when_sums_are_exact():
    # dyadic values: every partial sum is exact in fp32, so rounding between the
    # buckets changes nothing and the bucketed reduction must equal the one-shot
    # reduction bit for bit; the index set is the same for any values
    rng = np.random.default_rng(81)
    n, P, m = 5000, 12, 400
    parts = [np.sort(rng.choice(n, m, replace=False)).astype(np.uint32) for _ in range(P)]
    dy = [(rng.integers(-4096, 4097, m) / 256.0).astype(np.float32) for _ in range(P)]
    fl = [rand_f32(rng, m) for _ in range(P)]
    off = np.arange(P + 1, dtype=np.uint64) * m
    for vals, exact in ((dy, True), (fl, False)):
        one = orc.sparse_reduce(np.concatenate(parts), np.concatenate(vals), off, 100, 4000)
        buckets = []
        for b in range(0, P, 4):
            buckets.append((np.concatenate(parts[b:b + 4]), np.concatenate(vals[b:b + 4]),
                            np.arange(5, dtype=np.uint64) * m))
        got = orc.sparse_reduce_bucketed(buckets, 100, 4000)
        assert np.array_equal(got["idx"], one["idx"])
        if exact:
            assert np.array_equal(got["val"].view(np.uint32), one["val"].view(np.uint32))
        else:
            # three roundings instead of one: within 3 ulp-sized steps of sum|v|
            assert np.all(np.abs(got["val"].astype(np.float64) - one["val"]) <= 3 * 2.0 ** -24 * one["abs_sum"])
    # one bucket is the plain reduction
    single = orc.sparse_reduce_bucketed([(np.concatenate(parts), np.concatenate(fl), off)], 100, 4000)
    assert np.array_equal(single["val"].view(np.uint32), one["val"].view(np.uint32))


# --------------------------------------------------------------- data balancing
def apply_plan(buffers, chunks):
    """Move labelled entries as the plan says; returns the new buffers."""
    P = len(buffers)
    new = [dict() for _ in range(P)]
    for src, dst, so, do, count in chunks:
        for t in range(count):
            assert do + t not in new[dst]
            new[dst][do + t] = buffers[src][so + t]
    return [[b[t] for t in range(len(b))] for b in new]


def test_balance_plan_moves_every_entry_once_and_keeps_the_order():
    rng = np.random.default_rng(91)
    for P in (5, 8, 16, 33):
        for trial in range(6):
            sizes = [0] * P
            heavy = rng.choice(P, 1 + trial % 2, replace=False)
            for h in heavy:
                sizes[h] = int(rng.integers(200, 900))
            for i in range(P):
                if i not in heavy:
                    sizes[i] = int(rng.integers(0, 12))
            triggered, chunks = orc.balance_plan(sizes)
            T = sum(sizes)
            assert triggered == (max(sizes) * P > 4 * T)
            if not triggered:
                assert chunks == []
                continue
            buffers = [[(i, t) for t in range(sizes[i])] for i in range(P)]
            new = apply_plan(buffers, chunks)
            # nothing lost, nothing doubled, list order kept
            assert [e for b in new for e in b] == [e for b in buffers for e in b]
            # balanced: floor or ceil of T / P each
            assert all(len(b) in (T // P, -(-T // P)) for b in new)
            assert len(chunks) <= 2 * P - 1


def test_balance_plan_worked_by_hand():
    # T = 11 entries, all on worker 0 of P = 5 (11 > 4 x 2.2): balanced, worker j
    # holds list positions [floor(11 j / 5), floor(11 (j+1) / 5)) = [0,2) [2,4) [4,6) [6,8) [8,11)
    triggered, chunks = orc.balance_plan([11, 0, 0, 0, 0])
    assert triggered
    assert chunks == [(0, 0, 0, 0, 2), (0, 1, 2, 0, 2), (0, 2, 4, 0, 2), (0, 3, 6, 0, 2),
                      (0, 4, 8, 0, 3)]
    # T = 13 over P = 6, [1, 0, 12, 0, 0, 0] (12 > 4 x 13/6): the list is the one
    # entry of worker 0, then the twelve of worker 2; targets [0,2) [2,4) [4,6) [6,8) [8,10) [10,13)
    triggered, chunks = orc.balance_plan([1, 0, 12, 0, 0, 0])
    assert triggered
    assert chunks == [(0, 0, 0, 0, 1),          # list position 0 stays
                      (2, 0, 0, 1, 1),          # position 1: first of worker 2 -> second slot of worker 0
                      (2, 1, 1, 0, 2),          # positions 2-3
                      (2, 2, 3, 0, 2),          # positions 4-5: stay on worker 2
                      (2, 3, 5, 0, 2),          # positions 6-7
                      (2, 4, 7, 0, 2),          # positions 8-9
                      (2, 5, 9, 0, 3)]          # positions 10-12


def test_balance_plan_extreme_case_and_trigger_rule():
    # Sec. 3.1.2: all global top-k values on one worker; balancing then moves
    # k (P-1)/P entries = 2k (P-1)/P words, one chunk to every other worker
    gold = read_golden("balance_extreme.txt")
    k, P = 10_000, 8
    env = {"P": P, "k": k}
    for owner in (0, 3, P - 1):
        sizes = [0] * P
        sizes[owner] = k
        triggered, chunks = orc.balance_plan(sizes)
        assert triggered
        moved = [c for c in chunks if c[0] != c[1]]
        assert len(moved) == eval(gold["extreme_chunks_sent"], env)
        assert {c[1] for c in moved} == set(range(P)) - {owner}
        assert 2 * sum(c[4] for c in moved) == eval(gold["extreme_words_moved"], env)
    factor = int(gold["trigger_factor"])
    assert orc.balance_plan([factor * 8 + 1, 8, 8, 8, 7, 0, 0, 0])[0] is True      # avg 8
    assert orc.balance_plan([factor * 8, 8, 8, 8, 8, 0, 0, 0])[0] is False
    # "more than four times the average": exactly four times does not trigger
    assert orc.balance_plan([40, 10, 10, 10, 10, 10, 10, 10, 10, 10, 10, 10, 10])[0] is False   # avg 12.3, 4x = 49.2
    assert orc.balance_plan([16, 0, 0, 0])[0] is False            # P = 4: the max is at most 4 x avg
    assert orc.balance_plan([32, 8, 8, 8, 8, 0, 0, 0])[0] is False   # avg 8, max = 4 x avg
    assert orc.balance_plan([33, 8, 8, 8, 7, 0, 0, 0])[0] is True
    assert orc.balance_plan([0, 0, 0, 0, 0, 0])[0] is False
