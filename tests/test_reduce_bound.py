"""The bound the GPU parity tests hold reduced values to (tests/okt_harness.py):
a mistake that the stated tolerance alone would let through - one small
contribution dropped from a sum - must fall outside it, while the legitimate
differences (another order of the fp64 additions, one fp32 rounding) stay inside.
The mistake is planted in a copy of the oracle's result, on the CPU."""
import numpy as np

from oracle import okt_oracle as orc
from tests.okt_harness import reduce_tolerance, rounding_bound, stated_tolerance


def contributions(seed, P=24, m=3000, width=20_000):
    rng = np.random.default_rng(seed)
    idx, val, off = [], [], [0]
    for p in range(P):
        i = np.sort(rng.choice(width, m, replace=False)).astype(np.uint32)
        # magnitudes over seven decades: the small ones vanish inside 1e-6 * sum|v|
        v = (rng.standard_normal(m) * 10.0 ** rng.uniform(-9, -2, m)).astype(np.float32)
        idx.append(i), val.append(v), off.append(off[-1] + m)
    return np.concatenate(idx), np.concatenate(val), np.array(off, dtype=np.uint64)


def test_a_dropped_small_contribution_fails_the_bound_but_not_the_stated_tolerance():
    idx, val, off = contributions(5)
    ref = orc.sparse_reduce(idx, val, off, 0, 20_000)
    # drop, per output slot, its smallest contribution (where the slot has several)
    order = np.lexsort((np.abs(val), idx))                    # by slot, smallest magnitude first
    first = np.ones(order.size, dtype=bool)
    first[1:] = idx[order][1:] != idx[order][:-1]
    keep = np.ones(val.size, dtype=bool)
    several = np.isin(idx, ref["idx"][ref["hits"] > 1])
    keep[order[first]] = False
    keep |= ~several
    wrong = np.zeros(20_000, dtype=np.float64)
    np.add.at(wrong, idx[keep].astype(np.int64), val[keep].astype(np.float64))
    got = wrong[ref["idx"]].astype(np.float32)
    err = np.abs(got.astype(np.float64) - ref["val"].astype(np.float64))
    hidden = (err > 0) & (err <= stated_tolerance(ref))       # the stated tolerance lets these through
    assert hidden.sum() > 100
    # the bound in force does not, unless the dropped value is below a rounding step of
    # the sum (then no fp32 result can tell)
    caught = err[hidden] > rounding_bound(ref)[hidden]
    assert caught.sum() > 100 and caught.mean() > 0.5
    assert np.array_equal(err > reduce_tolerance(ref), (err > stated_tolerance(ref)) | (err > rounding_bound(ref)))


def test_reordered_fp64_sums_stay_inside_the_bound():
    idx, val, off = contributions(6)
    ref = orc.sparse_reduce(idx, val, off, 0, 20_000)
    rng = np.random.default_rng(7)
    for _ in range(3):
        perm = rng.permutation(val.size)                      # any order of the additions
        acc = np.zeros(20_000, dtype=np.float64)
        np.add.at(acc, idx[perm].astype(np.int64), val[perm].astype(np.float64))
        got = acc[ref["idx"]].astype(np.float32)
        err = np.abs(got.astype(np.float64) - ref["val"].astype(np.float64))
        assert np.all(err <= reduce_tolerance(ref))
