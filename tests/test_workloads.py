"""The seeded input generators: shapes, determinism and the structure the
reduce expects (strictly ascending indices inside each chunk, inside the region)."""
import numpy as np
import pytest

import workloads as wl


def test_k_and_m_of_the_five_configurations():
    assert wl.WORKLOADS["cfg1"].k == 10_486 and wl.WORKLOADS["cfg1"].m == 2_621
    assert wl.WORKLOADS["cfg2"].k == 255_571 and wl.WORKLOADS["cfg2"].m == 15_973
    assert wl.WORKLOADS["cfg3"].k == 1_100_000 and wl.WORKLOADS["cfg3"].m == 34_375
    assert wl.WORKLOADS["cfg4"].k == 336_000 and wl.WORKLOADS["cfg4"].m == 5_250
    assert wl.WORKLOADS["cfg5"].k == 1_100_000 and wl.WORKLOADS["cfg5"].m == 4_296


def test_refresh_schedule():
    assert [it for it in range(10) if wl.WORKLOADS["cfg2"].refresh(it)] == [0]
    assert [it for it in range(64) if wl.WORKLOADS["cfg3"].refresh(it)] == [0, 32]
    assert all(wl.WORKLOADS["cfg4"].refresh(it) for it in range(3))


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4"])
def test_gradient_is_deterministic_and_chunk_parallel_safe(name):
    w = wl.WORKLOADS[name].scaled((1 << 23) + 12345 if name == "cfg2" else 300_001)
    a = wl.gradient(w, 0)
    b = wl.gradient(w, 0)
    c = wl.gradient(w, 1)
    assert a.dtype == np.float32 and a.shape == (w.n,)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert np.isfinite(a).all() and a.std() > 0


def test_segment_table_covers_the_vector():
    w = wl.WORKLOADS["cfg2"].scaled(1_000_003)
    bounds, scale = wl.segment_table(w)
    assert bounds[0] == 0 and bounds[-1] == w.n and len(scale) == 161
    assert np.all(np.diff(bounds) >= 64)
    assert scale.min() >= 1e-5 and scale.max() <= 1e-2


@pytest.mark.parametrize("name,width", [("cfg1", 40_000), ("cfg3", 50_000), ("cfg5", 20_000)])
def test_contributions_structure(name, width):
    w = wl.WORKLOADS[name]
    lo, hi = 7 * width, 8 * width
    idx, val, off = wl.contributions(w, lo, hi, m=500, P=9)
    assert idx.dtype == np.uint32 and val.dtype == np.float32 and off.dtype == np.uint64
    assert off[0] == 0 and off[-1] == idx.size == 9 * 500
    for p in range(9):
        part = idx[int(off[p]):int(off[p + 1])].astype(np.int64)
        assert np.all(np.diff(part) > 0) and part[0] >= lo and part[-1] < hi
    again = wl.contributions(w, lo, hi, m=500, P=9)
    assert np.array_equal(idx, again[0]) and np.array_equal(val, again[1])
    other = wl.contributions(w, lo, hi, m=500, P=9, stream=1)
    assert not np.array_equal(idx, other[0])
    if name == "cfg3":       # 30 % of every worker's indices are one shared pool
        sets = [set(idx[int(off[p]):int(off[p + 1])]) for p in range(9)]
        assert len(set.intersection(*sets)) >= 150
    if name == "cfg5":       # Zipf through a shared permutation: hot indices collide
        _, counts = np.unique(idx, return_counts=True)
        assert counts.max() == 9
