"""The three-pass form of the select calls (per-tile slots; Sec. 3.1.3 threshold
selection, Sec. 3.1.2 packaging, Algorithm 2 line 6 residual update) on vectors
built tile by tile: tiles of 1024 elements that select nothing, a few entries
(the lane-per-tile copy), up to a slot-full (the half-wave copy), and more than a
slot holds (walked again), in runs and alone, with the output cut short inside
each kind.  Every result is compared with the oracle bit for bit, and the
one-kernel form has to give the same.
"""
import numpy as np
import pytest
import torch

import paper_2201_07598_amd as okt
from oracle import okt_oracle as orc
from tests.okt_harness import DEV, bits_equal, to_dev, u32, u64, workspace

pytestmark = pytest.mark.gpu

TILE = 1024          # elements per tile of the three-pass form
SLOT = 128           # entries a tile's slot holds
FEW = 4              # entries copied by the tile's own lane


def tiled_vector(rng, counts, last=TILE):
    """A vector of len(counts) tiles, the last one `last` elements long: tile t has
    counts[t] elements of magnitude in [1, 2) at random places, everything else
    lies below 0.5."""
    n = (len(counts) - 1) * TILE + last
    x = (rng.random(n, dtype=np.float32) * np.float32(0.5)).astype(np.float32)
    x *= rng.choice(np.array([-1.0, 1.0], dtype=np.float32), n)
    for t, c in enumerate(counts):
        width = TILE if t + 1 < len(counts) else last
        where = rng.choice(width, min(c, width), replace=False) + t * TILE
        x[where] = (1.0 + rng.random(where.size, dtype=np.float32)) * rng.choice(
            np.array([-1.0, 1.0], dtype=np.float32), where.size)
    return x


def run_select(form, call, x, th, cap, grad=None, lr=1.0):
    okt.okt_debug_slot_min_n(1 if form == "three_pass" else 1 << 40)
    try:
        n = x.size
        d = to_dev(x)
        d_th = to_dev(np.array([th], dtype=np.float32))
        idx = torch.full((max(cap, 1),), -1, dtype=torch.int32, device=DEV)
        val = torch.zeros(max(cap, 1), device=DEV)
        nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
        ws = workspace(okt.okt_workspace_bytes(n, 0))
        ws.fill_(0xCD)
        if call == "select":
            okt.okt_threshold_select(d, d_th, idx, val, nnz, ws, capacity=cap)
        elif call == "copy":
            okt.okt_threshold_select_copy(d, d_th, idx, val, nnz, ws, capacity=cap)
        else:
            okt.okt_accumulate_select(to_dev(grad), d, lr, d_th, idx, val, nnz, ws, capacity=cap)
        torch.cuda.synchronize()
        c = u64(nnz)
        e = int(c[0])
        return u32(idx[:e]).copy(), val[:e].cpu().numpy(), d.cpu().numpy(), (e, int(c[1]))
    finally:
        okt.okt_debug_slot_min_n(0)


def check_all_calls(x, th, cap, rng):
    ridx, rval, rres, total = orc.threshold_select(x, th, capacity=cap)
    for form in ("three_pass", "one_kernel"):
        gi, gv, gd, gc = run_select(form, "select", x, th, cap)
        assert gc == (ridx.size, total), form
        assert np.array_equal(gi, ridx) and bits_equal(gv, rval) and bits_equal(gd, rres), form
        gi, gv, gd, gc = run_select(form, "copy", x, th, cap)
        assert gc == (ridx.size, total), form
        assert np.array_equal(gi, ridx) and bits_equal(gv, rval) and bits_equal(gd, x), form
    # the accumulate on the way: eps + lr * G gives the vector built above (G = x / lr
    # with lr a power of two; eps carries x itself in places, with G = 0 there)
    g = (x * np.float32(4.0)).astype(np.float32)
    eps = np.zeros_like(x)
    carried = rng.random(x.size) < 0.3
    eps[carried], g[carried] = x[carried], 0.0
    acc = orc.residual_accumulate(g, eps, 0.25)
    ridx, rval, rres, total = orc.threshold_select(acc, th, capacity=cap)
    for form in ("three_pass", "one_kernel"):
        gi, gv, gd, gc = run_select(form, "fused", eps, th, cap, grad=g, lr=0.25)
        assert gc == (ridx.size, total), form
        assert np.array_equal(gi, ridx) and bits_equal(gv, rval) and bits_equal(gd, rres), form


@pytest.mark.parametrize("last", [TILE, 1, 700, 1023])
def test_every_kind_of_tile(last):
    rng = np.random.default_rng(40 + last)
    counts = [0, 1, FEW, FEW + 1, 0, SLOT - 1, SLOT, SLOT + 1, 0, 0, 2, 1024, 600, 3, 0, 5,
              SLOT + 1, SLOT, 1, 0]
    counts += [int(c) for c in rng.integers(0, 3, 70)]              # a sparse stretch
    counts += [int(c) for c in rng.integers(FEW + 1, SLOT + 1, 70)]  # a run of fuller slots
    counts += [int(c) for c in rng.integers(SLOT + 1, 400, 70)]      # a run of dense tiles
    counts += [int(c) for c in rng.integers(0, 2 * SLOT, 300)]       # everything mixed
    for c_last in (0, 3, 40):                                        # the last tile, whole or ragged
        x = tiled_vector(rng, counts + [c_last], last=last)
        total = int(np.count_nonzero(np.abs(x) >= 1.0))
        check_all_calls(x, 1.0, total + 3, rng)


def test_output_cut_short_inside_each_kind_of_tile():
    rng = np.random.default_rng(77)
    counts = [3, 0, 2, SLOT - 2, SLOT, 500, 4, 1, SLOT + 9, 2]
    x = tiled_vector(rng, counts)
    edges = np.cumsum([0] + counts)
    for cap in sorted({0, 1, 2, 4, edges[3] + 5, edges[4], edges[4] + 1, edges[5] + 7, edges[6],
                       edges[6] + 2, edges[8] + 4, edges[-1] - 1, edges[-1]}):
        check_all_calls(x, 1.0, int(cap), rng)


def test_thresholds_at_the_ends_of_the_order():
    rng = np.random.default_rng(5)
    x = tiled_vector(rng, [2, 40, 0, 7, 1024, 3, 9], last=100)
    x[5] = np.float32("nan")
    x[2000] = np.float32("inf")
    x[3000] = -np.float32("inf")
    n = x.size
    for th in (0.0, np.float32(1e-45), 1.0, np.float32("inf"), np.float32("nan")):
        check_all_calls(x, np.float32(th), n, rng)
        check_all_calls(x, np.float32(th), n // 3, rng)


@pytest.mark.parametrize("n", [1, 63, 1024, 1025, 4 * 1024, 4 * 1024 + 1, 5 * 1024 - 1])
def test_vectors_of_a_few_tiles(n):
    rng = np.random.default_rng(n)
    x = rng.laplace(0, 1.0, n).astype(np.float32)
    for th in (0.0, 0.5, 2.0, 50.0):
        check_all_calls(x, np.float32(th), n, rng)
        check_all_calls(x, np.float32(th), max(n // 2, 1), rng)


def test_a_workspace_without_room_for_slots_takes_the_one_kernel_form():
    rng = np.random.default_rng(12)
    x = tiled_vector(rng, [int(c) for c in rng.integers(0, 50, 200)])
    ridx, rval, rres, total = orc.threshold_select(x, 1.0, capacity=x.size)
    okt.okt_debug_slot_min_n(1)
    try:
        d = to_dev(x)
        d_th = to_dev(np.array([1.0], dtype=np.float32))
        idx = torch.full((x.size,), -1, dtype=torch.int32, device=DEV)
        val = torch.zeros(x.size, device=DEV)
        nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
        ws = workspace(32 * 1024)                    # scan state of the one-kernel form only
        okt.okt_threshold_select(d, d_th, idx, val, nnz, ws, capacity=x.size)
        torch.cuda.synchronize()
        assert (int(u64(nnz)[0]), int(u64(nnz)[1])) == (ridx.size, total)
        assert np.array_equal(u32(idx[:total]), ridx)
        assert bits_equal(val[:total].cpu().numpy(), rval) and bits_equal(d.cpu().numpy(), rres)
    finally:
        okt.okt_debug_slot_min_n(0)


def test_three_pass_waits_that_give_up_are_reported():
    """With a poll limit of 1 the scan over the tile counts either completes or
    reports UINT64_MAX counts; it never hangs."""
    rng = np.random.default_rng(3)
    n = 3_000_000                                   # several workgroups of the second pass
    x = rng.laplace(0, 1.0, n).astype(np.float32)
    ridx, rval, rres, total = orc.threshold_select(x, 3.0, capacity=n)
    okt.okt_debug_slot_min_n(1)
    okt.okt_debug_spin_limit(1)
    try:
        d_th = to_dev(np.array([3.0], dtype=np.float32))
        idx = torch.full((n,), -1, dtype=torch.int32, device=DEV)
        val = torch.zeros(n, device=DEV)
        nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
        ws = workspace(okt.okt_workspace_bytes(n, 0))
        for _ in range(4):
            okt.okt_threshold_select_copy(to_dev(x), d_th, idx, val, nnz, ws, capacity=n)
            torch.cuda.synchronize()
            c = u64(nnz)
            if int(c[1]) == 0xFFFFFFFFFFFFFFFF:
                assert int(c[0]) == 0xFFFFFFFFFFFFFFFF
            else:
                assert (int(c[0]), int(c[1])) == (total, total)
                assert np.array_equal(u32(idx[:total]), ridx)
    finally:
        okt.okt_debug_spin_limit(0)
        okt.okt_debug_slot_min_n(0)
