"""GPU parity of okt_accumulate_topk_select: a refresh iteration in one call
(accumulate, exact threshold, select; Algorithm 2, lines 4-6 with Algorithm 1,
lines 2-4) against the oracle's three definitions applied one after the other.
Everything is compared bit for bit.
"""
import numpy as np
import pytest
import torch

import paper_2201_07598_amd as okt
import workloads as wl
from oracle import okt_oracle as orc
from tests.okt_harness import DEV, bits_equal, to_dev, u32, u64, workspace

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("select_form")]


def lap(seed, n, scale=1e-3):
    return np.random.default_rng(seed).laplace(0, scale, n).astype(np.float32)


def check_refresh(g, e, lr, k, capacity, ws_bytes=None, method="partition"):
    n = g.size
    d_g, d_e = to_dev(g), to_dev(e)
    th = torch.full((1,), -7.0, dtype=torch.float32, device=DEV)
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    idx = torch.full((max(capacity, 1),), -1, dtype=torch.int32, device=DEV)
    val = torch.zeros(max(capacity, 1), dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(n, 0) if ws_bytes is None else ws_bytes)
    ws.fill_(0xAB)                                   # whatever the workspace held before
    okt.okt_accumulate_topk_select(d_g, d_e, lr, k, th, cnt, idx, val, nnz, ws, capacity=capacity)
    torch.cuda.synchronize()
    acc = orc.residual_accumulate(g, e, lr)
    rth, rcnt = orc.topk_threshold_exact(acc, k, method=method)
    ridx, rval, rres, rtotal = orc.threshold_select(acc, rth, capacity=capacity)
    got_th = th.cpu().numpy()
    assert got_th.view(np.uint32)[0] == np.float32(rth).view(np.uint32), (got_th, rth)
    assert int(u64(cnt)[0]) == rcnt == rtotal
    c = u64(nnz)
    assert (int(c[0]), int(c[1])) == (ridx.size, rtotal)
    assert np.array_equal(u32(idx[:ridx.size]), ridx)
    assert bits_equal(val[:ridx.size].cpu().numpy(), rval)
    assert bits_equal(d_e.cpu().numpy(), rres)
    assert bits_equal(d_g.cpu().numpy(), g)          # the gradient is read only
    return rtotal


@pytest.mark.parametrize("n", [1, 3, 1023, 4097, 70_001, 1_000_003])
def test_short_vectors_take_the_three_steps(n):
    g, e = lap(n + 3, n), lap(n + 4, n, 2e-3)
    e[::5] = 0
    for k in sorted({1, max(1, n // 100), n}):
        check_refresh(g, e, 0.25, k, n, method="sort" if n < 5000 else "partition")


@pytest.mark.timeout(300)
@pytest.mark.parametrize("n", [(1 << 22), (1 << 22) + 5, 6_000_011])
def test_long_vectors_one_pass(n):
    g, e = lap(n + 3, n), lap(n + 4, n, 2e-3)
    e[::5] = 0
    k = n // 100
    total = check_refresh(g, e, 0.25, k, 4 * k)
    assert total >= k
    # the output fills up: only what was emitted is zeroed, the counts say so
    check_refresh(g, e, 0.25, k, k // 3)
    check_refresh(g, e, 0.25, k, 0)
    # k = 1 and a k so large that the candidates do not fit (whole-vector path)
    check_refresh(g, e, -0.5, 1, 16)
    check_refresh(g, e, 1.0, n // 2, n // 2 + 8)
    check_refresh(g, e, 1.0, n, n)


@pytest.mark.timeout(300)
def test_workload_vector_with_carried_residual():
    """Layered gradients (whole layers above the bound: pieces overflow their
    stash while the candidates are collected) and a residual carried over."""
    w = wl.WORKLOADS["cfg2"].scaled(9_000_017)
    e = np.zeros(w.n, dtype=np.float32)
    for it in range(2):
        g = wl.gradient(w, it)
        check_refresh(g, e, 1.0, w.k, 4 * w.k)
        acc = orc.residual_accumulate(g, e, 1.0)
        th, _ = orc.topk_threshold_exact(acc, w.k, method="partition")
        e = orc.threshold_select(acc, th)[2]


@pytest.mark.timeout(300)
def test_sample_that_misleads_and_ties():
    n = 5_000_011
    zero = np.zeros(n, dtype=np.float32)
    # the large values hide in blocks the sample never looks at (it reads every
    # 4th block of 1024 elements at this length): fewer candidates than k
    hidden = lap(6, n, 1e-6)
    big = np.random.default_rng(7).laplace(0, 1.0, n).astype(np.float32)
    mask = ((np.arange(n) // 1024) % 4) == 1
    hidden[mask] = big[mask]
    for k in (10, 40_000, 1_000_000):
        check_refresh(hidden, zero, 1.0, k, k + 100)
    # every value equal: the candidates are the whole vector and do not fit
    same = np.full(4_500_000, 0.25, dtype=np.float32)
    assert check_refresh(same, np.zeros_like(same), 1.0, 45_000, 4_500_000) == 4_500_000
    # the same with pieces longer than a wave's stash (the whole-vector select then
    # walks part of every piece twice), once with room for everything, once cut short
    same = np.full(9_000_000, -0.25, dtype=np.float32)
    assert check_refresh(same, np.zeros_like(same), 1.0, 90_000, 9_000_000) == 9_000_000
    assert check_refresh(same, np.zeros_like(same), 1.0, 90_000, 5_000_001) == 9_000_000
    # heavy ties around rank k: all of them are selected
    tied = lap(8, n)
    tied[100_000:400_000] = np.float32(3e-3)
    above = int((np.abs(tied) > np.float32(3e-3)).sum())
    assert check_refresh(tied, zero, 1.0, above + 1000, above + 300_000) == above + 300_000
    # gradient and residual that cancel: acc is mostly zero
    g = lap(9, n)
    e = (-g).astype(np.float32)
    e[::1000] = 0
    check_refresh(g, e, 1.0, 1000, 4000)


@pytest.mark.timeout(300)
def test_small_workspace_same_result():
    n = 5_000_011
    g, e = lap(11, n), lap(12, n, 2e-3)
    k = 50_000
    need = okt.okt_workspace_bytes(n, 0)
    for ws_bytes in (need, need // 8, 128 * 1024):
        check_refresh(g, e, 0.5, k, 2 * k, ws_bytes=ws_bytes)
    with pytest.raises(okt.OktError):
        check_refresh(g, e, 0.5, k, 2 * k, ws_bytes=1024)


def test_nan_and_inf_elements():
    n = 4_200_000
    rng = np.random.default_rng(n)
    g = lap(n + 1, n)
    bits = g.view(np.uint32)
    where = rng.choice(n, 160, replace=False)
    bits[where[:100]] = (np.uint32(0x7F800001) + rng.integers(0, 0x7FFFFE, 100).astype(np.uint32)) \
        | (rng.integers(0, 2, 100).astype(np.uint32) << np.uint32(31))
    bits[where[100:]] = np.where(rng.integers(0, 2, 60) == 1, 0xFF800000, 0x7F800000).astype(np.uint32)
    e = np.zeros(n, dtype=np.float32)
    for k in (1, 100, 101, 161, 42_000):
        check_refresh(g, e, 1.0, k, k + 200)


def test_argument_errors_are_caught_on_the_host():
    n = 1000
    g, e = to_dev(lap(1, n)), to_dev(lap(2, n))
    th = torch.zeros(1, dtype=torch.float32, device=DEV)
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    idx = torch.zeros(8, dtype=torch.int32, device=DEV)
    val = torch.zeros(8, dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(n, 0))
    for k in (0, n + 1):
        with pytest.raises(okt.OktError):
            okt.okt_accumulate_topk_select(g, e, 1.0, k, th, cnt, idx, val, nnz, ws)
    with pytest.raises(okt.OktError):
        okt.okt_accumulate_topk_select(e, e, 1.0, 5, th, cnt, idx, val, nnz, ws)
    okt.okt_accumulate_topk_select(g, e, 1.0, 5, th, cnt, idx, val, nnz, ws)
    torch.cuda.synchronize()
    assert int(u64(nnz)[1]) >= 5


def test_bounded_waits_that_give_up_are_reported():
    """With the waits between workgroups limited to one poll (a test hook) the call
    never hangs: if the collection of the candidates gives up, the whole-vector
    path takes over, so the threshold and its count stay exact; if the final
    select gives up, its counts read UINT64_MAX, as okt_threshold_select's do."""
    n, k = 6_000_011, 60_000
    g, e = lap(21, n), lap(22, n, 2e-3)
    acc = orc.residual_accumulate(g, e, 0.5)
    rth, rcnt = orc.topk_threshold_exact(acc, k, method="partition")
    ridx, rval, rres, total = orc.threshold_select(acc, rth, capacity=2 * k)
    bad = 0xFFFFFFFFFFFFFFFF
    outcomes = []
    try:
        okt.okt_debug_spin_limit(1)
        for rep in range(3):
            d_g, d_e = to_dev(g), to_dev(e)
            th = torch.zeros(1, dtype=torch.float32, device=DEV)
            cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
            idx = torch.full((2 * k,), -1, dtype=torch.int32, device=DEV)
            val = torch.zeros(2 * k, dtype=torch.float32, device=DEV)
            nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
            ws = workspace(okt.okt_workspace_bytes(n, 0))
            okt.okt_accumulate_topk_select(d_g, d_e, 0.5, k, th, cnt, idx, val, nnz, ws)
            torch.cuda.synchronize()
            assert th.cpu().numpy().view(np.uint32)[0] == np.float32(rth).view(np.uint32)
            assert int(u64(cnt)[0]) == rcnt
            c = u64(nnz)
            if int(c[1]) == bad:
                outcomes.append("gave up")
                assert int(c[0]) == bad
            else:
                outcomes.append("completed")
                assert (int(c[0]), int(c[1])) == (ridx.size, total)
                assert np.array_equal(u32(idx[:total]), ridx) and bits_equal(d_e.cpu().numpy(), rres)
    finally:
        okt.okt_debug_spin_limit(0)
    print(outcomes, flush=True)
    check_refresh(g, e, 0.5, k, 2 * k)               # the limit restored: exact again


@pytest.mark.timeout(300)
def test_the_call_captured_in_a_hip_graph_replays_like_eager():
    """The call enqueues kernels only (its state is cleared by a kernel, not a
    memset), so it can be captured once and replayed: every replay - with eager
    work and synchronisations in between - against the oracle, which follows the
    carried residual.  Long enough for the one-pass path."""
    n, lr, k, rounds = 4_300_003, 0.5, 43_000, 4
    grads = [lap(400 + r, n) for r in range(rounds)]
    d_g = to_dev(grads[0])
    res = torch.zeros(n, dtype=torch.float32, device=DEV)
    th = torch.zeros(1, dtype=torch.float32, device=DEV)
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    cap = 2 * k
    idx = torch.full((cap,), -1, dtype=torch.int32, device=DEV)
    val = torch.zeros(cap, dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(n, 0))
    okt.load_library()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        okt.okt_accumulate_topk_select(d_g, res, lr, k, th, cnt, idx, val, nnz, ws, capacity=cap)
    res.zero_()                                    # capture does not run anything; start clean anyway
    host_res = np.zeros(n, dtype=np.float32)
    for r in range(rounds):
        d_g.copy_(torch.from_numpy(grads[r]))      # eager work between the replays
        idx.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        acc = orc.residual_accumulate(grads[r], host_res, lr)
        rth, rcnt = orc.topk_threshold_exact(acc, k, method="partition")
        ridx, rval, host_res, total = orc.threshold_select(acc, rth, capacity=cap)
        assert th.cpu().numpy().view(np.uint32)[0] == np.float32(rth).view(np.uint32), r
        assert int(u64(cnt)[0]) == rcnt == total, r
        c = u64(nnz)
        assert (int(c[0]), int(c[1])) == (ridx.size, total), r
        assert np.array_equal(u32(idx[:total]), ridx) and bits_equal(val[:total].cpu().numpy(), rval), r
        assert bits_equal(res.cpu().numpy(), host_res), r
