"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
element by element on the same seeded inputs.

Bar: bit-exact for the threshold, the counts, the selected index set, the copied
values, the residual and the region boundaries; reduced fp32 values within
1e-6 * sum|v| (1e-5 * sum|v| where more than 64 contributions collide).
"""
import numpy as np
import pytest
import torch

import paper_2201_07598_amd as okt
import workloads as wl
from oracle import okt_oracle as orc
from tests.okt_harness import (DEV, GpuPath, bits_equal, gpu_reduce, reduce_tolerance, to_dev,
                               u32, u64, workspace)

pytestmark = pytest.mark.gpu


def lap(seed, n, scale=1e-3):
    return np.random.default_rng(seed).laplace(0, scale, n).astype(np.float32)


# ------------------------------------------------------------------ accumulate
@pytest.mark.parametrize("n", [1, 3, 4, 5, 1023, 4096, 4097, 65536 + 7, (1 << 20) + 2])
@pytest.mark.parametrize("lr", [1.0, 0.1, -2.5e-3])
def test_accumulate_bitwise(n, lr):
    g, e = lap(n, n), lap(n + 1, n, 3e-3)
    e[::7] = 0
    d_e = to_dev(e)
    okt.okt_residual_accumulate(to_dev(g), d_e, lr)
    assert bits_equal(d_e.cpu().numpy(), orc.residual_accumulate(g, e, lr))


def test_time_next_kernel_brackets_one_launch():
    n = 4_000_000
    g, e = to_dev(lap(1, n)), to_dev(lap(2, n))
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(); b.record()                            # the events exist from here on
    torch.cuda.synchronize()
    okt.okt_time_next_kernel(a, b)
    okt.okt_residual_accumulate(g, e, 0.5)
    torch.cuda.synchronize()
    first = a.elapsed_time(b)
    assert 0.003 < first < 5.0                        # ms: one pass over 48 MB
    okt.okt_residual_accumulate(g, e, 0.5)            # the pair was used once: not recorded again
    torch.cuda.synchronize()
    assert a.elapsed_time(b) == first


@pytest.mark.parametrize("n", [0, 1, 3, 1024, 4099, 1 << 20, 4_000_003])
def test_streaming_ceiling_kernels(n):
    """The two measurement kernels move what they say: the copy is exact, the
    partial sums add up to the vector's sum (fp32 partials against an fp64 sum)."""
    x = lap(7, n)
    d_x = to_dev(x)
    d_y = torch.full((n + 8,), 7.0, dtype=torch.float32, device=DEV)
    okt.okt_stream_copy(d_x, d_y[:n])
    parts = torch.full((okt.STREAM_SUM_PARTIALS,), 7.0, dtype=torch.float32, device=DEV)
    okt.okt_stream_sum(d_x, parts)
    torch.cuda.synchronize()
    y = d_y.cpu().numpy()
    assert bits_equal(y[:n], x) and np.all(y[n:] == 7.0)
    total = float(parts.cpu().numpy().astype(np.float64).sum())
    assert abs(total - float(x.astype(np.float64).sum())) <= 1e-6 * float(np.abs(x).sum()) + 1e-30


def test_gather_ceiling_kernel_moves_every_entry_once():
    """The measurement kernel behind the reduce's traffic ceiling: same tiles and
    slice table as the batched reduce; every input entry of a region must come out
    at its own position, bit for bit, and nothing else may be written."""
    w = wl.WORKLOADS["cfg3"]
    B, P, width, m = 7, 12, 50_000, 1_900
    parts, offs, lohi = [], [], []
    base = 0
    for j in range(B):
        lo = 3_000_000 * j + 11
        hi = lo + width - 777 * j
        ci, cv, co = wl.contributions(w, lo, hi, m=m, P=P, stream=40 + j)
        parts.append((ci, cv))
        offs.append(co + np.uint64(base))
        lohi += [lo, hi]
        base += ci.size
    idx_cat = np.concatenate([p[0] for p in parts])
    val_cat = np.concatenate([p[1] for p in parts])
    cap = max(p[0].size for p in parts) + 5
    out_idx = torch.full((B * cap,), -1, dtype=torch.int32, device=DEV)
    out_val = torch.full((B * cap,), 7.0, dtype=torch.float32, device=DEV)
    ws = workspace(okt.okt_sparse_reduce_batch_workspace_bytes(B, P, width))
    okt.okt_stream_gather(to_dev(idx_cat), to_dev(val_cat), to_dev(np.concatenate(offs)),
                          to_dev(np.array(lohi, dtype=np.uint32)), B, P, width, out_idx, out_val, cap, ws)
    torch.cuda.synchronize()
    gi, gv = u32(out_idx).reshape(B, cap), out_val.cpu().numpy().reshape(B, cap)
    for j in range(B):
        e = parts[j][0].size
        assert np.array_equal(gi[j, :e], parts[j][0]) and bits_equal(gv[j, :e], parts[j][1]), j
        assert np.all(gi[j, e:] == 0xFFFFFFFF) and np.all(gv[j, e:] == 7.0), j


def test_accumulate_not_fused_and_subnormals():
    lr = 1.0 + 2.0 ** -12
    g = np.array([1.0 + 2.0 ** -12, 1e-40, -1e-45, 3e-39] * 8, dtype=np.float32)
    e = np.array([-(1.0 + 2.0 ** -11), 1e-41, 1e-45, -1e-39] * 8, dtype=np.float32)
    d_e = to_dev(e)
    okt.okt_residual_accumulate(to_dev(g), d_e, lr)
    got = d_e.cpu().numpy()
    assert got[0] == 0.0
    assert bits_equal(got, orc.residual_accumulate(g, e, lr))


# ------------------------------------------------------------------- threshold
def gpu_threshold(acc, k, ws_bytes=None):
    d = to_dev(acc)
    th = torch.zeros(1, dtype=torch.float32, device=DEV)
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(acc.size, 0) if ws_bytes is None else ws_bytes)
    okt.okt_topk_threshold_exact(d, k, th, cnt, ws)
    assert bits_equal(d.cpu().numpy(), acc)          # input untouched
    return th.cpu().numpy()[0], int(u64(cnt)[0])


@pytest.mark.parametrize("n,k", [(1, 1), (5, 2), (1000, 10), (4096, 4096), (4097, 1),
                                 (100_003, 1001), ((1 << 21) + 13, 20_972)])
def test_threshold_exact_bits(n, k):
    acc = lap(7 * n + k, n)
    th, cnt = gpu_threshold(acc, k)
    rth, rcnt = orc.topk_threshold_exact(acc, k)
    assert np.float32(th).view(np.uint32) == np.float32(rth).view(np.uint32)
    assert cnt == rcnt


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4"])
def test_threshold_on_workload_distributions(name):
    w = wl.WORKLOADS[name].scaled(3_000_017)
    acc = wl.gradient(w, 0)
    for k in (w.k, 1, w.n // 2):
        th, cnt = gpu_threshold(acc, k)
        rth, rcnt = orc.topk_threshold_exact(acc, k, method="partition")
        assert np.float32(th).view(np.uint32) == np.float32(rth).view(np.uint32) and cnt == rcnt


def test_threshold_ties_and_degenerate_inputs():
    same = np.full(70_001, -0.125, dtype=np.float32)
    assert gpu_threshold(same, 17) == (0.125, 70_001)
    zeros = np.zeros(9_999, dtype=np.float32)
    zeros[::2] = -0.0
    assert gpu_threshold(zeros, 5000) == (0.0, 9_999)
    # duplicates straddling rank k
    acc = lap(3, 200_000)
    acc[1000:1400] = np.float32(2.5e-3) * np.where(np.arange(400) % 2, 1, -1).astype(np.float32)
    above = int((np.abs(acc) > np.float32(2.5e-3)).sum())
    for k in (above + 1, above + 200, above + 400):
        th, cnt = gpu_threshold(acc, k)
        assert th == np.float32(2.5e-3) and cnt == above + 400
        assert (th, cnt) == orc.topk_threshold_exact(acc, k)
    # subnormals, zeros and an infinity
    odd = np.array([0.0, -0.0, 1e-45, -1e-40, 1.0, np.inf, -3.0] * 11, dtype=np.float32)
    for k in range(1, odd.size + 1, 5):
        th, cnt = gpu_threshold(odd, k)
        rth, rcnt = orc.topk_threshold_exact(odd, k)
        assert np.float32(th).view(np.uint32) == np.float32(rth).view(np.uint32) and cnt == rcnt


def test_threshold_sampled_path():
    """Vectors long enough for the sample-then-count path, including inputs on
    which the sample misleads and the full radix select has to take over."""
    n = 5_000_011
    acc = lap(5, n)
    for k in (1, 50_000, n // 2, n):
        th, cnt = gpu_threshold(acc, k)
        rth, rcnt = orc.topk_threshold_exact(acc, k, method="partition")
        assert np.float32(th).view(np.uint32) == np.float32(rth).view(np.uint32) and cnt == rcnt
    # the workspace too small for the candidates: same answer without sampling
    assert gpu_threshold(acc, 50_000, ws_bytes=64 * 1024) == gpu_threshold(acc, 50_000)
    # every value equal: the candidates are the whole vector and do not fit
    same = np.full(4_500_000, 0.25, dtype=np.float32)
    assert gpu_threshold(same, 45_000) == (0.25, 4_500_000)
    # the large values hide in blocks the sample never looks at (it reads every
    # 4th block of 1024 elements at this length)
    hidden = lap(6, n, 1e-6)
    big = np.random.default_rng(7).laplace(0, 1.0, n).astype(np.float32)
    blocks = np.arange(n) // 1024
    mask = (blocks % 4) == 1
    hidden[mask] = big[mask]
    for k in (10, 40_000, 1_000_000):
        th, cnt = gpu_threshold(hidden, k)
        rth, rcnt = orc.topk_threshold_exact(hidden, k, method="partition")
        assert np.float32(th).view(np.uint32) == np.float32(rth).view(np.uint32) and cnt == rcnt
    # heavy ties around rank k inside a long vector
    tied = lap(8, n)
    tied[100_000:400_000] = np.float32(3e-3)
    above = int((np.abs(tied) > np.float32(3e-3)).sum())
    th, cnt = gpu_threshold(tied, above + 1000)
    assert th == np.float32(3e-3) and cnt == int((np.abs(tied) >= np.float32(3e-3)).sum())


def test_threshold_small_workspace_same_result():
    acc = lap(17, 500_000)
    assert gpu_threshold(acc, 5000, ws_bytes=64 * 1024) == gpu_threshold(acc, 5000)


# ---------------------------------------------------------------------- select
def gpu_select(acc, th, capacity):
    d = to_dev(acc)
    d_th = to_dev(np.array([th], dtype=np.float32))
    idx = torch.full((max(capacity, 1),), -1, dtype=torch.int32, device=DEV)
    val = torch.zeros(max(capacity, 1), dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(max(acc.size, 1), 0))
    okt.okt_threshold_select(d, d_th, idx, val, nnz, ws, capacity=capacity)
    c = u64(nnz)
    e = int(c[0])
    w = min(e, capacity)          # e is UINT64_MAX when a call reports a failed wait
    return u32(idx[:w]), val[:w].cpu().numpy(), d.cpu().numpy(), e, int(c[1])


def check_select(acc, th, capacity):
    idx, val, res, emitted, total = gpu_select(acc, th, capacity)
    ridx, rval, rres, rtotal = orc.threshold_select(acc, th, capacity=capacity)
    assert total == rtotal and emitted == ridx.size
    assert np.array_equal(idx, ridx)
    assert bits_equal(val, rval)
    assert bits_equal(res, rres)
    return total


@pytest.mark.usefixtures("select_form")
@pytest.mark.parametrize("n", [1, 2, 4095, 4096, 4097, 3 * 4096 + 5, 1_000_003, (1 << 22) + 1])
def test_select_matches_oracle(n):
    acc = lap(n + 50, n)
    k = max(1, n // 100)
    th, cnt = orc.topk_threshold_exact(acc, k)
    assert check_select(acc, th, 4 * k) == cnt


@pytest.mark.usefixtures("select_form")
@pytest.mark.parametrize("n", [70_001, 5_000_003])
def test_threshold_and_select_with_nan_and_inf_elements(n):
    """Not a case the method meets (gradients are finite), but the order of the
    magnitude keys is defined for every bit pattern - Inf above finite, NaN above
    Inf - and both sides must follow it: NaNs of either sign and any payload are
    the largest elements, copied bit for bit; the k-th largest may itself be an
    Inf or a NaN (then the select compares keys, not floats).  n covers the
    three-pass and the sample-then-count path of the threshold."""
    rng = np.random.default_rng(n)
    acc = lap(n + 1, n)
    bits = acc.view(np.uint32)
    where = rng.choice(n, 160, replace=False)
    bits[where[:100]] = (np.uint32(0x7F800001) + rng.integers(0, 0x7FFFFE, 100).astype(np.uint32)) \
        | (rng.integers(0, 2, 100).astype(np.uint32) << np.uint32(31))          # NaNs
    bits[where[100:]] = np.where(rng.integers(0, 2, 60) == 1, 0xFF800000, 0x7F800000).astype(np.uint32)  # +-Inf
    assert np.isnan(acc).sum() == 100 and np.isinf(acc).sum() == 60
    for k in (1, 37, 100, 101, 160, 161, 5000):
        th, cnt = gpu_threshold(acc, k)
        rth, rcnt = orc.topk_threshold_exact(acc, k, method="partition")
        assert np.float32(th).view(np.uint32) == np.float32(rth).view(np.uint32) and cnt == rcnt, k
        assert check_select(acc, rth, cnt + 3) == cnt


@pytest.mark.usefixtures("select_form")
def test_select_degenerate_thresholds():
    acc = lap(99, 50_001)
    assert check_select(acc, np.float32(np.inf), 16) == 0
    assert check_select(acc, np.float32(0.0), acc.size) == acc.size      # dense: selects all
    assert check_select(acc, np.float32(-1e-3), acc.size) == check_select(acc, np.float32(1e-3), acc.size)
    acc[:] = 0.5
    assert check_select(acc, np.float32(0.5), acc.size) == acc.size


@pytest.mark.usefixtures("select_form")
def test_select_truncates_in_index_order():
    acc = lap(98, 300_000)
    total = check_select(acc, np.float32(1e-3), 1000)
    assert total > 1000
    check_select(acc, np.float32(1e-3), 0)
    check_select(acc, np.float32(1e-3), total)
    check_select(acc, np.float32(1e-3), total - 1)


@pytest.mark.usefixtures("select_form")
def test_select_empty_vector():
    nnz = torch.full((2,), 5, dtype=torch.int64, device=DEV)
    acc = torch.zeros(1, dtype=torch.float32, device=DEV)
    okt.okt_threshold_select(acc[:0], acc, acc.view(torch.int32), acc, nnz, workspace(256), capacity=0)
    assert list(u64(nnz)) == [0, 0]


@pytest.mark.usefixtures("select_form")
def test_select_is_deterministic():
    acc = lap(97, 2_000_000)
    a = gpu_select(acc, np.float32(2e-3), 100_000)
    b = gpu_select(acc, np.float32(2e-3), 100_000)
    assert all(np.array_equal(x, y) for x, y in zip(a[:3], b[:3])) and a[3:] == b[3:]


# ------------------------------------------------------- accumulate + select
def check_fused(g, e, lr, th, capacity):
    d_e = to_dev(e) if e.size else torch.zeros(1, dtype=torch.float32, device=DEV)[:0]
    d_g = to_dev(g) if g.size else torch.zeros(1, dtype=torch.float32, device=DEV)[:0]
    d_th = to_dev(np.array([th], dtype=np.float32))
    idx = torch.full((max(capacity, 1),), -1, dtype=torch.int32, device=DEV)
    val = torch.zeros(max(capacity, 1), dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(max(g.size, 1), 0))
    okt.okt_accumulate_select(d_g, d_e, lr, d_th, idx, val, nnz, ws, capacity=capacity)
    c = u64(nnz)
    acc = orc.residual_accumulate(g, e, lr)
    ridx, rval, rres, rtotal = orc.threshold_select(acc, th, capacity=capacity)
    assert (int(c[0]), int(c[1])) == (ridx.size, rtotal)
    assert np.array_equal(u32(idx[:ridx.size]), ridx)
    assert bits_equal(val[:ridx.size].cpu().numpy(), rval)
    assert bits_equal(d_e.cpu().numpy(), rres)
    assert bits_equal(d_g.cpu().numpy(), g)          # the gradient is read only
    return rtotal


@pytest.mark.usefixtures("select_form")
@pytest.mark.parametrize("n", [0, 1, 3, 1023, 4096, 4097, 70_001, 1_000_003, (1 << 22) + 5])
def test_accumulate_select_matches_the_two_calls(n):
    g, e = lap(n + 3, n), lap(n + 4, n, 2e-3)
    e[::5] = 0
    lr = 0.25
    if n == 0:
        check_fused(g, e, lr, np.float32(1.0), 4)
        return
    acc = orc.residual_accumulate(g, e, lr)
    k = max(1, n // 100)
    th, cnt = orc.topk_threshold_exact(acc, k)
    assert check_fused(g, e, lr, th, 4 * k) == cnt


@pytest.mark.usefixtures("select_form")
def test_accumulate_select_degenerate_and_truncated():
    n = 300_007
    g, e = lap(1, n), lap(2, n, 3e-3)
    assert check_fused(g, e, 1.0, np.float32(np.inf), 8) == 0
    assert check_fused(g, e, 1.0, np.float32(0.0), n) == n          # everything selected
    assert check_fused(g, e, 1.0, np.float32(0.0), 1000) == n       # dense and truncated
    total = check_fused(g, e, 0.5, np.float32(2e-3), n)
    assert total > 5000
    check_fused(g, e, 0.5, np.float32(2e-3), 1000)                  # output full: entries put back
    check_fused(g, e, 0.5, np.float32(2e-3), 0)
    check_fused(g, e, 0.5, np.float32(-2e-3), total - 1)
    # not fused: lr*g rounds to 1 + 2^-11, which the residual cancels exactly
    gg = np.full(5000, 1.0 + 2.0 ** -12, dtype=np.float32)
    ee = np.full(5000, -(1.0 + 2.0 ** -11), dtype=np.float32)
    assert check_fused(gg, ee, 1.0 + 2.0 ** -12, np.float32(1e-30), 5000) == 0


# ---------------------------------------------- selection that is dense in places
def layered(n, seed=5):
    """A vector whose selection is locally dense, as a real gradient's is: a third
    far above a threshold of 1 (84 % selected), a third far below (none), a third
    around it (32 %: some pieces overflow their stash part-way, some do not)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(n).astype(np.float32)
    x[: n // 3] *= 5.0
    x[n // 3: 2 * (n // 3)] *= 0.1
    return x


@pytest.mark.usefixtures("select_form")
@pytest.mark.timeout(300)
def test_calls_captured_in_a_hip_graph_replay_like_eager():
    """The entry points enqueue kernels only (the scan state is cleared by a small
    kernel, not a memset), so a sequence of them can be captured once and
    replayed.  Every replay - with eager work and synchronisations in between - is
    checked against the oracle, which follows the carried residual."""
    n, lr, R, rounds = 1_000_003, 0.5, 8, 4
    th = np.float32(3e-3)
    grads = [lap(300 + r, n) for r in range(rounds)]
    d_g = to_dev(grads[0])
    res = torch.zeros(n, dtype=torch.float32, device=DEV)
    d_th = to_dev(np.array([th], dtype=np.float32))
    cap = n // 4
    idx = torch.full((cap,), -1, dtype=torch.int32, device=DEV)
    val = torch.zeros(cap, dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    b = torch.zeros(R + 1, dtype=torch.int32, device=DEV)
    off = torch.zeros(R + 1, dtype=torch.int64, device=DEV)
    lo, hi = 100_000, 400_000
    cidx, cval, coff = wl.contributions(wl.WORKLOADS["cfg3"], lo, hi, m=3_000, P=8)
    d_ci, d_cv, d_co = to_dev(cidx), to_dev(cval), to_dev(coff)
    out_idx = torch.full((cidx.size,), -1, dtype=torch.int32, device=DEV)
    out_val = torch.zeros(cidx.size, dtype=torch.float32, device=DEV)
    out_nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(n, 8))
    ws2 = workspace(okt.okt_workspace_bytes(hi - lo, 8))
    okt.load_library()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        okt.okt_accumulate_select(d_g, res, lr, d_th, idx, val, nnz, ws, capacity=cap)
        okt.okt_region_partition(idx, nnz, n, R, b, off)
        okt.okt_sparse_reduce(d_ci, d_cv, d_co, lo, hi, out_idx, out_val, out_nnz, ws2)
    res.zero_()                                    # capture does not run anything; start clean anyway
    ref_red = orc.sparse_reduce(cidx, cval, coff, lo, hi)
    host_res = np.zeros(n, dtype=np.float32)
    for r in range(rounds):
        d_g.copy_(torch.from_numpy(grads[r]))      # eager work between the replays
        out_val.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        acc = orc.residual_accumulate(grads[r], host_res, lr)
        ridx, rval, host_res, total = orc.threshold_select(acc, th, capacity=cap)
        c = u64(nnz)
        assert (int(c[0]), int(c[1])) == (ridx.size, total), r
        assert np.array_equal(u32(idx[:total]), ridx) and bits_equal(val[:total].cpu().numpy(), rval), r
        assert bits_equal(res.cpu().numpy(), host_res), r
        rb, roff = orc.region_partition(ridx, n, R)
        assert np.array_equal(u32(b), rb) and np.array_equal(u64(off), roff), r
        U = ref_red["idx"].size
        assert int(u64(out_nnz)[1]) == U and np.array_equal(u32(out_idx[:U]), ref_red["idx"]), r
        err = np.abs(out_val[:U].cpu().numpy().astype(np.float64) - ref_red["val"].astype(np.float64))
        assert np.all(err <= reduce_tolerance(ref_red)), r


def test_two_host_threads_call_the_library_at_once():
    """The entry points keep no shared mutable state (the measurement hook and the
    last HIP error are per thread), so host threads with their own streams,
    buffers and workspaces may call them at the same time."""
    import threading
    n, lr, rounds = 1_500_011, 0.5, 6
    results, errors = {}, []

    def worker(j):
        try:
            st = torch.cuda.Stream()
            g = [lap(700 + 10 * j + r, n) for r in range(rounds)]
            th = np.float32(3e-3 + 1e-3 * j)
            with torch.cuda.stream(st):
                d_g = [to_dev(x) for x in g]
                res = torch.zeros(n, dtype=torch.float32, device=DEV)
                d_th = to_dev(np.array([th], dtype=np.float32))
                idx = [torch.full((n // 8,), -1, dtype=torch.int32, device=DEV) for _ in range(rounds)]
                val = [torch.zeros(n // 8, dtype=torch.float32, device=DEV) for _ in range(rounds)]
                nnz = [torch.zeros(2, dtype=torch.int64, device=DEV) for _ in range(rounds)]
                ws = workspace(okt.okt_workspace_bytes(n, 0))
                for r in range(rounds):
                    if (r + j) % 2:
                        okt.okt_accumulate_select(d_g[r], res, lr, d_th, idx[r], val[r], nnz[r], ws)
                    else:
                        okt.okt_residual_accumulate(d_g[r], res, lr)
                        okt.okt_threshold_select(res, d_th, idx[r], val[r], nnz[r], ws)
            st.synchronize()
            results[j] = (g, th, res.cpu().numpy(), [u32(t) for t in idx],
                          [t.cpu().numpy() for t in val], [u64(t) for t in nnz])
        except Exception as e:          # surfaces in the main thread below
            errors.append((j, repr(e)))

    threads = [threading.Thread(target=worker, args=(j,)) for j in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for j in range(2):
        g, th, res_gpu, idx, val, nnz = results[j]
        res = np.zeros(n, dtype=np.float32)
        for r in range(rounds):
            acc = orc.residual_accumulate(g[r], res, lr)
            ridx, rval, res, total = orc.threshold_select(acc, th, capacity=n // 8)
            assert (int(nnz[r][0]), int(nnz[r][1])) == (ridx.size, total), (j, r)
            assert np.array_equal(idx[r][:total], ridx) and bits_equal(val[r][:total], rval), (j, r)
        assert bits_equal(res_gpu, res), j


def test_a_wait_that_gives_up_is_reported():
    """Failure handling of the scan across workgroups, forced from the host: with
    the test hook's limit of one poll, a workgroup that finds a predecessor's
    count not yet published gives up at once.  Every kernel still runs to its
    end; a call either completes as usual or reports UINT64_MAX counts - never a
    wrong result with valid counts - and the next call with the built-in limit
    is right again."""
    n = 30_000_011
    acc = lap(500, n)
    th = np.float32(5e-3)
    ridx, rval, rres, total = orc.threshold_select(acc, th, capacity=n // 8)
    lo, hi = 0, 2_000_000
    cidx, cval, coff = wl.contributions(wl.WORKLOADS["cfg2"], lo, hi, m=20_000, P=16)
    ref = orc.sparse_reduce(cidx, cval, coff, lo, hi)
    bad = np.uint64(0xFFFFFFFFFFFFFFFF)
    outcomes = []
    try:
        okt.okt_debug_spin_limit(1)
        for rep in range(3):
            idx, val, res, e, t = gpu_select(acc, th, n // 8)
            if t == int(bad):
                outcomes.append("select gave up")
                assert e == int(bad)
            else:
                outcomes.append("select completed")
                assert (e, t) == (ridx.size, total) and np.array_equal(idx, ridx)
                assert bits_equal(val, rval) and bits_equal(res, rres)
            got = gpu_reduce(cidx, cval, coff, lo, hi, dense=False)
            if got["total"] == int(bad):
                outcomes.append("reduce gave up")
            else:
                outcomes.append("reduce completed")
                assert got["total"] == ref["idx"].size and np.array_equal(got["idx"], ref["idx"])
    finally:
        okt.okt_debug_spin_limit(0)
    print(outcomes, flush=True)
    idx, val, res, e, t = gpu_select(acc, th, n // 8)
    assert (e, t) == (ridx.size, total) and np.array_equal(idx, ridx) and bits_equal(res, rres)
    got = gpu_reduce(cidx, cval, coff, lo, hi, dense=False)
    assert got["total"] == ref["idx"].size and np.array_equal(got["idx"], ref["idx"])


@pytest.mark.usefixtures("select_form")
def test_two_streams_each_with_its_own_workspace():
    """Calls enqueued on two streams, each with its own workspace and outputs, run
    side by side without a synchronisation between them: the library keeps no
    state of its own between calls, so neither disturbs the other."""
    n, lr, rounds = 3_000_017, 0.75, 4
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    lanes = []
    for j, st in enumerate(streams):
        g = [lap(100 + 10 * j + r, n) for r in range(rounds)]
        th = np.float32(4e-3 + 1e-3 * j)
        lanes.append({
            "g": g, "th": th, "d_g": [to_dev(x) for x in g],
            "res": torch.zeros(n, dtype=torch.float32, device=DEV),
            "d_th": to_dev(np.array([th], dtype=np.float32)),
            "idx": [torch.full((n // 8,), -1, dtype=torch.int32, device=DEV) for _ in range(rounds)],
            "val": [torch.zeros(n // 8, dtype=torch.float32, device=DEV) for _ in range(rounds)],
            "nnz": [torch.zeros(2, dtype=torch.int64, device=DEV) for _ in range(rounds)],
            "ws": workspace(okt.okt_workspace_bytes(n, 0))})
    torch.cuda.synchronize()
    for r in range(rounds):
        for j, st in enumerate(streams):
            L = lanes[j]
            if (r + j) % 2:         # one stream takes the fused call while the other takes two
                okt.okt_accumulate_select(L["d_g"][r], L["res"], lr, L["d_th"], L["idx"][r],
                                          L["val"][r], L["nnz"][r], L["ws"], stream=st)
            else:
                okt.okt_residual_accumulate(L["d_g"][r], L["res"], lr, stream=st)
                okt.okt_threshold_select(L["res"], L["d_th"], L["idx"][r], L["val"][r],
                                         L["nnz"][r], L["ws"], stream=st)
    torch.cuda.synchronize()
    for j, L in enumerate(lanes):
        res = np.zeros(n, dtype=np.float32)
        for r in range(rounds):
            acc = orc.residual_accumulate(L["g"][r], res, lr)
            ridx, rval, res, total = orc.threshold_select(acc, L["th"], capacity=n // 8)
            c = u64(L["nnz"][r])
            assert (int(c[0]), int(c[1])) == (ridx.size, total), (j, r)
            assert np.array_equal(u32(L["idx"][r][:total]), ridx), (j, r)
            assert bits_equal(L["val"][r][:total].cpu().numpy(), rval), (j, r)
        assert bits_equal(L["res"].cpu().numpy(), res), j


@pytest.mark.usefixtures("select_form")
def test_select_where_pieces_overflow_their_stash():
    # long enough that a wave's piece (about n / 4096) holds more selected entries
    # than its stash where the selection is dense
    n = 12_000_003
    acc = layered(n)
    one = np.float32(1.0)
    total = check_select(acc, one, n)
    assert 0.35 * n < total < 0.45 * n
    for cap in (1000, total // 5, total // 2 + 3, total - 1):
        check_select(acc, one, cap)                  # the output fills up at various places
    assert check_select(acc, np.float32(0.0), n) == n
    # the same selection without the zeroing, and over a COO of the same length
    d_acc, d_th = to_dev(acc), to_dev(np.array([1.0], dtype=np.float32))
    ridx, rval, _, _ = orc.threshold_select(acc, one)
    idx = torch.full((total,), -1, dtype=torch.int32, device=DEV)
    val = torch.zeros(total, dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(n, 0))
    okt.okt_threshold_select_copy(d_acc, d_th, idx, val, nnz, ws)
    assert tuple(u64(nnz)) == (total, total)
    assert np.array_equal(u32(idx), ridx) and bits_equal(val.cpu().numpy(), rval)
    assert bits_equal(d_acc.cpu().numpy(), acc)
    coo_idx = (np.arange(n, dtype=np.uint64) * 3 + 7).astype(np.uint32)
    idx.fill_(-1)
    okt.okt_coo_threshold_select(to_dev(coo_idx), d_acc, to_dev(np.array([n], dtype=np.uint64)), d_th,
                                 idx, val, nnz, ws)
    assert tuple(u64(nnz)) == (total, total)
    assert np.array_equal(u32(idx), coo_idx[ridx]) and bits_equal(val.cpu().numpy(), rval)


@pytest.mark.usefixtures("select_form")
@pytest.mark.timeout(300)
def test_accumulate_select_where_pieces_overflow_their_stash():
    n = 12_000_003
    acc = layered(n, seed=6)
    g = lap(7, n, 0.3)
    e = (acc - g * np.float32(0.5)).astype(np.float32)      # eps + 0.5 g is near `acc`, layered alike
    total = check_fused(g, e, 0.5, np.float32(1.0), n)
    assert 0.3 * n < total < 0.5 * n
    for cap in (1000, total // 3 + 1, total - 1):
        check_fused(g, e, 0.5, np.float32(1.0), cap)
    assert check_fused(g, e, 0.5, np.float32(0.0), n) == n


# ------------------------------------------------------------------- partition
def gpu_partition(idx, n, R):
    d_idx = to_dev(idx) if idx.size else torch.zeros(1, dtype=torch.int32, device=DEV)
    nnz = to_dev(np.array([idx.size, idx.size], dtype=np.uint64))
    b = torch.full((R + 1,), -1, dtype=torch.int32, device=DEV)
    off = torch.full((R + 1,), -1, dtype=torch.int64, device=DEV)
    okt.okt_region_partition(d_idx, nnz, n, R, b, off)
    return u32(b), u64(off)


@pytest.mark.parametrize("nnz,R", [(0, 8), (1, 1), (5, 8), (64, 64), (1000, 4), (10_486, 4),
                                   (255_571, 16), (336_000, 64), (100_000, 256), (999, 1000)])
def test_partition_matches_oracle(nnz, R):
    n = 3_000_000
    rng = np.random.default_rng(nnz + R)
    idx = np.sort(rng.choice(n, nnz, replace=False)).astype(np.uint32)
    b, off = gpu_partition(idx, n, R)
    rb, roff = orc.region_partition(idx, n, R)
    assert np.array_equal(b, rb) and np.array_equal(off, roff)


def test_partition_clustered_indices_and_top_of_index_space():
    n = (1 << 32) - 1
    idx = np.sort(np.random.default_rng(5).choice(1 << 20, 50_000, replace=False)).astype(np.uint32)
    idx[-100:] = np.arange(n - 100, n, dtype=np.uint64).astype(np.uint32)
    b, off = gpu_partition(idx, n, 32)
    rb, roff = orc.region_partition(idx, n, 32)
    assert np.array_equal(b, rb) and np.array_equal(off, roff)
    assert set(np.diff(off.astype(np.int64))) <= {50_000 // 32, 50_000 // 32 + 1}


# ---------------------------------------------------------------------- reduce
def check_reduce(idx_cat, val_cat, off, lo, hi, capacity=None):
    got = gpu_reduce(idx_cat, val_cat, off, lo, hi, capacity=capacity)
    ref = orc.sparse_reduce(idx_cat, val_cat, off, lo, hi)
    U = ref["idx"].size
    assert got["total"] == U
    e = U if capacity is None else min(U, capacity)
    assert got["emitted"] == e
    assert np.array_equal(got["idx"], ref["idx"][:e])
    tol = reduce_tolerance(ref)
    err = np.abs(got["val"].astype(np.float64) - ref["val"][:e].astype(np.float64))
    assert np.all(err <= tol[:e]), float((err / np.maximum(tol[:e], 1e-300)).max())
    dense_tol = np.zeros(hi - lo)
    dense_tol[ref["idx"].astype(np.int64) - lo] = tol
    derr = np.abs(got["dense"].astype(np.float64) - ref["dense"].astype(np.float64))
    assert np.all(derr <= dense_tol)
    absent = np.ones(hi - lo, dtype=bool)
    absent[ref["idx"].astype(np.int64) - lo] = False
    assert not got["dense"][absent].view(np.uint32).any()        # +0.0f where nothing landed
    return got, ref


REDUCE_CASES = [
    # name, lo, hi, m, P   (several tiles of 4096 slots and a ragged last tile)
    ("cfg1", 0, 262_144, 700, 4),
    ("cfg2", 1_597_314, 1_597_314 + 150_001, 1_500, 16),
    ("cfg3", 3_437_500, 3_437_500 + 120_007, 1_200, 32),
    ("cfg4", 100, 100 + 400_003, 400, 64),
    ("cfg5", 55_000_064, 55_000_064 + 30_001, 300, 256),
    # the top of the 32-bit index space: hi = 2^32 - 1, overlapping draws
    ("cfg3", (1 << 32) - 1 - 300_001, (1 << 32) - 1, 2_000, 8),
]


@pytest.mark.parametrize("name,lo,hi,m,P", REDUCE_CASES)
def test_reduce_scaled_configurations(name, lo, hi, m, P):
    idx, val, off = wl.contributions(wl.WORKLOADS[name], lo, hi, m=m, P=P)
    check_reduce(idx, val, off, lo, hi)


def test_reduce_whole_space_chunks_one_region():
    w = wl.WORKLOADS["cfg1"]            # the literal first configuration
    idx, val, off = wl.whole_space_contributions(w)
    got, ref = check_reduce(idx, val, off, 0, w.n // 4)
    assert 2000 < got["total"] <= 4 * 700


def test_reduce_special_cases():
    rng = np.random.default_rng(8)
    n = 20_000
    idx = np.sort(rng.choice(n, 3000, replace=False)).astype(np.uint32)
    val = lap(9, 3000)
    one = np.array([0, 3000], dtype=np.uint64)
    # P = 1: the slice comes back bit for bit
    got, _ = check_reduce(idx, val, one, 5000, 15_000)
    inside = (idx >= 5000) & (idx < 15_000)
    assert bits_equal(got["val"], val[inside])
    # a contribution and its negation: structural zeros stay
    two = np.array([0, 3000, 6000], dtype=np.uint64)
    got, _ = check_reduce(np.tile(idx, 2), np.concatenate([val, -val]), two, 0, n)
    assert got["total"] == 3000 and not got["val"].any()
    # identical supports
    got, _ = check_reduce(np.tile(idx, 3), np.tile(val, 3), np.array([0, 3000, 6000, 9000], np.uint64), 0, n)
    assert got["total"] == 3000
    # empty region, region without entries, empty contributions, truncation
    check_reduce(idx, val, one, 7000, 7000)
    check_reduce(idx[:0], val[:0], np.zeros(5, np.uint64), 0, 5000)
    check_reduce(idx, val, np.array([0, 0, 3000, 3000], np.uint64), 0, n)
    check_reduce(idx, val, one, 0, n, capacity=100)
    check_reduce(idx, val, one, 0, n, capacity=0)


def test_reduce_tile_modes():
    """Wide tiles with accumulators indexed by rank (sparse regions), narrow
    tiles with accumulator = slot (dense regions), and the several-rounds path
    taken when a wide tile turns out to hold more hit slots than accumulators."""
    rng = np.random.default_rng(77)
    # every slot of a 40,000 wide region hit by each of three contributions
    idx = np.arange(1000, 41_000, dtype=np.uint32)
    vals = [lap(70 + p, idx.size) for p in range(3)]
    off = np.arange(4, dtype=np.uint64) * idx.size
    cat_i, cat_v = np.tile(idx, 3), np.concatenate(vals)
    got, _ = check_reduce(cat_i, cat_v, off, 1000, 41_000)               # dense estimate
    assert got["total"] == 40_000
    got, _ = check_reduce(cat_i, cat_v, off, 1000, 41_000, capacity=50)  # sparse estimate, dense data
    assert got["total"] == 40_000 and got["emitted"] == 50
    got, _ = check_reduce(cat_i, cat_v, off, 500, 70_001, capacity=50)
    # a sparse region: 3,000 entries over 900,001 slots
    sp = np.sort(rng.choice(900_001, 1000, replace=False)).astype(np.uint32) + np.uint32(123)
    parts = [sp, np.sort(rng.choice(900_001, 1000, replace=False)).astype(np.uint32) + np.uint32(123), sp]
    sv = [lap(80 + p, 1000) for p in range(3)]
    got, ref = check_reduce(np.concatenate(parts), np.concatenate(sv),
                            np.arange(4, dtype=np.uint64) * 1000, 123, 900_124)
    assert 1000 < got["total"] <= 2000
    # clustered entries inside a region estimated sparse: one tile overflows its accumulators
    cl = np.concatenate([np.arange(200_000, 209_000), rng.choice(800_000, 500, replace=False) + 300_000])
    cl = np.sort(np.unique(cl)).astype(np.uint32)
    got, _ = check_reduce(cl, lap(90, cl.size), np.array([0, cl.size], np.uint64), 0, 1_200_000)
    assert got["total"] == cl.size


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_reduce_more_contributions_than_one_sweep_over_ranked_tiles(seed):
    """300 contributions (more than the 256 a sweep takes at a time) over a
    region wide enough for ranked tiles, most slices of a tile empty: every
    pass over the entries reloads the slice table twice, and a wave with nothing
    to do in the first part runs far ahead of the others."""
    rng = np.random.default_rng(1000 + seed)
    width, P = 700_000, 300
    lo = int(rng.integers(0, (1 << 32) - 1 - width))
    parts = []
    for p in range(P):
        m = int(rng.integers(0, 4001))
        mode = p % 3
        if m == 0:
            loc = np.zeros(0, np.int64)
        elif mode == 0:
            loc = np.sort(rng.choice(width, m, replace=False))
        elif mode == 1:                                   # clustered: empty slices elsewhere
            a = int(rng.integers(0, width - 2 * m))
            loc = np.sort(rng.choice(2 * m, m, replace=False)) + a
        else:                                             # shared support: collisions
            loc = np.sort(np.random.default_rng(7).choice(width, m, replace=False))
        parts.append((loc + lo).astype(np.uint32))
    cat_i = np.concatenate(parts)
    cat_v = lap(600 + seed, cat_i.size)
    off = np.concatenate([[0], np.cumsum([x.size for x in parts])]).astype(np.uint64)
    got, ref = check_reduce(cat_i, cat_v, off, lo, lo + width)
    assert ref["hits"].max() > 8 and got["total"] > 300_000


@pytest.mark.parametrize("want", [30_000, 32_768, 33_000, 34_900, 35_100, 40_000, 49_000, 49_152, 60_000, 400_000])
def test_reduce_tile_shapes_around_the_switch_to_the_sparse_shape(want):
    """The capacity steers the tile width (about `want` slots here): up to 32,768
    slots with 4,096 accumulators, beyond that the sparse shape of the kernel, up
    to 49,152 slots with 3,840 accumulators.  Same result from every shape."""
    width, P = 1_000_003, 8
    cap = int(0.9 * 4096 * width / want)
    rng = np.random.default_rng(want)
    m = max(cap // P - 3, 1)
    parts = [np.sort(rng.choice(width, m, replace=False)).astype(np.uint32) + np.uint32(1234) for _ in range(P)]
    parts[3] = parts[0]                                   # one support twice: collisions
    cat_i = np.concatenate(parts)
    cat_v = lap(want, cat_i.size)
    off = np.arange(P + 1, dtype=np.uint64) * m
    got, ref = check_reduce(cat_i, cat_v, off, 1234, 1234 + width, capacity=cap)
    assert got["total"] == ref["idx"].size <= cap


def test_reduce_paper_shaped_regions():
    """The shapes of the paper's runs (16 .. 64 contributions hitting 6 .. 30 % of a
    region) and what can go wrong around them, steered by the density estimate
    (the capacity) and the data: identical supports (many entries per hit slot),
    more hit slots than accumulators (several rounds), accumulator = slot, tile
    widths that are no power of two and end inside a 32-slot bitmap word, empty
    tiles between full ones, empty contributions, a region of one slot."""
    rng = np.random.default_rng(123)
    # 16 contributions, 16 % of the slots hit: the shape of a ResNet-sized run
    width, P, m = 100_003, 16, 1000
    parts = [np.sort(rng.choice(width, m, replace=False)).astype(np.uint32) + np.uint32(77) for _ in range(P)]
    cat_i = np.concatenate(parts)
    cat_v = lap(500, cat_i.size)
    off = np.arange(P + 1, dtype=np.uint64) * m
    got, ref = check_reduce(cat_i, cat_v, off, 77, 77 + width)
    assert ref["hits"].max() >= 2
    check_reduce(cat_i, cat_v, off, 77, 77 + width, capacity=P * m // 3)   # truncated output
    check_reduce(cat_i, cat_v, off, 5077, 60_001)                       # entries outside the region
    # every contribution has the same support: 12 x the entries a tile's registers hold
    same = np.sort(rng.choice(60_000, 6000, replace=False)).astype(np.uint32)
    cat_i = np.tile(same, 12)
    cat_v = lap(501, cat_i.size)
    off = np.arange(13, dtype=np.uint64) * same.size
    got, ref = check_reduce(cat_i, cat_v, off, 0, 60_000, capacity=6000)
    assert got["total"] == 6000 and ref["hits"].min() == 12
    # estimated sparse (wide ranked tiles), in fact every slot hit: 16 rounds per tile
    full = np.arange(300, 50_300, dtype=np.uint32)
    cat_i = np.tile(full, 3)
    cat_v = lap(502, cat_i.size)
    off = np.arange(4, dtype=np.uint64) * full.size
    got, _ = check_reduce(cat_i, cat_v, off, 300, 50_300, capacity=2500)
    assert got["total"] == 50_000 and got["emitted"] == 2500
    check_reduce(cat_i, cat_v, off, 0, 70_001, capacity=70_001)         # accumulator = slot
    # a cluster and a desert in one region
    cl = np.unique(np.concatenate([np.arange(20_000, 23_000), rng.choice(400_000, 30_000, replace=False)]))
    cl = cl.astype(np.uint32)
    cl = cl[(cl < 100_000) | (cl > 200_000)]
    two = [cl, cl[::3]]
    cat_i = np.concatenate(two)
    got, _ = check_reduce(cat_i, lap(503, cat_i.size), np.array([0, cl.size, cat_i.size], np.uint64),
                          0, 400_000)
    assert got["total"] == cl.size
    # 64 and 65 contributions take different kernels and must agree with the oracle alike
    for P in (64, 65):
        parts = [np.sort(rng.choice(80_000, 300, replace=False)).astype(np.uint32) for _ in range(P)]
        cat_i = np.concatenate(parts)
        check_reduce(cat_i, lap(504 + P, cat_i.size), np.arange(P + 1, dtype=np.uint64) * 300, 0, 80_000)
    # empty contributions among the 64, a single entry, a region of one slot
    lens = np.array([0, 5, 0, 0, 700, 0, 1] + [0] * 57)
    parts = [np.sort(rng.choice(9000, n, replace=False)).astype(np.uint32) for n in lens]
    cat_i = np.concatenate(parts)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)
    check_reduce(cat_i, lap(600, cat_i.size), off, 0, 9000)
    check_reduce(cat_i, lap(600, cat_i.size), off, int(cat_i[5]), int(cat_i[5]) + 1)


def test_reduce_segments_in_any_order():
    rng = np.random.default_rng(31)
    n, m = 50_000, 900
    parts = [np.sort(rng.choice(n, m - 100 * p, replace=False)).astype(np.uint32) for p in range(5)]
    vals = [lap(40 + p, parts[p].size) for p in range(5)]
    # the buffer holds the contributions out of order, with gaps, and one slice
    # whose end lies below its begin (empty)
    order, gap = [3, 0, 4, 1, 2], 37
    begin, end = [0] * 6, [0] * 6
    buf_i, buf_v, at = [], [], 11
    buf_i.append(np.full(at, 0xFFFFFFFF, np.uint32)); buf_v.append(np.full(at, 9e9, np.float32))
    for p in order:
        begin[p], end[p] = at, at + parts[p].size
        buf_i += [parts[p], np.full(gap, 0xFFFFFFFF, np.uint32)]
        buf_v += [vals[p], np.full(gap, 9e9, np.float32)]
        at += parts[p].size + gap
    begin[5], end[5] = 500, 400
    cat_i, cat_v = np.concatenate(buf_i), np.concatenate(buf_v)
    ref = orc.sparse_reduce(np.concatenate(parts), np.concatenate(vals),
                            np.concatenate([[0], np.cumsum([q.size for q in parts])]).astype(np.uint64),
                            1000, 45_001)
    U = ref["idx"].size
    out_i = torch.full((U + 5,), -1, dtype=torch.int32, device=DEV)
    out_v = torch.zeros(U + 5, dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(44_001, 6))
    okt.okt_sparse_reduce_segments(to_dev(cat_i), to_dev(cat_v), to_dev(np.array(begin, np.uint64)),
                                   to_dev(np.array(end, np.uint64)), 6, 1000, 45_001, out_i, out_v,
                                   nnz, ws)
    c = u64(nnz)
    assert int(c[0]) == int(c[1]) == U
    assert np.array_equal(u32(out_i[:U]), ref["idx"])
    err = np.abs(out_v[:U].cpu().numpy().astype(np.float64) - ref["val"])
    assert np.all(err <= reduce_tolerance(ref))


@pytest.mark.parametrize("exact", [True, False])
def test_reduce_in_buckets_with_carried_partial(exact):
    """Three buckets of four contributions; the partial result is the last slice of
    the next call and is never copied: two buffers in turn, the count written
    straight into the end word of that slice."""
    rng = np.random.default_rng(32)
    lo, hi, m, per, nb = 5000, 205_000, 3000, 4, 3
    cap = per * nb * m
    buckets = []
    for b in range(nb):
        parts = [np.sort(rng.choice(hi - lo, m, replace=False)).astype(np.uint32) + np.uint32(lo)
                 for _ in range(per)]
        if exact:
            vals = [(rng.integers(-2048, 2049, m) / 128.0).astype(np.float32) for _ in range(per)]
        else:
            vals = [lap(900 + 10 * b + p, m) for p in range(per)]
        buckets.append((np.concatenate(parts), np.concatenate(vals), np.arange(per + 1, dtype=np.uint64) * m))
    ref = orc.sparse_reduce_bucketed(buckets, lo, hi)

    size = cap + per * m
    buf_i = [torch.zeros(size, dtype=torch.int32, device=DEV) for _ in range(2)]
    buf_v = [torch.zeros(size, dtype=torch.float32, device=DEV) for _ in range(2)]
    begin = to_dev(np.array([cap + p * m for p in range(per)] + [0], dtype=np.uint64))
    ends = [to_dev(np.array([cap + (p + 1) * m for p in range(per)] + [0, 0], dtype=np.uint64))
            for _ in range(2)]                       # [.., end of the carried slice, spare word]
    ws = workspace(okt.okt_workspace_bytes(hi - lo, per + 1))
    for b, (ci, cv, _) in enumerate(buckets):
        src, dst = b % 2, (b + 1) % 2
        buf_i[src][cap:] = to_dev(ci)                # "received" behind the carried partial
        buf_v[src][cap:] = to_dev(cv)
        okt.okt_sparse_reduce_segments(buf_i[src], buf_v[src], begin, ends[src], per + 1, lo, hi,
                                       buf_i[dst][:cap], buf_v[dst][:cap], ends[dst][per:per + 2], ws)
    torch.cuda.synchronize()
    final = nb % 2
    counts = u64(ends[final][per:per + 2])
    U = ref["idx"].size
    assert int(counts[0]) == int(counts[1]) == U
    assert np.array_equal(u32(buf_i[final][:U]), ref["idx"])
    got = buf_v[final][:U].cpu().numpy()
    if exact:
        assert bits_equal(got, ref["val"])
    else:
        # every call is within the stated tolerance of its own exact sums; over the
        # chain the bound is taken against the sum of all magnitudes, once per bucket
        one = orc.sparse_reduce(np.concatenate([b[0] for b in buckets]), np.concatenate([b[1] for b in buckets]),
                                np.arange(per * nb + 1, dtype=np.uint64) * m, lo, hi)
        err = np.abs(got.astype(np.float64) - ref["val"].astype(np.float64))
        assert np.all(err <= nb * 1e-6 * one["abs_sum"])


def test_reduce_disjoint_contributions_fill_in():
    # non-overlapping indexes: the union is the sum of the sizes and every value
    # is a bit copy (the fill-in arithmetic of the paper's Introduction)
    rng = np.random.default_rng(10)
    perm = rng.permutation(100_000)
    parts = [np.sort(perm[p * 2500:(p + 1) * 2500]).astype(np.uint32) for p in range(8)]
    vals = [lap(20 + p, 2500) for p in range(8)]
    off = np.arange(9, dtype=np.uint64) * 2500
    got, ref = check_reduce(np.concatenate(parts), np.concatenate(vals), off, 0, 100_000)
    assert got["total"] == 20_000
    assert bits_equal(got["val"], ref["val"])


def test_reduce_more_contributions_than_one_sweep():
    w = wl.WORKLOADS["cfg5"]
    idx, val, off = wl.contributions(w, 1000, 1000 + 9000, m=40, P=2500)
    got, ref = check_reduce(idx, val, off, 1000, 10_000)
    assert ref["hits"].max() > 1024


def test_reduce_batch_matches_single_regions():
    w = wl.WORKLOADS["cfg3"]
    B, P, width, m = 5, 12, 20_000, 900
    parts, offs, lohi = [], [], []
    base = 0
    for j in range(B):
        lo = 1_000_000 * j + 17
        hi = lo + width - 1000 * j            # regions of different widths
        idx, val, off = wl.contributions(w, lo, hi, m=m, P=P, stream=j)
        parts.append((idx, val))
        offs.append(off + np.uint64(base))
        lohi += [lo, hi]
        base += idx.size
    idx_cat = np.concatenate([p[0] for p in parts])
    val_cat = np.concatenate([p[1] for p in parts])
    cap = P * m
    out_idx = torch.full((B * cap,), -1, dtype=torch.int32, device=DEV)
    out_val = torch.zeros(B * cap, dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2 * B, dtype=torch.int64, device=DEV)
    dense = torch.full((B * width,), 3.0, dtype=torch.float32, device=DEV)
    ws = workspace(okt.okt_sparse_reduce_batch_workspace_bytes(B, P, width))
    okt.okt_sparse_reduce_batch(to_dev(idx_cat), to_dev(val_cat), to_dev(np.concatenate(offs)),
                                to_dev(np.array(lohi, dtype=np.uint32)), B, P, width,
                                out_idx, out_val, cap, nnz, ws, dense_out=dense)
    counts = u64(nnz)
    for j in range(B):
        lo, hi = lohi[2 * j], lohi[2 * j + 1]
        ref = orc.sparse_reduce(parts[j][0], parts[j][1], offs[j] - offs[j][0], lo, hi)
        U = ref["idx"].size
        assert counts[2 * j] == counts[2 * j + 1] == U
        assert np.array_equal(u32(out_idx[j * cap:j * cap + U]), ref["idx"])
        err = np.abs(out_val[j * cap:j * cap + U].cpu().numpy().astype(np.float64) - ref["val"])
        assert np.all(err <= reduce_tolerance(ref))
        d = dense[j * width:j * width + hi - lo].cpu().numpy()
        assert np.allclose(d, ref["dense"], rtol=1e-5, atol=1e-12)


def test_reduce_batch_with_clustered_contributions():
    """A launch with so many tile boundaries (more than 2^17) that the boundary
    search starts from a guess - the place a boundary would have if the indices
    were spread evenly - and brackets from there.  Here they are not spread
    evenly: clusters at either end of the region, two clusters, geometric
    spacing, entries outside the region on both sides, empty contributions."""
    rng = np.random.default_rng(123)
    B, P, width, m = 128, 32, 2_000_000, 300
    idx_parts, val_parts, offs, lohi = [], [], [0], []
    for j in range(B):
        lo = 4_000_000 * j + 1000
        hi = lo + width
        lohi += [lo, hi]
        for p in range(P):
            kind = (j + p) % 7
            if kind == 0:
                x = rng.choice(width, m, replace=False)
            elif kind == 1:
                x = rng.choice(width // 100, m, replace=False)                     # all at the start
            elif kind == 2:
                x = width - 1 - rng.choice(width // 100, m, replace=False)         # all at the end
            elif kind == 3:
                x = np.concatenate([rng.choice(5000, m // 2, replace=False) + width // 3,
                                    rng.choice(5000, m - m // 2, replace=False) + 2 * (width // 3)])
            elif kind == 4:
                x = np.unique((width * (1.0 - 0.97 ** np.arange(1, 4 * m))).astype(np.int64))[:m]
            elif kind == 5:                                                        # mostly outside the region
                x = np.concatenate([-1 - rng.choice(900, 100, replace=False),
                                    rng.choice(width, m - 200, replace=False),
                                    width + rng.choice(900, 100, replace=False)])
            else:
                x = np.zeros(0, dtype=np.int64)                                    # nothing at all
            x = np.sort(np.unique(x.astype(np.int64))) + lo
            idx_parts.append(x.astype(np.uint32))
            val_parts.append(rng.standard_normal(x.size).astype(np.float32))
            offs.append(offs[-1] + x.size)
        if j < B - 1:
            offs.append(offs[-1])               # the next region's first offset
    off = np.array(offs, dtype=np.uint64)
    assert off.size == B * (P + 1)
    idx_cat, val_cat = np.concatenate(idx_parts), np.concatenate(val_parts)
    cap = P * m
    out_idx = torch.full((B * cap,), -1, dtype=torch.int32, device=DEV)
    out_val = torch.zeros(B * cap, dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2 * B, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_sparse_reduce_batch_workspace_bytes(B, P, width))
    okt.okt_sparse_reduce_batch(to_dev(idx_cat), to_dev(val_cat), to_dev(off),
                                to_dev(np.array(lohi, dtype=np.uint32)), B, P, width,
                                out_idx, out_val, cap, nnz, ws)
    counts = u64(nnz)
    for j in range(B):
        lo, hi = lohi[2 * j], lohi[2 * j + 1]
        o = off[j * (P + 1):(j + 1) * (P + 1)]
        a, b = int(o[0]), int(o[-1])
        ref = orc.sparse_reduce(idx_cat[a:b], val_cat[a:b], o - o[0], lo, hi)
        U = ref["idx"].size
        assert counts[2 * j] == counts[2 * j + 1] == U, j
        assert np.array_equal(u32(out_idx[j * cap:j * cap + U]), ref["idx"]), j
        err = np.abs(out_val[j * cap:j * cap + U].cpu().numpy().astype(np.float64) - ref["val"])
        assert np.all(err <= reduce_tolerance(ref)), j


# ----------------------------------------------------------- the whole hot path
def run_loop(w, iterations, R, fused=False):
    """Alternate the GPU path and the oracle over `iterations` of Ok-Topk SGD's
    local part and compare every intermediate result bit for bit."""
    gpu = GpuPath(w.n, 4 * w.k)
    res = np.zeros(w.n, dtype=np.float32)
    th = None
    counts = []
    for it in range(iterations):
        g = wl.gradient(w, it)
        acc = orc.residual_accumulate(g, res, w.lr)
        if fused and not w.refresh(it):
            # reuse iteration: accumulate and select in one call
            okt.okt_accumulate_select(to_dev(g), gpu.residual, w.lr, gpu.th, gpu.idx, gpu.val,
                                      gpu.nnz, gpu.ws, capacity=gpu.capacity)
        else:
            gpu.accumulate(to_dev(g), w.lr)
            assert bits_equal(gpu.residual.cpu().numpy(), acc), f"acc it={it}"
            if w.refresh(it):
                gpu.threshold(w.k)
                th, cnt = orc.topk_threshold_exact(acc, w.k, method="partition")
                assert gpu.th.cpu().numpy().view(np.uint32)[0] == np.float32(th).view(np.uint32)
                assert int(u64(gpu.count_ge)[0]) == cnt
            gpu.select()
        ridx, rval, res, total = orc.threshold_select(acc, th, capacity=4 * w.k)
        idx, val, emitted, gtotal = gpu.selected()
        assert (emitted, gtotal) == (ridx.size, total), f"nnz it={it}"
        assert np.array_equal(idx, ridx) and bits_equal(val, rval), f"coo it={it}"
        assert bits_equal(gpu.residual.cpu().numpy(), res), f"residual it={it}"
        if w.refresh(it):
            assert total == cnt
        counts.append(total)
    b = torch.zeros(R + 1, dtype=torch.int32, device=DEV)
    off = torch.zeros(R + 1, dtype=torch.int64, device=DEV)
    okt.okt_region_partition(gpu.idx, gpu.nnz, w.n, R, b, off)
    rb, roff = orc.region_partition(ridx, w.n, R)
    assert np.array_equal(u32(b), rb) and np.array_equal(u64(off), roff)
    return counts, rb


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("name,n,iters", [("cfg1", 1_048_576, 1), ("cfg2", 2_000_003, 10),
                                          ("cfg3", 1_500_001, 34), ("cfg4", 4_000_007, 3)])
@pytest.mark.usefixtures("select_form")
def test_hot_path_loop_scaled(name, n, iters, fused):
    w = wl.WORKLOADS[name].scaled(n)
    counts, _ = run_loop(w, iters, w.P, fused=fused)
    # threshold reuse keeps the selected count near k on these stationary inputs
    # (the paper reports an average deviation below 11 %); reported, not a bar
    print(name, "max |nnz-k|/k =", max(abs(c - w.k) / w.k for c in counts))
