"""GPU parity of the global stage: top-k selection on a reduced sparse region,
indexes = local ∩ global, and the residual update that follows it (Algorithm 1,
lines 9-14; Algorithm 2, line 6).  Everything here is bit-exact.
"""
import numpy as np
import pytest
import torch

import paper_2201_07598_amd as okt
import workloads as wl
from oracle import okt_oracle as orc
from tests.okt_harness import DEV, GpuPath, bits_equal, gpu_reduce, to_dev, u32, u64, workspace

pytestmark = pytest.mark.gpu


def lap(seed, n, scale=1e-3):
    return np.random.default_rng(seed).laplace(0, scale, n).astype(np.float32)


def sorted_indices(seed, space, count):
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(space, count, replace=False)).astype(np.uint32)


def padded(a, extra, fill):
    """The array followed by `extra` elements the library must not look at."""
    pad = np.full(extra, fill, dtype=a.dtype)
    return to_dev(np.concatenate([a, pad]))


def gpu_coo_select(idx, val, th, capacity=None, slack=0):
    nnz = idx.size
    bound = nnz + slack
    cap = bound if capacity is None else capacity
    d_idx = padded(idx, slack + 4, 0xDEADBEEF)
    d_val = padded(val, slack + 4, np.float32(1e30))      # would be selected if it were read
    d_nnz = to_dev(np.array([nnz], dtype=np.uint64))
    out_idx = torch.full((max(cap, 1),), -1, dtype=torch.int32, device=DEV)
    out_val = torch.zeros(max(cap, 1), dtype=torch.float32, device=DEV)
    out_nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(max(bound, 1), 0))
    okt.okt_coo_threshold_select(d_idx, d_val, d_nnz, to_dev(np.array([th], dtype=np.float32)),
                                 out_idx, out_val, out_nnz, ws, max_nnz=bound, capacity=cap)
    torch.cuda.synchronize()
    c = u64(out_nnz)
    e = int(c[0])
    # the input is left as it was
    assert np.array_equal(u32(d_idx[:nnz]), idx) and bits_equal(d_val[:nnz].cpu().numpy(), val)
    return u32(out_idx[:e]), out_val[:e].cpu().numpy(), e, int(c[1])


# ------------------------------------------------------------ global selection
@pytest.mark.parametrize("nnz", [0, 1, 3, 255, 256, 1000, 16_384 * 16 + 5, 70_001, 2_000_003])
@pytest.mark.parametrize("fraction", [0.0, 0.03, 0.5, 1.0])
def test_coo_select_bitwise(nnz, fraction):
    idx = sorted_indices(nnz + 1, max(4 * nnz, 16), nnz)
    val = lap(nnz + 2, nnz)
    if nnz > 10:
        val[::97] = 0.0
        val[5] = -val[6]
    if fraction == 0.0:
        th = 1e30
    elif fraction == 1.0 or nnz == 0:
        th = 0.0
    else:
        th = float(np.sort(np.abs(val))[::-1][max(int(fraction * nnz) - 1, 0)])
    ri, rv, rtotal = orc.coo_threshold_select(idx, val, th)
    gi, gv, emitted, total = gpu_coo_select(idx, val, th)
    assert (emitted, total) == (ri.size, rtotal)
    assert np.array_equal(gi, ri) and bits_equal(gv, rv)


def test_coo_select_device_count_capacity_and_odd_thresholds():
    nnz = 300_007
    idx = sorted_indices(5, 10_000_000, nnz)
    val = lap(6, nnz)
    val[100] = np.nan
    val[200] = np.inf
    val[300] = -np.inf
    th = float(np.sort(np.abs(val[np.isfinite(val)]))[-3000])
    # fewer entries on the device than the host-side bound
    ri, rv, rtotal = orc.coo_threshold_select(idx, val, th)
    gi, gv, emitted, total = gpu_coo_select(idx, val, th, slack=50_000)
    assert (emitted, total) == (ri.size, rtotal)
    assert np.array_equal(gi, ri) and bits_equal(gv, rv)
    # truncated output
    for cap in (0, 1, 777, rtotal - 1, rtotal, rtotal + 5):
        ri, rv, rtotal = orc.coo_threshold_select(idx, val, th, capacity=cap)
        gi, gv, emitted, total = gpu_coo_select(idx, val, th, capacity=cap)
        assert (emitted, total) == (ri.size, rtotal), cap
        assert np.array_equal(gi, ri) and bits_equal(gv, rv), cap
    # negative, infinite and NaN thresholds
    for odd in (-th, np.inf, np.nan, -0.0):
        ri, rv, rtotal = orc.coo_threshold_select(idx, val, odd)
        gi, gv, emitted, total = gpu_coo_select(idx, val, odd)
        assert (emitted, total) == (ri.size, rtotal), odd
        assert np.array_equal(gi, ri) and bits_equal(gv, rv), odd


# ----------------------------------------------- indexes and residual update
def gpu_restore(acc, local_idx, global_idx, want_indexes=True, slack_l=0, slack_g=0, zero=False):
    """zero=False: the residual as the select leaves it (all local entries
    zeroed), then the library's intersect + restore.  zero=True: the untouched
    accumulator, then the library's intersect + zero."""
    residual = acc.copy()
    if not zero:
        residual[local_idx.astype(np.int64)] = 0.0
    local_val = acc[local_idx.astype(np.int64)]
    d_res = to_dev(residual)
    d_li = padded(local_idx, slack_l + 1, 0)
    d_lv = padded(local_val, slack_l + 1, np.float32(123.0))
    d_gi = padded(global_idx, slack_g + 1, 0)
    d_ln = to_dev(np.array([local_idx.size], dtype=np.uint64))
    d_gn = to_dev(np.array([global_idx.size], dtype=np.uint64))
    bound_l = local_idx.size + slack_l
    out = torch.full((max(bound_l, 1),), -1, dtype=torch.int32, device=DEV) if want_indexes else None
    cnt = torch.full((1,), -5, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(max(bound_l, 1), 0))
    if zero:
        okt.okt_index_intersect_zero(d_res, d_li, d_ln, d_gi, d_gn, cnt, ws, indexes_out=out,
                                     max_local=bound_l, max_global=global_idx.size + slack_g)
    else:
        okt.okt_index_intersect_restore(d_res, d_li, d_lv, d_ln, d_gi, d_gn, cnt, ws,
                                        indexes_out=out, max_local=bound_l,
                                        max_global=global_idx.size + slack_g)
    torch.cuda.synchronize()
    c = int(u64(cnt)[0])
    return d_res.cpu().numpy(), (u32(out[:c]) if want_indexes else None), c


@pytest.mark.parametrize("nl,ng", [(0, 0), (0, 50), (50, 0), (1, 1), (1023, 700), (1024, 1024),
                                   (1025, 3), (5000, 5000), (200_003, 150_001),
                                   (64 * 1024 + 1, 400_000), (300_000, 17), (900, 3_000_000)])
@pytest.mark.parametrize("zero", [False, True])
def test_intersect_restore_bitwise(nl, ng, zero):
    n = max(4 * max(nl, ng), 64)
    acc = lap(nl * 7 + ng, n)
    local_idx = sorted_indices(nl + 11, n, nl)
    # about half of the global list comes from the local one
    rng = np.random.default_rng(ng + 13)
    from_local = rng.choice(local_idx, min(ng // 2, nl), replace=False) if nl else np.zeros(0, np.uint32)
    others = rng.choice(n, ng - from_local.size, replace=False)
    global_idx = np.unique(np.concatenate([from_local, others]).astype(np.uint32))
    indexes = orc.index_intersection(local_idx, global_idx)
    eps = orc.residual_update(acc, indexes)
    res, gidx, count = gpu_restore(acc, local_idx, global_idx, zero=zero)
    assert count == indexes.size
    assert np.array_equal(gidx, indexes)
    assert bits_equal(res, eps)
    res, _, count = gpu_restore(acc, local_idx, global_idx, want_indexes=False, slack_l=333,
                                slack_g=77, zero=zero)
    assert count == indexes.size and bits_equal(res, eps)


def test_intersect_restore_special_lists():
    n = 100_000
    acc = lap(3, n)
    acc[acc == 0] = 1e-3
    local_idx = sorted_indices(4, n, 9000)
    local_idx[0], local_idx[-1] = 0, n - 1
    everything = np.arange(n, dtype=np.uint32)
    cases = {
        "identical": local_idx,                       # eps = the select's residual
        "superset": everything,
        "disjoint": np.setdiff1d(everything, local_idx).astype(np.uint32),
        "ends only": np.array([0, n - 1], dtype=np.uint32),
        "one block": local_idx[2000:3100],
        "below all": np.array([0], dtype=np.uint32),
    }
    for name, global_idx in cases.items():
        indexes = orc.index_intersection(local_idx, global_idx)
        for zero in (False, True):
            res, gidx, count = gpu_restore(acc, local_idx, global_idx, zero=zero)
            assert count == indexes.size, name
            assert np.array_equal(gidx, indexes), name
            assert bits_equal(res, orc.residual_update(acc, indexes)), name


@pytest.mark.parametrize("n", [1, 255, 4097, 1_000_003, 5_000_011])
def test_select_copy_leaves_the_accumulator(n):
    acc = lap(n + 9, n)
    k = max(n // 100, 1)
    th, _ = orc.topk_threshold_exact(acc, k, method="partition")
    for cap in (None, k // 2):
        ri, rv, _, rtotal = orc.threshold_select(acc, th, capacity=cap)
        d_acc = to_dev(acc)
        size = max(2 * k if cap is None else cap, 1)
        idx = torch.full((size,), -1, dtype=torch.int32, device=DEV)
        val = torch.zeros(size, dtype=torch.float32, device=DEV)
        nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
        ws = workspace(okt.okt_workspace_bytes(n, 0))
        okt.okt_threshold_select_copy(d_acc, to_dev(np.array([th], dtype=np.float32)), idx, val,
                                      nnz, ws, capacity=(size if cap is None else cap))
        torch.cuda.synchronize()
        c = u64(nnz)
        assert (int(c[0]), int(c[1])) == (ri.size, rtotal)
        assert np.array_equal(u32(idx[:ri.size]), ri) and bits_equal(val[:ri.size].cpu().numpy(), rv)
        assert bits_equal(d_acc.cpu().numpy(), acc)


# ------------------------------------------------ the whole algorithm, P workers
@pytest.mark.parametrize("name,n,P", [("cfg1", 300_007, 4), ("cfg2", 1_000_003, 8)])
def test_allreduce_and_residuals_over_simulated_workers(name, n, P):
    """Algorithm 1 with the collectives replaced by host-side concatenation, every
    worker's arithmetic on the GPU, against the same chain in the oracle.  With P
    contributions whose magnitudes all lie within a factor 2^20 the fp64 sums are
    exact, so the reduced values, the global threshold and every set that depends
    on them are bit-identical."""
    w = wl.WORKLOADS[name].scaled(n)
    k = w.k
    accs, ref_local, gpu_paths = [], [], []
    for p in range(P):
        g = wl.gradient(w, 1000 * p)                 # a different gradient per worker
        acc = orc.residual_accumulate(g, np.zeros(n, dtype=np.float32), w.lr)
        th, _ = orc.topk_threshold_exact(acc, k, method="partition")
        li, lv, _, _ = orc.threshold_select(acc, th)
        accs.append(acc)
        ref_local.append((li, lv))
        path = GpuPath(n, 2 * k)
        path.accumulate(to_dev(g), w.lr)
        path.threshold(k)
        if p % 2 == 0:
            path.select()                            # zero now, put back later
        else:                                        # keep acc, zero `indexes` later
            okt.okt_threshold_select_copy(path.residual, path.th, path.idx, path.val, path.nnz,
                                          path.ws, capacity=path.capacity)
        gi, gv, emitted, total = path.selected()
        assert total == li.size and np.array_equal(gi, li) and bits_equal(gv, lv)
        gpu_paths.append(path)

    off = np.zeros(P + 1, dtype=np.uint64)
    off[1:] = np.cumsum([li.size for li, _ in ref_local])
    idx_cat = np.concatenate([li for li, _ in ref_local])
    val_cat = np.concatenate([lv for _, lv in ref_local])
    lo_mag, hi_mag = np.abs(val_cat).min(), np.abs(val_cat).max()
    assert 0 < lo_mag and hi_mag / lo_mag < 2.0 ** 20

    # split and reduce over R = P regions, one region per worker
    bounds, _ = orc.region_partition(ref_local[0][0], n, P)
    ref_regions, gpu_regions = [], []
    for r in range(P):
        lo, hi = int(bounds[r]), int(bounds[r + 1])
        ref = orc.sparse_reduce(idx_cat, val_cat, off, lo, hi)
        got = gpu_reduce(idx_cat, val_cat, off, lo, hi, dense=False)
        assert np.array_equal(got["idx"], ref["idx"]) and bits_equal(got["val"], ref["val"]), r
        ref_regions.append(ref)
        gpu_regions.append(got)

    # global threshold: the k-th largest of all reduced values (gathered)
    all_val = np.concatenate([ref["val"] for ref in ref_regions])
    gth, gcnt = orc.topk_threshold_exact(all_val, k, method="partition")
    d_th = torch.zeros(1, dtype=torch.float32, device=DEV)
    d_cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    ws = workspace(okt.okt_workspace_bytes(all_val.size, 0))
    okt.okt_topk_threshold_exact(to_dev(all_val), k, d_th, d_cnt, ws)
    assert d_th.cpu().numpy().view(np.uint32)[0] == np.float32(gth).view(np.uint32)
    assert int(u64(d_cnt)[0]) == gcnt

    # global selection per region, concatenated in region order = u_t
    ref_u_idx, gpu_u_idx = [], []
    for r in range(P):
        ref = ref_regions[r]
        ri, rv, rtotal = orc.coo_threshold_select(ref["idx"], ref["val"], gth)
        gi, gv, emitted, total = gpu_coo_select(ref["idx"], ref["val"], gth)
        assert total == rtotal and np.array_equal(gi, ri) and bits_equal(gv, rv), r
        ref_u_idx.append(ri)
        gpu_u_idx.append(gi)
    u_idx = np.concatenate(ref_u_idx)
    assert u_idx.size == gcnt and np.all(np.diff(u_idx.astype(np.int64)) > 0)

    # indexes and residuals of every worker
    d_u = to_dev(np.concatenate(gpu_u_idx))
    d_un = to_dev(np.array([u_idx.size], dtype=np.uint64))
    kept_back = 0
    for p in range(P):
        path = gpu_paths[p]
        indexes = orc.index_intersection(ref_local[p][0], u_idx)
        eps = orc.residual_update(accs[p], indexes)
        out = torch.full((path.capacity,), -1, dtype=torch.int32, device=DEV)
        cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
        if p % 2 == 0:
            okt.okt_index_intersect_restore(path.residual, path.idx, path.val, path.nnz[:1], d_u,
                                            d_un, cnt, path.ws, indexes_out=out)
        else:
            okt.okt_index_intersect_zero(path.residual, path.idx, path.nnz[:1], d_u, d_un, cnt,
                                         path.ws, indexes_out=out)
        c = int(u64(cnt)[0])
        assert c == indexes.size and np.array_equal(u32(out[:c]), indexes), p
        assert bits_equal(path.residual.cpu().numpy(), eps), p
        kept_back += ref_local[p][0].size - indexes.size
    assert kept_back > 0                             # the restore had something to do
