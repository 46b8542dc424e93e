"""Seeded random shapes through every entry point, each compared with the oracle:
vector lengths, densities, thresholds, capacities, numbers of contributions (up
to several sweeps' worth), region widths and positions (up to the top of the
32-bit index space), batches with regions of unequal width, segments in any
order.  The fixed cases elsewhere pin known corners; this sweep covers the
combinations nobody thought of (it found the reload race of the reduce kernel's
slice table with more than 256 contributions over ranked tiles)."""
import numpy as np
import pytest
import torch

import paper_2201_07598_amd as okt
from oracle import okt_oracle as orc
from tests.okt_harness import (DEV, bits_equal, gpu_reduce, reduce_tolerance, to_dev, u32, u64,
                               workspace)

pytestmark = pytest.mark.gpu


def structured(rng, n):
    """Layered scales, dense runs, ties, zeros and subnormals, by turns."""
    kind = int(rng.integers(0, 5))
    x = rng.laplace(0, 1e-3, n).astype(np.float32)
    if kind == 1 and n > 8:
        cuts = np.sort(rng.integers(0, n, 6))
        for a, b in zip(cuts[:-1], cuts[1:]):
            x[a:b] *= np.float32(10.0 ** rng.integers(-3, 3))
    if kind == 2 and n > 8:
        for _ in range(3):
            a = int(rng.integers(0, n))
            b = min(n, a + int(rng.integers(1, 40_000)))
            x[a:b] = rng.choice([-1.0, 1.0], b - a).astype(np.float32) * np.float32(0.5)
    if kind == 3:
        x = rng.choice(np.array([0.0, -0.0, 1e-3, -1e-3, 2e-3, 1e-40, 3e-3], dtype=np.float32), n)
    if kind == 4 and n > 0:
        x[rng.random(n) < 0.97] = 0.0
    return x


def selected_matches(idx, val, nnz, ridx, rval, total):
    c = u64(nnz)
    return ((int(c[0]), int(c[1])) == (ridx.size, total)
            and np.array_equal(u32(idx[:ridx.size]), ridx)
            and bits_equal(val[:ridx.size].cpu().numpy(), rval))


@pytest.mark.usefixtures("select_form")
@pytest.mark.parametrize("seed", range(6))
def test_random_iterations_of_the_dense_path(seed):
    rng = np.random.default_rng(9000 + seed)
    for case in range(12):
        n = int(rng.choice([rng.integers(1, 5000), rng.integers(5000, 300_000),
                            rng.integers(300_000, 3_000_000)]))
        acc0, g, g2 = structured(rng, n), structured(rng, n), structured(rng, n)
        lr = float(rng.choice([1.0, 0.5, -0.25, 0.1]))
        k = int(rng.integers(1, n + 1)) if rng.random() < 0.2 else \
            max(1, int(n * rng.choice([0.001, 0.01, 0.05, 0.3])))
        where = f"seed {seed} case {case}: n={n} k={k} lr={lr}"
        ws = workspace(okt.okt_workspace_bytes(n, 0))
        d_res = to_dev(acc0)
        okt.okt_residual_accumulate(to_dev(g), d_res, lr)
        a1 = orc.residual_accumulate(g, acc0, lr)
        assert bits_equal(d_res.cpu().numpy(), a1), where
        th = torch.zeros(1, device=DEV)
        cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
        okt.okt_topk_threshold_exact(d_res, k, th, cnt, workspace(70_000) if rng.random() < 0.3 else ws)
        rth, rcnt = orc.topk_threshold_exact(a1, k, method="partition")
        assert th.cpu().numpy().view(np.uint32)[0] == np.float32(rth).view(np.uint32), where
        assert int(u64(cnt)[0]) == rcnt, where
        cap = int(rng.choice([rcnt, max(rcnt // 2, 1), rcnt + 7, 4 * k]))
        idx = torch.full((cap,), -1, dtype=torch.int32, device=DEV)
        val = torch.zeros(cap, device=DEV)
        nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
        ridx, rval, rres, total = orc.threshold_select(a1, rth, capacity=cap)
        d_copy = d_res.clone()
        okt.okt_threshold_select_copy(d_copy, th, idx, val, nnz, ws, capacity=cap)
        assert selected_matches(idx, val, nnz, ridx, rval, total), where
        assert bits_equal(d_copy.cpu().numpy(), a1), where
        okt.okt_threshold_select(d_res, th, idx, val, nnz, ws, capacity=cap)
        assert selected_matches(idx, val, nnz, ridx, rval, total), where
        assert bits_equal(d_res.cpu().numpy(), rres), where
        R = int(rng.choice([1, 2, 7, 16, 64, 300]))
        b = torch.zeros(R + 1, dtype=torch.int32, device=DEV)
        off = torch.zeros(R + 1, dtype=torch.int64, device=DEV)
        okt.okt_region_partition(idx, nnz, n, R, b, off)
        rb, roff = orc.region_partition(ridx, n, R)
        assert np.array_equal(u32(b), rb) and np.array_equal(u64(off), roff), where
        okt.okt_accumulate_select(to_dev(g2), d_res, lr, th, idx, val, nnz, ws, capacity=cap)
        a2 = orc.residual_accumulate(g2, rres, lr)
        ridx2, rval2, rres2, total2 = orc.threshold_select(a2, rth, capacity=cap)
        assert selected_matches(idx, val, nnz, ridx2, rval2, total2), where
        assert bits_equal(d_res.cpu().numpy(), rres2), where


def contribution(rng, width, lo, m, mode, shared):
    m = min(m, width)
    if m == 0:
        return np.zeros(0, np.uint32)
    if mode == 0:
        loc = rng.choice(width, m, replace=False)
    elif mode == 1:                                  # clustered
        span = min(width, 2 * m)
        loc = rng.choice(span, m, replace=False) + int(rng.integers(0, width - span + 1))
    elif mode == 2:                                  # a support shared by everyone
        loc = shared[:m]
    else:                                            # a dense run
        loc = np.arange(m) + int(rng.integers(0, width - m + 1))
    return (np.sort(loc) + lo).astype(np.uint32)


def reduced_matches(idx, val, nnz, dense, ref, cap, lo):
    U = ref["idx"].size
    e = min(U, cap)
    if (int(nnz[0]), int(nnz[1])) != (e, U) or not np.array_equal(idx[:e], ref["idx"][:e]):
        return False
    tol = reduce_tolerance(ref)
    if np.any(np.abs(val[:e].astype(np.float64) - ref["val"][:e].astype(np.float64)) > tol[:e]):
        return False
    if dense is not None:
        width = ref["dense"].size
        dt = np.zeros(width)
        dt[ref["idx"].astype(np.int64) - lo] = tol
        return bool(np.all(np.abs(dense[:width].astype(np.float64) - ref["dense"]) <= dt))
    return True


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes_of_the_reduce_family(seed):
    rng = np.random.default_rng(9100 + seed)
    for case in range(14):
        P = int(rng.choice([1, 3, 16, 64, 255, 256, 257, 300, 513, 1000, 2500]))
        width = int(rng.choice([1, 31, 4096, 4100, 33_000, 70_000, 700_000, 3_000_000]))
        mmax = int(rng.choice([0, 3, 70, 500, 4000, 20_000]))
        if P * mmax > 2_000_000:
            mmax = 2_000_000 // P
        B = int(rng.choice([1, 1, 2, 5, 17]))
        if B * width > 8_000_000:
            B = 1
        where = f"seed {seed} case {case}: P={P} width={width} mmax={mmax} B={B}"
        base = int(rng.integers(0, (1 << 32) - 1 - B * width))
        regions = []
        for j in range(B):
            w_j = width if (j == 0 or rng.random() < 0.5) else int(rng.integers(0, width + 1))
            lo = base + j * width
            shared = np.sort(rng.choice(max(w_j, 1), min(max(w_j, 1), max(mmax, 1)), replace=False))
            parts = [contribution(rng, w_j, lo, int(rng.integers(0, mmax + 1)),
                                  int(rng.integers(0, 4)), shared) if w_j else np.zeros(0, np.uint32)
                     for p in range(P)]
            regions.append((lo, lo + w_j, parts))
        sizes = [x.size for r in regions for x in r[2]]
        E1 = [sum(x.size for x in r[2]) for r in regions]
        idx_cat = np.concatenate([x for r in regions for x in r[2]]) if sum(sizes) else np.zeros(0, np.uint32)
        val_cat = rng.laplace(0, 1e-3, idx_cat.size).astype(np.float32)
        starts = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
        offs = np.zeros(B * (P + 1), dtype=np.uint64)
        for j in range(B):
            offs[j * (P + 1):(j + 1) * (P + 1)] = starts[j * P:(j + 1) * P + 1]
        cap = int(rng.choice([max(E1), max(max(E1) // 3, 1), 0 if rng.random() < 0.1 else max(E1) + 5]))
        d_idx = to_dev(idx_cat) if idx_cat.size else torch.zeros(1, dtype=torch.int32, device=DEV)
        d_val = to_dev(val_cat) if idx_cat.size else torch.zeros(1, device=DEV)
        lohi = np.array([[r[0], r[1]] for r in regions], dtype=np.uint32).reshape(-1)
        out_idx = torch.full((max(B * cap, 1),), -1, dtype=torch.int32, device=DEV)
        out_val = torch.zeros(max(B * cap, 1), device=DEV)
        nnz = torch.zeros(2 * B, dtype=torch.int64, device=DEV)
        dense = torch.full((B * width,), 7.0, device=DEV) if rng.random() < 0.6 else None
        ws = workspace(okt.okt_sparse_reduce_batch_workspace_bytes(B, P, width))
        okt.okt_sparse_reduce_batch(d_idx, d_val, to_dev(offs), to_dev(lohi), B, P, width, out_idx,
                                    out_val, cap, nnz, ws, dense_out=dense)
        torch.cuda.synchronize()
        g_idx, g_val, g_nnz = u32(out_idx), out_val.cpu().numpy(), u64(nnz)
        g_dense = dense.cpu().numpy() if dense is not None else None
        for j, (lo, hi, _) in enumerate(regions):
            ref = orc.sparse_reduce(idx_cat, val_cat, offs[j * (P + 1):(j + 1) * (P + 1)], lo, hi)
            assert reduced_matches(g_idx[j * cap:(j + 1) * cap], g_val[j * cap:(j + 1) * cap],
                                   g_nnz[2 * j:2 * j + 2],
                                   g_dense[j * width:(j + 1) * width] if dense is not None else None,
                                   ref, cap, lo), f"{where} batch region {j} cap={cap}"
        # the first region alone, and as segments handed over in any order
        lo, hi, _ = regions[0]
        co = offs[:P + 1].copy()
        ref = orc.sparse_reduce(idx_cat, val_cat, co, lo, hi)
        cap1 = max(E1[0], 1)
        o_i = torch.full((cap1,), -1, dtype=torch.int32, device=DEV)
        o_v = torch.zeros(cap1, device=DEV)
        o_n = torch.zeros(2, dtype=torch.int64, device=DEV)
        ws1 = workspace(okt.okt_workspace_bytes(max(hi - lo, 1), P))
        okt.okt_sparse_reduce(d_idx, d_val, to_dev(co), lo, hi, o_i, o_v, o_n, ws1, capacity=cap1)
        torch.cuda.synchronize()
        assert reduced_matches(u32(o_i), o_v.cpu().numpy(), u64(o_n), None, ref, cap1, lo), f"{where} single"
        perm = rng.permutation(P)
        okt.okt_sparse_reduce_segments(d_idx, d_val, to_dev(co[:-1][perm].copy()),
                                       to_dev(co[1:][perm].copy()), P, lo, hi, o_i, o_v, o_n, ws1,
                                       capacity=cap1)
        torch.cuda.synchronize()
        assert reduced_matches(u32(o_i), o_v.cpu().numpy(), u64(o_n), None, ref, cap1, lo), f"{where} segments"
        # the global stage on what was reduced
        U = ref["idx"].size
        if U:
            gth = np.float32(np.abs(ref["val"]).max() * rng.choice([0.0, 0.3, 0.9, 1.5]))
            s_i = torch.full((U,), -1, dtype=torch.int32, device=DEV)
            s_v = torch.zeros(U, device=DEV)
            s_n = torch.zeros(2, dtype=torch.int64, device=DEV)
            wsr = workspace(okt.okt_workspace_bytes(max(U, hi - lo), 0))
            okt.okt_coo_threshold_select(to_dev(ref["idx"]), to_dev(ref["val"]),
                                         to_dev(np.array([U], dtype=np.uint64)),
                                         to_dev(np.array([gth], dtype=np.float32)), s_i, s_v, s_n,
                                         wsr, max_nnz=U)
            gi, gv, gt = orc.coo_threshold_select(ref["idx"], ref["val"], gth)
            assert selected_matches(s_i, s_v, s_n, gi, gv, gt), f"{where} global select"
            # a local list over the same region: random indices and some of the global ones
            w0 = hi - lo
            nl = int(rng.integers(0, min(w0, 5000) + 1))
            loc = rng.choice(w0, nl, replace=False).astype(np.int64)
            if gt:
                loc = np.concatenate([loc, gi[rng.random(gt) < 0.5].astype(np.int64) - lo])
            li = np.unique(loc).astype(np.uint32)
            gli = (gi.astype(np.int64) - lo).astype(np.uint32)
            vals = rng.laplace(0, 1e-3, li.size).astype(np.float32)
            acc_l = np.zeros(w0, dtype=np.float32)
            acc_l[li.astype(np.int64)] = vals
            want = orc.index_intersection(li, gli)
            eps = orc.residual_update(acc_l, want)
            some = lambda a, dt: to_dev(a) if a.size else torch.zeros(1, dtype=dt, device=DEV)
            d_li, d_gli = some(li, torch.int32), some(gli, torch.int32)
            n_l = to_dev(np.array([li.size], dtype=np.uint64))
            n_g = to_dev(np.array([gli.size], dtype=np.uint64))
            inter = torch.full((max(li.size, 1),), -1, dtype=torch.int32, device=DEV)
            count = torch.zeros(1, dtype=torch.int64, device=DEV)
            d_vec = torch.zeros(w0, device=DEV)              # every local entry already zeroed
            okt.okt_index_intersect_restore(d_vec, d_li, some(vals, torch.float32), n_l, d_gli, n_g,
                                            count, wsr, indexes_out=inter, max_local=li.size,
                                            max_global=gli.size)
            assert int(u64(count)[0]) == want.size, f"{where} intersect restore"
            assert np.array_equal(u32(inter[:want.size]), want), f"{where} intersect restore"
            assert bits_equal(d_vec.cpu().numpy(), eps), f"{where} intersect restore"
            d_vec = to_dev(acc_l)                            # the untouched accumulator
            okt.okt_index_intersect_zero(d_vec, d_li, n_l, d_gli, n_g, count, wsr, indexes_out=inter,
                                         max_local=li.size, max_global=gli.size)
            assert int(u64(count)[0]) == want.size, f"{where} intersect zero"
            assert bits_equal(d_vec.cpu().numpy(), eps), f"{where} intersect zero"


@pytest.mark.parametrize("seed", range(3))
def test_random_vectors_through_the_sampled_threshold(seed):
    """Vectors long enough for the sample-then-count path of the exact threshold,
    of kinds on which a sample says much, little or the wrong thing, at ranks
    from 1 to n and with workspaces from the smallest to the full one."""
    rng = np.random.default_rng(9200 + seed)
    for case in range(5):
        n = int(rng.integers(4_194_304 - 5, 16_000_000))
        kind = int(rng.integers(0, 7))
        x = rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)
        if kind == 1:                                # layers of different scale
            cuts = np.sort(rng.integers(0, n, 8))
            for a, b in zip(cuts[:-1], cuts[1:]):
                x[a:b] *= np.float32(10.0 ** rng.integers(-4, 4))
        if kind == 2:                                # the large values sit in a few short blocks
            x *= np.float32(1e-3)
            for _ in range(int(rng.integers(1, 6))):
                a = int(rng.integers(0, n))
                b = min(n, a + int(rng.integers(1, 3000)))
                x[a:b] = rng.standard_normal(b - a).astype(np.float32)
        if kind == 3:                                # five distinct values
            x = rng.choice(np.array([0.0, 1e-3, -1e-3, 2e-3, 5e-4], dtype=np.float32), n)
        if kind == 4:                                # nearly all zero
            x[rng.random(n) < 0.999] = 0.0
        if kind == 5:                                # all equal
            x[:] = np.float32(rng.choice([0.0, 1.5, -2.0, 1e-40]))
        if kind == 6:                                # one exponent: the first digit says little
            x = np.abs(x) + np.float32(1.0)
        d = to_dev(x)
        full = workspace(okt.okt_workspace_bytes(n, 0))
        for k in (1, n, int(rng.integers(1, n + 1)), max(1, n // 1000), max(1, n // 100), max(1, n // 7)):
            ws = full if rng.random() < 0.6 else workspace(int(rng.choice([70_000, 300_000, 4_000_000])))
            th = torch.zeros(1, device=DEV)
            cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
            okt.okt_topk_threshold_exact(d, k, th, cnt, ws)
            rth, rcnt = orc.topk_threshold_exact(x, k, method="partition")
            where = f"seed {seed} case {case}: n={n} kind={kind} k={k} ws={ws.numel()}"
            assert th.cpu().numpy().view(np.uint32)[0] == np.float32(rth).view(np.uint32), where
            assert int(u64(cnt)[0]) == rcnt, where


@pytest.mark.usefixtures("select_form")
@pytest.mark.timeout(300)
@pytest.mark.parametrize("seed", range(3))
def test_random_refresh_iterations_in_one_call(seed):
    """okt_accumulate_topk_select on long vectors of the same kinds, with a
    residual of a random scale, ranks from 1 to n, outputs that fill up, and
    workspaces from the smallest to the full one, against the oracle's accumulate,
    exact threshold and select applied in turn."""
    rng = np.random.default_rng(9300 + seed)
    for case in range(4):
        n = int(rng.integers(4_194_304 - 5, 12_000_000))
        kind = int(rng.integers(0, 6))
        g = rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)
        if kind == 1:                                # layers of different scale
            cuts = np.sort(rng.integers(0, n, 8))
            for a, b in zip(cuts[:-1], cuts[1:]):
                g[a:b] *= np.float32(10.0 ** rng.integers(-4, 4))
        if kind == 2:                                # the large values sit in a few short blocks
            g *= np.float32(1e-3)
            for _ in range(int(rng.integers(1, 6))):
                a = int(rng.integers(0, n))
                b = min(n, a + int(rng.integers(1, 3000)))
                g[a:b] = rng.standard_normal(b - a).astype(np.float32)
        if kind == 3:                                # five distinct values
            g = rng.choice(np.array([0.0, 1e-3, -1e-3, 2e-3, 5e-4], dtype=np.float32), n)
        if kind == 4:                                # nearly all zero
            g[rng.random(n) < 0.999] = 0.0
        if kind == 5:                                # one exponent: the first digit says little
            g = np.abs(g) + np.float32(1.0)
        e = rng.standard_normal(n, dtype=np.float32) * np.float32(rng.choice([0.0, 1e-4, 1e-2]))
        lr = float(rng.choice([1.0, 0.5, -0.25]))
        acc = orc.residual_accumulate(g, e, lr)
        d_g = to_dev(g)
        full = okt.okt_workspace_bytes(n, 0)
        for k in (int(rng.integers(1, n + 1)), max(1, n // 1000), max(1, n // 100)):
            ws = workspace(full if rng.random() < 0.7 else int(rng.choice([70_000, 300_000, 4_000_000])))
            rth, rcnt = orc.topk_threshold_exact(acc, k, method="partition")
            cap = int(rng.choice([rcnt, rcnt + 5, rcnt // 2, 0]))
            ridx, rval, rres, total = orc.threshold_select(acc, rth, capacity=cap)
            d_e = to_dev(e)
            th = torch.zeros(1, device=DEV)
            cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
            idx = torch.full((max(cap, 1),), -1, dtype=torch.int32, device=DEV)
            val = torch.zeros(max(cap, 1), dtype=torch.float32, device=DEV)
            nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
            okt.okt_accumulate_topk_select(d_g, d_e, lr, k, th, cnt, idx, val, nnz, ws, capacity=cap)
            where = f"seed {seed} case {case}: n={n} kind={kind} k={k} cap={cap} ws={ws.numel()}"
            assert th.cpu().numpy().view(np.uint32)[0] == np.float32(rth).view(np.uint32), where
            assert int(u64(cnt)[0]) == rcnt == total, where
            assert selected_matches(idx, val, nnz, ridx, rval, total), where
            assert bits_equal(d_e.cpu().numpy(), rres), where
