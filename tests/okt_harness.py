"""Helpers for the GPU parity tests: move numpy arrays to the device, call the
HIP library through its Python binding, bring results back.  No arithmetic."""
from __future__ import annotations

import numpy as np
import torch

import paper_2201_07598_amd as okt

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(DEV)
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def u32(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def u64(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def workspace(nbytes: int) -> torch.Tensor:
    # filled with a pattern: the library must not rely on a zeroed workspace
    return torch.full((max(int(nbytes), 256),), 0xA5, dtype=torch.uint8, device=DEV)


def bits_equal(a: np.ndarray, b: np.ndarray) -> bool:
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))


class GpuPath:
    """One worker's state on the device, driven through the five library calls."""

    def __init__(self, n: int, capacity: int):
        self.n = n
        self.capacity = capacity
        self.residual = torch.zeros(n, dtype=torch.float32, device=DEV)
        self.th = torch.zeros(1, dtype=torch.float32, device=DEV)
        self.count_ge = torch.zeros(1, dtype=torch.int64, device=DEV)
        self.idx = torch.full((max(capacity, 1),), -1, dtype=torch.int32, device=DEV)
        self.val = torch.zeros(max(capacity, 1), dtype=torch.float32, device=DEV)
        self.nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
        self.ws = workspace(okt.okt_workspace_bytes(n, 0))

    def accumulate(self, grad: torch.Tensor, lr: float):
        okt.okt_residual_accumulate(grad, self.residual, lr)

    def threshold(self, k: int):
        okt.okt_topk_threshold_exact(self.residual, k, self.th, self.count_ge, self.ws)

    def select(self):
        okt.okt_threshold_select(self.residual, self.th, self.idx, self.val, self.nnz, self.ws,
                                 capacity=self.capacity)

    def selected(self):
        nnz = u64(self.nnz)
        e = int(nnz[0])
        return u32(self.idx[:e]), self.val[:e].cpu().numpy(), int(nnz[0]), int(nnz[1])


def gpu_reduce(idx_cat, val_cat, chunk_off, lo, hi, capacity=None, dense=True):
    E = len(idx_cat)
    cap = E if capacity is None else capacity
    d_idx = to_dev(idx_cat) if E else torch.zeros(1, dtype=torch.int32, device=DEV)
    d_val = to_dev(val_cat) if E else torch.zeros(1, dtype=torch.float32, device=DEV)
    d_off = to_dev(np.asarray(chunk_off, dtype=np.uint64))
    out_idx = torch.full((max(cap, 1),), -1, dtype=torch.int32, device=DEV)
    out_val = torch.zeros(max(cap, 1), dtype=torch.float32, device=DEV)
    nnz = torch.zeros(2, dtype=torch.int64, device=DEV)
    d_dense = torch.full((max(hi - lo, 1),), 7.0, dtype=torch.float32, device=DEV) if dense else None
    ws = workspace(okt.okt_workspace_bytes(max(hi - lo, 1), len(chunk_off) - 1))
    okt.okt_sparse_reduce(d_idx, d_val, d_off, lo, hi, out_idx, out_val, nnz, ws,
                          dense_out=d_dense, capacity=cap)
    torch.cuda.synchronize()
    c = u64(nnz)
    e = int(c[0])
    w = min(e, cap)               # e is UINT64_MAX when the call reports a failed wait
    return {"idx": u32(out_idx[:w]), "val": out_val[:w].cpu().numpy(),
            "emitted": e, "total": int(c[1]),
            "dense": d_dense[:hi - lo].cpu().numpy() if dense else None}


def stated_tolerance(ref):
    """|gpu - ref| <= rtol * sum|v|: rtol 1e-6, or 1e-5 where more than 64
    contributions collide (the stated acceptance of the reduced fp32 values)."""
    return np.where(ref["hits"] > 64, 1e-5, 1e-6) * ref["abs_sum"]


def rounding_bound(ref):
    """What a sum accumulated in fp64, in any order, and rounded once to fp32 can
    differ from the oracle's by: one fp32 rounding step of the result
    (2^-23 |ref|, or the subnormal spacing 2^-149) plus the two fp64 sums' own
    error, at most hits * 2^-53 * sum|v| each."""
    return (2.0 ** -23 * np.abs(ref["val"].astype(np.float64)) + 2.0 ** -149 +
            ref["hits"] * 2.0 ** -52 * ref["abs_sum"])


def reduce_tolerance(ref):
    """The bound every reduced value is held to: the stated tolerance AND the
    rounding bound above (the smaller of the two per entry), so that a dropped or
    doubled contribution cannot hide inside 1e-6 * sum|v|."""
    return np.minimum(stated_tolerance(ref), rounding_bound(ref))
