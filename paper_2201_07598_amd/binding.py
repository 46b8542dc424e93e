"""ctypes binding of the C ABI declared in include/okt.h.

Argument marshalling only: every function takes torch CUDA tensors (device
memory) and plain Python scalars, checks dtype / device / contiguity, passes raw
pointers and the current HIP stream, and raises OktError on a non-zero status.
No arithmetic of the method happens here.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

c_u32, c_u64, c_sz, c_vp, c_f32, c_int = (ctypes.c_uint32, ctypes.c_uint64, ctypes.c_size_t,
                                          ctypes.c_void_p, ctypes.c_float, ctypes.c_int)

# name -> (restype, argtypes); mirrors include/okt.h
SIGNATURES = {
    "okt_status_string": (ctypes.c_char_p, [c_int]),
    "okt_last_hip_error": (ctypes.c_char_p, []),
    "okt_time_next_kernel": (None, [c_vp, c_vp]),
    "okt_debug_spin_limit": (None, [c_u32]),
    "okt_debug_slot_min_n": (None, [c_u64]),
    "okt_slot_min_n": (c_u64, [c_int]),
    "okt_version": (c_int, []),
    "okt_stream_copy": (c_int, [c_vp, c_vp, c_u64, c_vp]),
    "okt_stream_sum": (c_int, [c_vp, c_u64, c_vp, c_vp]),
    "okt_stream_gather": (c_int, [c_vp, c_vp, c_vp, c_vp, c_u32, c_u32, c_u32, c_vp, c_vp, c_u64, c_vp,
                                  c_sz, c_vp]),
    "okt_workspace_bytes": (c_sz, [c_u64, c_u32]),
    "okt_sparse_reduce_batch_workspace_bytes": (c_sz, [c_u32, c_u32, c_u32]),
    "okt_residual_accumulate": (c_int, [c_vp, c_vp, c_f32, c_u64, c_vp]),
    "okt_topk_threshold_exact": (c_int, [c_vp, c_u64, c_u64, c_vp, c_vp, c_vp, c_sz, c_vp]),
    "okt_threshold_select": (c_int, [c_vp, c_u64, c_vp, c_vp, c_vp, c_u64, c_vp, c_vp, c_sz, c_vp]),
    "okt_threshold_select_noalloc": (c_int, [c_vp, c_u64, c_vp, c_vp, c_vp, c_u64, c_vp, c_vp]),
    "okt_threshold_select_copy": (c_int, [c_vp, c_u64, c_vp, c_vp, c_vp, c_u64, c_vp, c_vp, c_sz, c_vp]),
    "okt_index_intersect_zero": (c_int, [c_vp, c_u64, c_vp, c_vp, c_u64, c_vp, c_vp, c_u64, c_vp, c_vp,
                                         c_vp, c_sz, c_vp]),
    "okt_accumulate_select": (c_int, [c_vp, c_vp, c_f32, c_u64, c_vp, c_vp, c_vp, c_u64, c_vp, c_vp,
                                      c_sz, c_vp]),
    "okt_accumulate_topk_select": (c_int, [c_vp, c_vp, c_f32, c_u64, c_u64, c_vp, c_vp, c_vp, c_vp,
                                           c_u64, c_vp, c_vp, c_sz, c_vp]),
    "okt_coo_threshold_select": (c_int, [c_vp, c_vp, c_vp, c_u64, c_vp, c_vp, c_vp, c_u64, c_vp, c_vp,
                                         c_sz, c_vp]),
    "okt_index_intersect_restore": (c_int, [c_vp, c_u64, c_vp, c_vp, c_vp, c_u64, c_vp, c_vp, c_u64,
                                            c_vp, c_vp, c_vp, c_sz, c_vp]),
    "okt_region_partition": (c_int, [c_vp, c_vp, c_u64, c_u32, c_vp, c_vp, c_vp]),
    "okt_sparse_reduce": (c_int, [c_vp, c_vp, c_vp, c_u32, c_u32, c_u32, c_vp, c_vp, c_u64, c_vp,
                                  c_vp, c_vp, c_sz, c_vp]),
    "okt_sparse_reduce_segments": (c_int, [c_vp, c_vp, c_vp, c_vp, c_u32, c_u32, c_u32, c_vp, c_vp, c_u64,
                                           c_vp, c_vp, c_vp, c_sz, c_vp]),
    "okt_balance_plan": (c_int, [c_vp, c_u32, c_vp, c_u32, c_vp, c_vp]),
    "okt_sparse_reduce_batch": (c_int, [c_vp, c_vp, c_vp, c_vp, c_u32, c_u32, c_u32, c_vp, c_vp,
                                        c_u64, c_vp, c_vp, c_vp, c_sz, c_vp]),
}


class OktChunk(ctypes.Structure):
    _fields_ = [("src", c_u32), ("dst", c_u32), ("src_offset", c_u64), ("dst_offset", c_u64),
                ("count", c_u64)]


class OktError(RuntimeError):
    def __init__(self, call: str, status: int, text: str):
        super().__init__(f"{call} failed: {text} (status {status})")
        self.status = status


def library_path() -> str:
    return os.path.join(_HERE, "libokt.so")


def load_library() -> ctypes.CDLL:
    """Load libokt.so (built in-tree by paper_2201_07598_amd.build)."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise OktError("load_library", -100,
                           f"{path} is missing: run `python -m paper_2201_07598_amd.build`")
        # torch first: the library must bind to the HIP runtime torch brings along,
        # the one that owns the streams and the device memory it is handed
        _torch()
        lib = ctypes.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _LIB = lib
    return _LIB


def okt_status_string(status: int) -> str:
    return load_library().okt_status_string(int(status)).decode()


def okt_last_hip_error() -> str:
    return load_library().okt_last_hip_error().decode()


def okt_time_next_kernel(start_event, stop_event) -> None:
    """torch.cuda.Event objects (already recorded once, so that they exist) or None."""
    load_library().okt_time_next_kernel(
        ctypes.c_void_p(start_event.cuda_event if start_event is not None else None),
        ctypes.c_void_p(stop_event.cuda_event if stop_event is not None else None))


def okt_debug_spin_limit(polls: int) -> None:
    """Test hook: polls a wait between workgroups may take (0 = built-in limit)."""
    load_library().okt_debug_spin_limit(int(polls))


def okt_debug_slot_min_n(n: int) -> None:
    """Test hook: shortest vector that takes the three-pass select (0 = built-in length)."""
    load_library().okt_debug_slot_min_n(int(n))


def okt_slot_min_n(accumulating: bool = False) -> int:
    """Vectors at least this long take the three-pass form (plain selects, or the
    calls that form the accumulator on the way)."""
    return load_library().okt_slot_min_n(1 if accumulating else 0)


def okt_version() -> int:
    return load_library().okt_version()


def okt_workspace_bytes(n_max: int, P_max: int = 0) -> int:
    return load_library().okt_workspace_bytes(int(n_max), int(P_max))


def okt_sparse_reduce_batch_workspace_bytes(B: int, P: int, max_width: int) -> int:
    return load_library().okt_sparse_reduce_batch_workspace_bytes(int(B), int(P), int(max_width))


# --------------------------------------------------------------------------
def _torch():
    import torch
    return torch


def _ptr(t, dtype, name, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise TypeError(f"{name} is required")
    torch = _torch()
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor (device memory)")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise TypeError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = _torch().cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(call, status):
    if status != 0:
        text = okt_status_string(status)
        if status == -3:
            text += ": " + okt_last_hip_error()
        raise OktError(call, status, text)


def _u64(torch):
    # device-side uint64 scalars are carried in int64 tensors (same bytes)
    return torch.int64


def _u32(torch):
    return torch.int32


def okt_residual_accumulate(grad, residual_inout, lr: float, stream=None) -> None:
    torch = _torch()
    _ptr(residual_inout, torch.float32, "residual_inout")
    _ptr(grad, torch.float32, "grad")
    n = residual_inout.numel()
    if grad.numel() != n:
        raise ValueError("grad and residual must have the same length")
    _check("okt_residual_accumulate", load_library().okt_residual_accumulate(
        _ptr(grad, torch.float32, "grad"), _ptr(residual_inout, torch.float32, "residual_inout"),
        float(lr), n, _stream(stream)))


STREAM_SUM_PARTIALS = 2048     # OKT_STREAM_SUM_PARTIALS


def okt_stream_copy(src, dst, stream=None) -> None:
    """Measurement only: dst[:] = src with the library's plain copy kernel."""
    torch = _torch()
    if src.numel() != dst.numel():
        raise ValueError("src and dst must have the same length")
    _check("okt_stream_copy", load_library().okt_stream_copy(
        _ptr(src, torch.float32, "src"), _ptr(dst, torch.float32, "dst"), src.numel(),
        _stream(stream)))


def okt_stream_sum(src, partials_out, stream=None) -> None:
    """Measurement only: one read of src; STREAM_SUM_PARTIALS fp32 partial sums out."""
    torch = _torch()
    if partials_out.numel() < STREAM_SUM_PARTIALS:
        raise ValueError(f"partials_out needs {STREAM_SUM_PARTIALS} elements")
    _check("okt_stream_sum", load_library().okt_stream_sum(
        _ptr(src, torch.float32, "src"), src.numel(),
        _ptr(partials_out, torch.float32, "partials_out"), _stream(stream)))


def okt_stream_gather(idx_cat, val_cat, chunk_off, lo_hi, B: int, P: int, max_width: int, idx_out,
                      val_out, capacity: int, ws, stream=None) -> None:
    """Measurement only: the batched reduce's reads and writes without its arithmetic."""
    torch = _torch()
    if chunk_off.numel() < B * (P + 1) or lo_hi.numel() < 2 * B:
        raise ValueError("chunk_off needs B*(P+1), lo_hi 2*B elements")
    if idx_out.numel() < B * capacity or val_out.numel() < B * capacity:
        raise ValueError("output buffers need B*capacity elements")
    _check("okt_stream_gather", load_library().okt_stream_gather(
        _ptr(idx_cat, _u32(torch), "idx_cat"), _ptr(val_cat, torch.float32, "val_cat"),
        _ptr(chunk_off, _u64(torch), "chunk_off"), _ptr(lo_hi, _u32(torch), "lo_hi"),
        int(B), int(P), int(max_width),
        _ptr(idx_out, _u32(torch), "idx_out"), _ptr(val_out, torch.float32, "val_out"),
        int(capacity), _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream(stream)))


def okt_topk_threshold_exact(acc, k: int, threshold_out, count_ge_out, ws, stream=None) -> None:
    torch = _torch()
    if threshold_out.numel() < 1 or count_ge_out.numel() < 1:
        raise ValueError("threshold_out and count_ge_out need one element")
    _check("okt_topk_threshold_exact", load_library().okt_topk_threshold_exact(
        _ptr(acc, torch.float32, "acc"), acc.numel(), int(k),
        _ptr(threshold_out, torch.float32, "threshold_out"),
        _ptr(count_ge_out, _u64(torch), "count_ge_out"),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream(stream)))


def okt_threshold_select(acc_inout, threshold, idx_out, val_out, nnz_out, ws, capacity=None,
                         stream=None, _call="okt_threshold_select") -> None:
    torch = _torch()
    cap = min(idx_out.numel(), val_out.numel()) if capacity is None else int(capacity)
    if cap > idx_out.numel() or cap > val_out.numel():
        raise ValueError("capacity exceeds the output buffers")
    if nnz_out.numel() < 2 or threshold.numel() < 1:
        raise ValueError("nnz_out needs two elements, threshold one")
    _check(_call, getattr(load_library(), _call)(
        _ptr(acc_inout, torch.float32, "acc_inout"), acc_inout.numel(),
        _ptr(threshold, torch.float32, "threshold"),
        _ptr(idx_out, _u32(torch), "idx_out"), _ptr(val_out, torch.float32, "val_out"), cap,
        _ptr(nnz_out, _u64(torch), "nnz_out"), _ptr(ws, torch.uint8, "ws"), ws.numel(),
        _stream(stream)))


def okt_threshold_select_noalloc(acc_inout, threshold, idx_out, val_out, nnz_out, capacity=None,
                                 stream=None) -> None:
    """okt_threshold_select on the library's own scan state: no workspace argument."""
    torch = _torch()
    cap = min(idx_out.numel(), val_out.numel()) if capacity is None else int(capacity)
    if cap > idx_out.numel() or cap > val_out.numel():
        raise ValueError("capacity exceeds the output buffers")
    if nnz_out.numel() < 2 or threshold.numel() < 1:
        raise ValueError("nnz_out needs two elements, threshold one")
    _check("okt_threshold_select_noalloc", load_library().okt_threshold_select_noalloc(
        _ptr(acc_inout, torch.float32, "acc_inout"), acc_inout.numel(),
        _ptr(threshold, torch.float32, "threshold"),
        _ptr(idx_out, _u32(torch), "idx_out"), _ptr(val_out, torch.float32, "val_out"), cap,
        _ptr(nnz_out, _u64(torch), "nnz_out"), _stream(stream)))


def okt_threshold_select_copy(acc, threshold, idx_out, val_out, nnz_out, ws, capacity=None,
                              stream=None) -> None:
    okt_threshold_select(acc, threshold, idx_out, val_out, nnz_out, ws, capacity=capacity,
                         stream=stream, _call="okt_threshold_select_copy")


def okt_accumulate_select(grad, residual_inout, lr: float, threshold, idx_out, val_out, nnz_out, ws,
                          capacity=None, stream=None) -> None:
    torch = _torch()
    _ptr(residual_inout, torch.float32, "residual_inout")
    if grad.numel() != residual_inout.numel():
        raise ValueError("grad and residual must have the same length")
    cap = min(idx_out.numel(), val_out.numel()) if capacity is None else int(capacity)
    if cap > idx_out.numel() or cap > val_out.numel():
        raise ValueError("capacity exceeds the output buffers")
    if nnz_out.numel() < 2 or threshold.numel() < 1:
        raise ValueError("nnz_out needs two elements, threshold one")
    _check("okt_accumulate_select", load_library().okt_accumulate_select(
        _ptr(grad, torch.float32, "grad"), residual_inout.data_ptr(), float(lr),
        residual_inout.numel(), _ptr(threshold, torch.float32, "threshold"),
        _ptr(idx_out, _u32(torch), "idx_out"), _ptr(val_out, torch.float32, "val_out"), cap,
        _ptr(nnz_out, _u64(torch), "nnz_out"), _ptr(ws, torch.uint8, "ws"), ws.numel(),
        _stream(stream)))


def okt_accumulate_topk_select(grad, residual_inout, lr: float, k: int, threshold_out, count_ge_out,
                               idx_out, val_out, nnz_out, ws, capacity=None, stream=None) -> None:
    torch = _torch()
    _ptr(residual_inout, torch.float32, "residual_inout")
    if grad.numel() != residual_inout.numel():
        raise ValueError("grad and residual must have the same length")
    cap = min(idx_out.numel(), val_out.numel()) if capacity is None else int(capacity)
    if cap > idx_out.numel() or cap > val_out.numel():
        raise ValueError("capacity exceeds the output buffers")
    if nnz_out.numel() < 2 or threshold_out.numel() < 1 or count_ge_out.numel() < 1:
        raise ValueError("nnz_out needs two elements, threshold_out and count_ge_out one")
    _check("okt_accumulate_topk_select", load_library().okt_accumulate_topk_select(
        _ptr(grad, torch.float32, "grad"), residual_inout.data_ptr(), float(lr),
        residual_inout.numel(), int(k), _ptr(threshold_out, torch.float32, "threshold_out"),
        _ptr(count_ge_out, _u64(torch), "count_ge_out"),
        _ptr(idx_out, _u32(torch), "idx_out"), _ptr(val_out, torch.float32, "val_out"), cap,
        _ptr(nnz_out, _u64(torch), "nnz_out"), _ptr(ws, torch.uint8, "ws"), ws.numel(),
        _stream(stream)))


def okt_region_partition(idx, nnz, n: int, R: int, bounds_out, offsets_out, stream=None) -> None:
    torch = _torch()
    if bounds_out.numel() < R + 1 or offsets_out.numel() < R + 1:
        raise ValueError("bounds_out and offsets_out need R+1 elements")
    _check("okt_region_partition", load_library().okt_region_partition(
        _ptr(idx, _u32(torch), "idx"), _ptr(nnz, _u64(torch), "nnz"), int(n), int(R),
        _ptr(bounds_out, _u32(torch), "bounds_out"),
        _ptr(offsets_out, _u64(torch), "offsets_out"), _stream(stream)))


def okt_sparse_reduce(idx_cat, val_cat, chunk_off, lo: int, hi: int, idx_out, val_out, nnz_out,
                      ws, dense_out=None, capacity=None, stream=None) -> None:
    torch = _torch()
    P = chunk_off.numel() - 1
    cap = min(idx_out.numel(), val_out.numel()) if capacity is None else int(capacity)
    if cap > idx_out.numel() or cap > val_out.numel():
        raise ValueError("capacity exceeds the output buffers")
    if dense_out is not None and dense_out.numel() < hi - lo:
        raise ValueError("dense_out needs hi-lo elements")
    if nnz_out.numel() < 2 or val_cat.numel() != idx_cat.numel():
        raise ValueError("nnz_out needs two elements; idx_cat and val_cat the same length")
    _check("okt_sparse_reduce", load_library().okt_sparse_reduce(
        _ptr(idx_cat, _u32(torch), "idx_cat"), _ptr(val_cat, torch.float32, "val_cat"),
        _ptr(chunk_off, _u64(torch), "chunk_off"), P, int(lo), int(hi),
        _ptr(idx_out, _u32(torch), "idx_out"), _ptr(val_out, torch.float32, "val_out"), cap,
        _ptr(nnz_out, _u64(torch), "nnz_out"),
        _ptr(dense_out, torch.float32, "dense_out", allow_none=True),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream(stream)))


def okt_sparse_reduce_batch(idx_cat, val_cat, chunk_off, lo_hi, B: int, P: int, max_width: int,
                            idx_out, val_out, capacity: int, nnz_out, ws, dense_out=None,
                            stream=None) -> None:
    torch = _torch()
    if chunk_off.numel() < B * (P + 1) or lo_hi.numel() < 2 * B or nnz_out.numel() < 2 * B:
        raise ValueError("chunk_off needs B*(P+1), lo_hi and nnz_out 2*B elements")
    if idx_out.numel() < B * capacity or val_out.numel() < B * capacity:
        raise ValueError("output buffers need B*capacity elements")
    if dense_out is not None and dense_out.numel() < B * max_width:
        raise ValueError("dense_out needs B*max_width elements")
    _check("okt_sparse_reduce_batch", load_library().okt_sparse_reduce_batch(
        _ptr(idx_cat, _u32(torch), "idx_cat"), _ptr(val_cat, torch.float32, "val_cat"),
        _ptr(chunk_off, _u64(torch), "chunk_off"), _ptr(lo_hi, _u32(torch), "lo_hi"),
        int(B), int(P), int(max_width),
        _ptr(idx_out, _u32(torch), "idx_out"), _ptr(val_out, torch.float32, "val_out"),
        int(capacity), _ptr(nnz_out, _u64(torch), "nnz_out"),
        _ptr(dense_out, torch.float32, "dense_out", allow_none=True),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream(stream)))


def okt_coo_threshold_select(idx_in, val_in, nnz_in, threshold, idx_out, val_out, nnz_out, ws,
                             max_nnz=None, capacity=None, stream=None) -> None:
    torch = _torch()
    bound = min(idx_in.numel(), val_in.numel()) if max_nnz is None else int(max_nnz)
    if bound > idx_in.numel() or bound > val_in.numel():
        raise ValueError("max_nnz exceeds the input buffers")
    cap = min(idx_out.numel(), val_out.numel()) if capacity is None else int(capacity)
    if cap > idx_out.numel() or cap > val_out.numel():
        raise ValueError("capacity exceeds the output buffers")
    if nnz_out.numel() < 2 or threshold.numel() < 1 or nnz_in.numel() < 1:
        raise ValueError("nnz_out needs two elements, threshold and nnz_in one")
    _check("okt_coo_threshold_select", load_library().okt_coo_threshold_select(
        _ptr(idx_in, _u32(torch), "idx_in"), _ptr(val_in, torch.float32, "val_in"),
        _ptr(nnz_in, _u64(torch), "nnz_in"), bound, _ptr(threshold, torch.float32, "threshold"),
        _ptr(idx_out, _u32(torch), "idx_out"), _ptr(val_out, torch.float32, "val_out"), cap,
        _ptr(nnz_out, _u64(torch), "nnz_out"), _ptr(ws, torch.uint8, "ws"), ws.numel(),
        _stream(stream)))


def okt_index_intersect_restore(residual_inout, local_idx, local_val, local_nnz, global_idx,
                                global_nnz, count_out, ws, indexes_out=None, max_local=None,
                                max_global=None, stream=None) -> None:
    torch = _torch()
    bound_l = min(local_idx.numel(), local_val.numel()) if max_local is None else int(max_local)
    bound_g = global_idx.numel() if max_global is None else int(max_global)
    if bound_l > local_idx.numel() or bound_l > local_val.numel() or bound_g > global_idx.numel():
        raise ValueError("max_local / max_global exceed the input buffers")
    if indexes_out is not None and indexes_out.numel() < bound_l:
        raise ValueError("indexes_out needs max_local elements")
    if count_out.numel() < 1 or local_nnz.numel() < 1 or global_nnz.numel() < 1:
        raise ValueError("count_out, local_nnz and global_nnz need one element")
    _check("okt_index_intersect_restore", load_library().okt_index_intersect_restore(
        _ptr(residual_inout, torch.float32, "residual_inout"), residual_inout.numel(),
        _ptr(local_idx, _u32(torch), "local_idx"), _ptr(local_val, torch.float32, "local_val"),
        _ptr(local_nnz, _u64(torch), "local_nnz"), bound_l,
        _ptr(global_idx, _u32(torch), "global_idx"), _ptr(global_nnz, _u64(torch), "global_nnz"),
        bound_g, _ptr(indexes_out, _u32(torch), "indexes_out", allow_none=True),
        _ptr(count_out, _u64(torch), "count_out"), _ptr(ws, torch.uint8, "ws"), ws.numel(),
        _stream(stream)))


def okt_index_intersect_zero(acc_inout, local_idx, local_nnz, global_idx, global_nnz, count_out, ws,
                             indexes_out=None, max_local=None, max_global=None,
                             stream=None) -> None:
    torch = _torch()
    bound_l = local_idx.numel() if max_local is None else int(max_local)
    bound_g = global_idx.numel() if max_global is None else int(max_global)
    if bound_l > local_idx.numel() or bound_g > global_idx.numel():
        raise ValueError("max_local / max_global exceed the input buffers")
    if indexes_out is not None and indexes_out.numel() < bound_l:
        raise ValueError("indexes_out needs max_local elements")
    if count_out.numel() < 1 or local_nnz.numel() < 1 or global_nnz.numel() < 1:
        raise ValueError("count_out, local_nnz and global_nnz need one element")
    _check("okt_index_intersect_zero", load_library().okt_index_intersect_zero(
        _ptr(acc_inout, torch.float32, "acc_inout"), acc_inout.numel(),
        _ptr(local_idx, _u32(torch), "local_idx"), _ptr(local_nnz, _u64(torch), "local_nnz"),
        bound_l, _ptr(global_idx, _u32(torch), "global_idx"),
        _ptr(global_nnz, _u64(torch), "global_nnz"), bound_g,
        _ptr(indexes_out, _u32(torch), "indexes_out", allow_none=True),
        _ptr(count_out, _u64(torch), "count_out"), _ptr(ws, torch.uint8, "ws"), ws.numel(),
        _stream(stream)))


def okt_sparse_reduce_segments(idx_cat, val_cat, seg_begin, seg_end, P: int, lo: int, hi: int,
                               idx_out, val_out, nnz_out, ws, dense_out=None, capacity=None,
                               stream=None) -> None:
    torch = _torch()
    cap = min(idx_out.numel(), val_out.numel()) if capacity is None else int(capacity)
    if cap > idx_out.numel() or cap > val_out.numel():
        raise ValueError("capacity exceeds the output buffers")
    if seg_begin.numel() < P or seg_end.numel() < P:
        raise ValueError("seg_begin and seg_end need P elements")
    if dense_out is not None and dense_out.numel() < hi - lo:
        raise ValueError("dense_out needs hi-lo elements")
    if nnz_out.numel() < 2 or val_cat.numel() != idx_cat.numel():
        raise ValueError("nnz_out needs two elements; idx_cat and val_cat the same length")
    _check("okt_sparse_reduce_segments", load_library().okt_sparse_reduce_segments(
        _ptr(idx_cat, _u32(torch), "idx_cat"), _ptr(val_cat, torch.float32, "val_cat"),
        _ptr(seg_begin, _u64(torch), "seg_begin"), _ptr(seg_end, _u64(torch), "seg_end"),
        int(P), int(lo), int(hi),
        _ptr(idx_out, _u32(torch), "idx_out"), _ptr(val_out, torch.float32, "val_out"), cap,
        _ptr(nnz_out, _u64(torch), "nnz_out"),
        _ptr(dense_out, torch.float32, "dense_out", allow_none=True),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream(stream)))


def okt_balance_plan(sizes):
    """Host-side: returns (triggered, [(src, dst, src_offset, dst_offset, count), ...])."""
    P = len(sizes)
    h_sizes = (c_u64 * max(P, 1))(*[int(x) for x in sizes])
    plan = (OktChunk * max(2 * P, 1))()
    n = c_u32(0)
    triggered = c_int(0)
    _check("okt_balance_plan", load_library().okt_balance_plan(
        ctypes.cast(h_sizes, c_vp), P, ctypes.cast(plan, c_vp), 2 * P, ctypes.cast(ctypes.pointer(n), c_vp),
        ctypes.cast(ctypes.pointer(triggered), c_vp)))
    return bool(triggered.value), [(c.src, c.dst, c.src_offset, c.dst_offset, c.count)
                                   for c in plan[:n.value]]
