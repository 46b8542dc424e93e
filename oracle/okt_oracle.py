"""CPU oracle for the Ok-Topk one-GPU hot path.  TEST INFRASTRUCTURE ONLY.

This file is the plain, slow, obviously-correct statement of what the
library calls compute.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import it; the product path never does, and this file
imports nothing from the HIP side.  It is written from the paper's
definitions with numpy; it is never tuned for speed.

What the paper fixes, and where:
  * accumulate        acc = eps + lr * G               (Algorithm 2, line 4)
  * top-k             the k components largest in absolute value  (Sec. 2)
  * exact threshold   sort the values, take the k-th largest      (Sec. 3.1.3)
  * threshold select  compare every component with the threshold,
                      package (index, value) into one consecutive
                      COO buffer                        (Sec. 3.1.3, 3.1.2)
  * residual update   eps = acc with the selected entries set to 0
                                                        (Algorithm 2, line 6)
  * balanced split    boundaries of P regions that balance the local
                      top-k entries                     (Sec. 3.1.1)
  * local reduction   plain sum of the sparse pieces received for
                      the own region                    (Sec. 3.1, 3.1.1)
  * global select     the same threshold comparison on the reduced
                      sparse values of the own region   (Sec. 3.1.2;
                                                        Algorithm 1, line 13)
  * indexes           local top-k indexes intersected with the global
                      top-k indexes                     (Algorithm 1, line 14)

Readings taken where the paper is silent (listed again in the design notes):
  magnitude order is the order of the fp32 bit pattern with the sign bit
  cleared; "at or above" the threshold (>=), so ties at the k-th value are all
  selected; two roundings in the accumulate (multiply, then add, no fused
  multiply-add); zeroed residual entries are +0.0; equal-count quantiles of
  the sorted local index list as balanced boundaries; the reduction keeps every
  index present in any contribution, sums in float64 in worker order and rounds
  once to fp32; no 1/P inside the reduction.

Precision: fp32 storage is the paper's (PyTorch fp32 tensors); integer work is
exact; the reduction accumulates in fp64.
"""
from __future__ import annotations

import numpy as np

_ABS_MASK = np.uint32(0x7FFFFFFF)


def magnitude_key(x: np.ndarray) -> np.ndarray:
    """Order-preserving integer key of |x| for fp32 x: the bit pattern with the
    sign cleared.  For finite values key(a) >= key(b) <=> |a| >= |b| (Sec. 2:
    top-k is by absolute value)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return x.view(np.uint32) & _ABS_MASK


def residual_accumulate(grad: np.ndarray, residual: np.ndarray, lr: float) -> np.ndarray:
    """acc[i] = fl32(residual[i] + fl32(lr * grad[i]))   (Algorithm 2, line 4)."""
    grad = np.asarray(grad, dtype=np.float32)
    residual = np.asarray(residual, dtype=np.float32)
    scaled = np.multiply(np.float32(lr), grad, dtype=np.float32)
    return np.add(residual, scaled, dtype=np.float32)


def topk_threshold_exact(acc: np.ndarray, k: int, method: str = "sort"):
    """The exact local top-k threshold (Sec. 3.1.3: sort, return the k-th largest).

    Returns (th, count_ge): th >= 0 is the fp32 whose magnitude key is the k-th
    largest key with multiplicity; count_ge = #{i : key(acc[i]) >= key(th)}.
    method="sort" is the definition written out; method="partition" replaces the
    full sort by the library's selection routine (same k-th order statistic) for
    vectors too long to sort in a test.
    """
    keys = magnitude_key(acc)
    n = keys.size
    if not 1 <= k <= n:
        raise ValueError("need 1 <= k <= n")
    if method == "sort":
        descending = np.sort(keys)[::-1]
        th_key = descending[k - 1]
    elif method == "partition":
        th_key = np.partition(keys, n - k)[n - k]
    else:
        raise ValueError(method)
    count_ge = int(np.count_nonzero(keys >= th_key))
    th = np.array([th_key], dtype=np.uint32).view(np.float32)[0]
    return th, count_ge


def threshold_select(acc: np.ndarray, th, capacity: int | None = None):
    """Threshold top-k selection, packaging and residual update.

    S = {i : |acc[i]| >= th} in ascending i (Sec. 3.1.3); (idx, val) is the
    consecutive COO buffer (Sec. 3.1.2); residual = acc with S zeroed
    (Algorithm 2, line 6).  With a capacity only the first `capacity` members of
    S are emitted and zeroed; the rest stay in the residual.
    Returns (idx uint32, val fp32, residual fp32, total = |S|).
    """
    acc = np.ascontiguousarray(acc, dtype=np.float32)
    th_key = magnitude_key(np.array([th], dtype=np.float32))[0]
    selected = np.flatnonzero(magnitude_key(acc) >= th_key)
    total = int(selected.size)
    if capacity is not None:
        selected = selected[:capacity]
    idx = selected.astype(np.uint32)
    val = acc[selected].copy()
    residual = acc.copy()
    residual[selected] = np.float32(0.0)
    return idx, val, residual, total


def region_partition(idx: np.ndarray, n: int, R: int):
    """Balanced split of [0, n) into R regions by the local top-k entries
    (Sec. 3.1.1), and the slice of the sorted COO that falls in each region.

    b[0] = 0, b[R] = n, b[r] = idx[floor(r * nnz / R)] for 0 < r < R (equal
    count quantiles; per-region counts differ by at most one).  Without any
    entry the split is the naive equal one, b[r] = floor(r * n / R).
    off[r] = number of entries with index < b[r]  (first COO position of region
    r), off[R] = nnz.
    Returns (b uint32[R+1], off uint64[R+1]).
    """
    idx = np.asarray(idx, dtype=np.uint32)
    nnz = int(idx.size)
    if R < 1:
        raise ValueError("R >= 1")
    b = np.zeros(R + 1, dtype=np.uint64)
    b[R] = n
    for r in range(1, R):
        if nnz > 0:
            b[r] = int(idx[(r * nnz) // R])
        else:
            b[r] = (r * n) // R
    off = np.zeros(R + 1, dtype=np.uint64)
    idx64 = idx.astype(np.uint64)
    for r in range(R):
        off[r] = int(np.count_nonzero(idx64 < b[r]))
    off[R] = nnz
    return b.astype(np.uint32), off


def sparse_reduce(idx_cat: np.ndarray, val_cat: np.ndarray, chunk_off: np.ndarray,
                  lo: int, hi: int):
    """Local reduction of P sparse contributions over region [lo, hi)
    (Sec. 3.1 semantic: plain sum; Sec. 3.1.1: each worker reduces its region).

    Dense float64 accumulator over the region, contributions added in worker
    order p = 0..P-1, entries outside the region ignored; the output holds every
    index present in any contribution (also when the sum is zero), ascending,
    with the sum rounded once to fp32.
    Returns dict(idx uint32[U], val fp32[U], dense fp32[hi-lo],
                 abs_sum float64[U]  (sum of |v| per output entry, for tolerances),
                 hits int64[U]       (contributions per output entry)).
    """
    idx_cat = np.asarray(idx_cat, dtype=np.uint32)
    val_cat = np.asarray(val_cat, dtype=np.float32)
    chunk_off = np.asarray(chunk_off, dtype=np.uint64)
    P = chunk_off.size - 1
    width = hi - lo
    D = np.zeros(width, dtype=np.float64)
    A = np.zeros(width, dtype=np.float64)
    hits = np.zeros(width, dtype=np.int64)
    for p in range(P):
        a, e = int(chunk_off[p]), int(chunk_off[p + 1])
        i = idx_cat[a:e].astype(np.int64)
        v = val_cat[a:e].astype(np.float64)
        inside = (i >= lo) & (i < hi)
        slot = i[inside] - lo
        # indices are distinct inside one chunk, so this is one add per slot
        D[slot] += v[inside]
        A[slot] += np.abs(v[inside])
        hits[slot] += 1
    present = np.flatnonzero(hits > 0)
    dense = D.astype(np.float32)
    return {
        "idx": (present + lo).astype(np.uint32),
        "val": dense[present].copy(),
        "dense": dense,
        "abs_sum": A[present].copy(),
        "hits": hits[present].copy(),
    }


def sparse_reduce_bucketed(buckets, lo: int, hi: int):
    """The local reduction taken bucket by bucket (Sec. 3.1.1: the exchange is cut
    into buckets so that the reduction of one overlaps the transfer of the next).
    `buckets` is a list of (idx_cat, val_cat, chunk_off) triples.  The partial
    result so far - already rounded to fp32 - joins the next bucket as one more
    contribution, listed last; each step is sparse_reduce.  Returns the final dict
    of sparse_reduce (abs_sum and hits of the last step only)."""
    partial = None
    for idx_cat, val_cat, chunk_off in buckets:
        idx_cat = np.asarray(idx_cat, dtype=np.uint32)
        val_cat = np.asarray(val_cat, dtype=np.float32)
        chunk_off = np.asarray(chunk_off, dtype=np.uint64)
        if partial is not None:
            idx_cat = np.concatenate([idx_cat, partial["idx"]])
            val_cat = np.concatenate([val_cat, partial["val"]])
            chunk_off = np.concatenate([chunk_off, [chunk_off[-1] + np.uint64(partial["idx"].size)]])
        partial = sparse_reduce(idx_cat, val_cat, chunk_off.astype(np.uint64), lo, hi)
    return partial


def balance_plan(sizes):
    """Data balancing before the allgatherv of the global top-k values
    (Sec. 3.1.2), taken when the largest buffer is more than four times the
    average (Sec. 5.3).  The P buffers in worker order are one list of T entries;
    balanced, worker j holds list positions [floor(j T / P), floor((j+1) T / P)).
    Every pair (old buffer i, new buffer j) whose ranges of list positions overlap
    gives one chunk (src, dst, src_offset, dst_offset, count).
    Returns (triggered, chunks in list order); no chunks when not triggered."""
    sizes = [int(x) for x in sizes]
    P, T = len(sizes), sum(sizes)
    triggered = max(sizes) * P > 4 * T
    if not triggered:
        return False, []
    old_first = [sum(sizes[:i]) for i in range(P)]
    new_first = [(j * T) // P for j in range(P + 1)]
    chunks = []
    for i in range(P):
        for j in range(P):
            a = max(old_first[i], new_first[j])
            b = min(old_first[i] + sizes[i], new_first[j + 1])
            if b > a:
                chunks.append((i, j, a - old_first[i], a - new_first[j], b - a))
    chunks.sort(key=lambda c: old_first[c[0]] + c[2])
    return True, chunks


def coo_threshold_select(idx: np.ndarray, val: np.ndarray, th, capacity: int | None = None):
    """Global top-k selection on a reduced sparse region (Sec. 3.1.2: each
    worker selects the global top-k values from the reduced top-k values of its
    region, by the global threshold, and packages them into a consecutive
    buffer; Algorithm 1, line 13).

    Keeps the entries (idx[j], val[j]) with |val[j]| >= th, in their order; the
    input is not changed.  With a capacity only the first `capacity` of them are
    emitted.  Returns (idx uint32, val fp32, total).
    """
    idx = np.asarray(idx, dtype=np.uint32)
    val = np.ascontiguousarray(val, dtype=np.float32)
    th_key = magnitude_key(np.array([th], dtype=np.float32))[0]
    keep = np.flatnonzero(magnitude_key(val) >= th_key)
    total = int(keep.size)
    if capacity is not None:
        keep = keep[:capacity]
    return idx[keep].copy(), val[keep].copy(), total


def index_intersection(local_idx: np.ndarray, global_idx: np.ndarray) -> np.ndarray:
    """indexes = local_topk_indexes ∩ global_topk_indexes (Algorithm 1, line 14):
    the positions whose local value contributed to a global top-k value.
    Ascending uint32."""
    local_idx = np.asarray(local_idx, dtype=np.uint32)
    global_idx = np.asarray(global_idx, dtype=np.uint32)
    member = np.isin(local_idx, global_idx)
    return np.sort(local_idx[member]).astype(np.uint32)


def residual_update(acc: np.ndarray, indexes: np.ndarray) -> np.ndarray:
    """eps = acc - acc(indexes) (Algorithm 2, line 6): the accumulator with the
    entries marked by `indexes` set to +0.0, everything else kept."""
    eps = np.array(acc, dtype=np.float32, copy=True)
    eps[np.asarray(indexes, dtype=np.int64)] = np.float32(0.0)
    return eps


def k_from_density(n: int, num: int, den: int) -> int:
    """k = ceil(n * density) with density = num/den = k/n (Sec. 3.1.3, Fig. 4)."""
    return -(-n * num // den)
