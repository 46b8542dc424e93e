#!/usr/bin/env python3
"""Benchmark of the Ok-Topk one-GPU hot path on MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload: the ResNet-50-sized configuration (n = 25,557,032 fp32, 161 layer
segments, density 1 %, P = 16).  One STEP is one refresh period of the local
part of Ok-Topk SGD for one simulated worker, 10 iterations:

    iteration 0:     okt_accumulate_topk_select (accumulate, exact threshold and
                     select reading the gradient and the residual once: the same
                     results, bit for bit, as okt_residual_accumulate ->
                     okt_topk_threshold_exact -> okt_threshold_select)
                     -> okt_region_partition
    iterations 1-9:  okt_accumulate_select (the same accumulate and select, bit for
                     bit, in one pass: the threshold is reused, so it is known
                     before the accumulator is)
    every iteration: okt_sparse_reduce (P = 16 contributions over one region of n/16)

with the error-feedback residual carried from iteration to iteration and from
step to step.  `two_call_path` in the output is the same step made of the separate
calls (okt_residual_accumulate, okt_topk_threshold_exact at iteration 0,
okt_threshold_select).  Steps rotate over several independent simulated workers and the
reduce rotates over a pool of contribution sets, so that no vector is served
from the 256 MB Infinity Cache on re-use.  All inputs are seeded, synthetic and
resident in HBM before the timed region starts.

Prints ONE JSON line (see the driver's contract) with `roofline` (the dominant
kernel, timed with HIP events inside the timed region) and `cpu_baseline` (the
numpy oracle on the same workload, on the host cores).
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
ITERS_PER_STEP = 10
WORKLOAD = "cfg2"
CALLS = ("accumulate", "threshold", "select", "accumulate_topk_select", "accumulate_select",
         "partition", "reduce")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workers", type=int, default=4, help="independent simulated workers")
    ap.add_argument("--contrib-sets", type=int, default=24)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="leave the per-kernel HIP events out of the timed region")
    ap.add_argument("--reduce-dense", action="store_true",
                    help="also have every reduce of the step write the densified region "
                         "(a checking aid, not a step of the method)")
    ap.add_argument("--reduce-batch", type=int, default=0,
                    help="also time the batched reduce over this many regions (0 = auto)")
    return ap.parse_args()


class Worker:
    """Device state of one simulated worker."""

    def __init__(self, torch, okt, w, grads_host):
        dev = "cuda:0"
        self.grads = [torch.from_numpy(g).to(dev) for g in grads_host]
        self.residual = torch.zeros(w.n, dtype=torch.float32, device=dev)
        self.th = torch.zeros(1, dtype=torch.float32, device=dev)
        self.count_ge = torch.zeros(1, dtype=torch.int64, device=dev)
        self.cap = 4 * w.k
        self.idx = torch.zeros(self.cap, dtype=torch.int32, device=dev)
        self.val = torch.zeros(self.cap, dtype=torch.float32, device=dev)
        self.nnz = torch.zeros(2, dtype=torch.int64, device=dev)
        self.bounds = torch.zeros(w.P + 1, dtype=torch.int32, device=dev)
        self.offsets = torch.zeros(w.P + 1, dtype=torch.int64, device=dev)
        self.ws = torch.empty(okt.okt_workspace_bytes(w.n, w.P), dtype=torch.uint8, device=dev)


def main():
    args = parse()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; collectives and sharding across GPUs are "
            "not part of it (--gpus must be 1).")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2201_07598_amd as okt
    import workloads as wl

    okt.load_library()            # fails loudly when the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.WORKLOADS[WORKLOAD]
    n, k, P = w.n, w.k, w.P
    lo, hi = 0, n // P                         # the region this worker reduces
    t0 = time.time()

    # ---------------- inputs: generated on the host, uploaded before timing ----
    workers = []
    host_grads0 = None
    for r in range(args.workers):
        wr = w if r == 0 else dataclasses.replace(w, seed=w.seed + 7919 * r)
        grads = [wl.gradient(wr, it) for it in range(ITERS_PER_STEP)]
        if r == 0:
            host_grads0 = grads
        workers.append(Worker(torch, okt, w, grads))
        log(f"[bench] worker {r}: {ITERS_PER_STEP} gradients of {n} fp32 uploaded "
            f"({time.time() - t0:.1f}s)")
    contrib = []
    host_contrib0 = None
    for s in range(args.contrib_sets):
        ci, cv, co = wl.contributions(w, lo, hi, stream=s)
        if s == 0:
            host_contrib0 = (ci, cv, co)
        contrib.append((torch.from_numpy(ci.view(np.int32)).to(dev), torch.from_numpy(cv).to(dev),
                        torch.from_numpy(co.view(np.int64)).to(dev)))
    E = int(contrib[0][0].numel())
    red_idx = torch.zeros(E, dtype=torch.int32, device=dev)
    red_val = torch.zeros(E, dtype=torch.float32, device=dev)
    red_nnz = torch.zeros(2, dtype=torch.int64, device=dev)
    # the reduced region stays sparse, as in Alg.1 (its global top-k selection comes next);
    # the optional densified copy is a checking aid
    red_dense = torch.zeros(hi - lo, dtype=torch.float32, device=dev) if args.reduce_dense else None
    log(f"[bench] {args.contrib_sets} contribution sets (P={P}, E={E}) uploaded "
        f"({time.time() - t0:.1f}s)")

    stream = torch.cuda.current_stream()
    side = torch.cuda.Stream()                 # default priority; used by the overlapped variant only
    side_ws = torch.empty(okt.okt_workspace_bytes(hi - lo, P), dtype=torch.uint8, device=dev)
    counter = {"reduce": 0}

    def event_pairs(count):
        """Events that exist already (recorded once), for okt_time_next_kernel."""
        pairs = []
        for _ in range(count):
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record(stream)
            b.record(stream)
            pairs.append((a, b))
        return pairs

    def run_step(step, ev=None, only=None, fused=True, overlap=False, kernel_pairs=None,
                 nnz_log=None):
        """One step = ITERS_PER_STEP iterations of one worker.  `ev` collects
        (call, start_event, end_event) for the calls named in `only`.  overlap: the
        reduce of an iteration goes to a second stream (own workspace), where it runs
        beside the next iteration's accumulate+select, which does not depend on it."""
        st = workers[step % len(workers)]

        def timed(name, fn):
            # inside the timed region only one launch per step is bracketed (the
            # middle iteration): an event pair costs several microseconds
            if ev is not None and (only is None or (name in only and it == ITERS_PER_STEP // 2)):
                if kernel_pairs is not None:
                    # the library records the pair around the call's main kernel
                    a, b = kernel_pairs.pop()
                    okt.okt_time_next_kernel(a, b)
                    fn()
                else:
                    a = torch.cuda.Event(enable_timing=True)
                    b = torch.cuda.Event(enable_timing=True)
                    a.record(stream)
                    fn()
                    b.record(stream)
                ev.append((name, a, b))
            else:
                fn()

        for it in range(ITERS_PER_STEP):
            if fused and it == 0:
                # refresh iteration: accumulate, exact threshold and select in one call
                timed("accumulate_topk_select", lambda: okt.okt_accumulate_topk_select(
                    st.grads[it], st.residual, w.lr, k, st.th, st.count_ge, st.idx, st.val,
                    st.nnz, st.ws, capacity=st.cap))
            elif fused:
                # reuse iteration: the threshold is already known, one pass does both
                timed("accumulate_select", lambda: okt.okt_accumulate_select(
                    st.grads[it], st.residual, w.lr, st.th, st.idx, st.val, st.nnz, st.ws,
                    capacity=st.cap))
            else:
                timed("accumulate", lambda: okt.okt_residual_accumulate(
                    st.grads[it], st.residual, w.lr))
                if it == 0:
                    timed("threshold", lambda: okt.okt_topk_threshold_exact(
                        st.residual, k, st.th, st.count_ge, st.ws))
                timed("select", lambda: okt.okt_threshold_select(
                    st.residual, st.th, st.idx, st.val, st.nnz, st.ws, capacity=st.cap))
            if it == 0:
                timed("partition", lambda: okt.okt_region_partition(
                    st.idx, st.nnz, n, P, st.bounds, st.offsets))
            ci, cv, co = contrib[counter["reduce"] % len(contrib)]
            counter["reduce"] += 1
            if overlap:
                okt.okt_sparse_reduce(ci, cv, co, lo, hi, red_idx, red_val, red_nnz, side_ws,
                                      dense_out=red_dense, stream=side)
            else:
                timed("reduce", lambda: okt.okt_sparse_reduce(
                    ci, cv, co, lo, hi, red_idx, red_val, red_nnz, st.ws, dense_out=red_dense))
            if nnz_log is not None:          # untimed passes only: this reads back
                nnz_log.append(int(st.nnz.cpu().numpy().view(np.uint64)[1]))

    def summarise(ev, tail=1.0):
        """name -> (mean, median, count, min) of the event times in us; `tail` keeps only
        the last fraction of each call's samples (the first ones run cold)."""
        per = {}
        for name, a, b in ev:
            per.setdefault(name, []).append(a.elapsed_time(b) * 1e3)      # us
        out = {}
        for name, v in per.items():
            v = v[len(v) - max(1, int(len(v) * tail)):]
            out[name] = (float(np.mean(v)), float(np.median(v)), len(v), float(np.min(v)))
        return out

    # ---------------- warmup (instrumented: finds the dominant call) ----------
    ev = []
    for s in range(args.warmup):
        run_step(s, ev=ev)
    torch.cuda.synchronize()
    warm = summarise(ev, tail=0.5) if ev else {}
    nnz_seen = int(workers[0].nnz.cpu().numpy().view(np.uint64)[1]) if args.warmup else k
    calls_per_step = {"accumulate": 1, "threshold": 1, "select": 1, "accumulate_topk_select": 1,
                      "accumulate_select": ITERS_PER_STEP - 1, "partition": 1,
                      "reduce": ITERS_PER_STEP}
    if warm:
        dominant = max(warm, key=lambda c: warm[c][1] * calls_per_step[c])   # by median
    else:
        dominant = "accumulate"
    for c in CALLS:
        if c in warm:
            log(f"[bench] warmup {c:10s} mean {warm[c][0]:8.1f} us  median {warm[c][1]:8.1f} us "
                f"x{calls_per_step[c]}/step")
    log(f"[bench] dominant call: {dominant}")

    # ---------------- the timed region: exactly K steps -----------------------
    ev = None if args.no_kernel_events else []
    pairs = event_pairs(args.steps + 1) if ev is not None else None
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for s in range(args.steps):
        run_step(args.warmup + s, ev=ev, only=(dominant,), kernel_pairs=pairs)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    value = ITERS_PER_STEP * n / (ms_per_step * 1e-3)
    timed_stats = summarise(ev) if ev else {}

    # ---------------- per-call table (instrumented pass, outside the timing) --
    ev2 = []
    for s in range(max(4, args.warmup)):
        run_step(args.warmup + args.steps + s, ev=ev2)
    torch.cuda.synchronize()
    table = summarise(ev2)
    # the same pass again with the events around the main kernel of every call
    ev2k = []
    pairs2 = event_pairs(64 * max(4, args.warmup))
    for s in range(max(4, args.warmup)):
        run_step(args.warmup + args.steps + s, ev=ev2k, kernel_pairs=pairs2)
    torch.cuda.synchronize()
    table_kernel = summarise(ev2k)
    # the separate calls (not part of the step any more) for the same table
    ev2s, ev2sk = [], []
    pairs3 = event_pairs(64 * 4)
    for s in range(4):
        run_step(args.warmup + args.steps + s, ev=ev2s, fused=False)
    for s in range(4):
        run_step(args.warmup + args.steps + s, ev=ev2sk, fused=False, kernel_pairs=pairs3)
    torch.cuda.synchronize()
    for c, v in summarise(ev2s).items():
        table.setdefault(c, v)
    for c, v in summarise(ev2sk).items():
        table_kernel.setdefault(c, v)
    nnz_now = int(workers[0].nnz.cpu().numpy().view(np.uint64)[1])
    U = int(red_nnz.cpu().numpy().view(np.uint64)[1])

    # algorithmic bytes per launch of each call at this workload
    alg_bytes = {
        "accumulate": 12.0 * n,                               # read G, read eps, write acc
        "threshold": 4.0 * n,                                 # one read of acc is the floor
        "select": 4.0 * n + 12.0 * nnz_now,                   # read acc; idx, val, zero per entry
        "accumulate_select": 12.0 * n + 8.0 * nnz_now,        # read G, eps; write eps; idx, val
        "accumulate_topk_select": 12.0 * n + 12.0 * nnz_now,  # the same, and a zero per entry
        "reduce": 8.0 * E + 8.0 * U + (4.0 * (hi - lo) if args.reduce_dense else 0.0),   # entries in, union out
    }
    kernels = {}
    for c in CALLS:
        if c in table and c in alg_bytes:
            us = table[c][0]
            kernels[c] = {"us_per_call": round(us, 2), "us_median": round(table[c][1], 2),
                          "us_min": round(table[c][3], 2), "samples": table[c][2],
                          "calls_per_step": calls_per_step[c],
                          "algorithmic_bytes": alg_bytes[c],
                          "achieved_GBs": round(alg_bytes[c] / us * 1e-3, 1),
                          "frac_of_hbm_peak": round(alg_bytes[c] / us * 1e-3 / HBM_PEAK_GBS, 4)}
            if c in table_kernel:
                kernels[c]["us_main_kernel"] = round(table_kernel[c][0], 2)
        elif c in table:
            kernels[c] = {"us_per_call": round(table[c][0], 2), "calls_per_step": calls_per_step[c]}
    dom_us = timed_stats[dominant][0] if dominant in timed_stats else table[dominant][0]
    achieved = alg_bytes[dominant] / dom_us * 1e-3
    roofline = {"bound": "hbm", "kernel": dominant, "timed": "events recorded by the library right "
                "before and after the launch of the call's main kernel, one launch per step inside "
                "the timed region", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": read_traffic(dominant), "us_per_launch": round(dom_us, 2),
                "algorithmic_bytes_per_launch": alg_bytes[dominant]}

    # ---------------- the same step with two calls on the reuse iterations ----
    torch.cuda.synchronize()
    t_f = time.perf_counter()
    for s in range(args.steps):
        run_step(args.warmup + s, fused=False)
    torch.cuda.synchronize()
    ms_two = (time.perf_counter() - t_f) * 1e3 / args.steps
    ev3 = []
    for s in range(4):
        run_step(s, ev=ev3, only=("accumulate", "select"), fused=False)
    torch.cuda.synchronize()
    two = summarise(ev3)
    two_call_path = {"what": "the same step made of the separate calls: okt_residual_accumulate, "
                             "okt_topk_threshold_exact (iteration 0), okt_threshold_select",
                     "ms_per_step": ms_two, "value": ITERS_PER_STEP * n / (ms_two * 1e-3)}
    for c in ("accumulate", "select"):
        us = two[c][0]
        two_call_path[c] = {"us_per_call": round(us, 2), "algorithmic_bytes": alg_bytes[c],
                            "achieved_GBs": round(alg_bytes[c] / us * 1e-3, 1),
                            "frac_of_hbm_peak": round(alg_bytes[c] / us * 1e-3 / HBM_PEAK_GBS, 4)}

    # ---------------- the same step with the reduce on a second stream --------
    torch.cuda.synchronize()
    t_o = time.perf_counter()
    for s in range(args.steps):
        run_step(args.warmup + s, overlap=True)
    torch.cuda.synchronize()
    ms_overlap = (time.perf_counter() - t_o) * 1e3 / args.steps
    overlapped_path = {"what": "the same step with every okt_sparse_reduce enqueued on a second HIP "
                               "stream (own workspace), beside the next iteration's accumulate+select; "
                               "not the headline: one stream is",
                       "ms_per_step": ms_overlap, "value": ITERS_PER_STEP * n / (ms_overlap * 1e-3)}

    # ---------------- sustained reduce over a batch of regions ----------------
    reduce_batch = time_reduce_batch(args, torch, np, okt, wl, w, lo, hi)

    # ---------------- report only: how far a reused threshold drifts ----------
    # entries selected in each iteration of one more (untimed) step over k
    # (Sec. 5.2 reports the same ratio for real training runs), and the size of
    # the reduced union over the k/P entries one worker contributes (fill-in)
    nnz_log = []
    run_step(args.warmup + args.steps, nnz_log=nnz_log)
    sanity = {"selected_over_k_per_iteration": [round(v / k, 4) for v in nnz_log],
              "max_abs_drift": round(max(abs(v - k) / k for v in nnz_log), 4),
              "reduce_union_over_contribution": round(U / max(E // P, 1), 3)}

    # ---------------- plain streaming kernels: the achievable ceiling ---------
    ceilings = time_ceilings(torch, np, okt, w, workers)
    roofline["frac_of_copy_kernel"] = round(achieved / ceilings["copy"]["GBs"], 4)
    for c in kernels:
        if "achieved_GBs" in kernels[c] and c != "reduce":
            kernels[c]["frac_of_copy_kernel"] = round(
                kernels[c]["achieved_GBs"] / ceilings["copy"]["GBs"], 4)

    # ---------------- the global stage on this worker's share -----------------
    global_stage = time_global_stage(torch, np, okt, w, workers, red_idx, red_val, red_nnz)

    # ---------------- the oracle on the host cores ----------------------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(np, w, host_grads0, host_contrib0, lo, hi)

    out = {
        "metric": "gradient elems/s sparsified & sparse-reduce GB/s; % of MI355X HBM peak",
        "value": value, "unit": "elements/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg2: n=25,557,032 fp32 (ResNet-50-sized, 161 segments), "
                               "density 1% (k=255,571), 10 iterations per step with carried "
                               "residual, exact threshold at iteration 0 then reused (iterations "
                               "1-9 accumulate and select in one pass), P=16 contributions "
                               "reduced over one region of n/16",
                   "n": n, "k": k, "P": P, "iterations_per_step": ITERS_PER_STEP,
                   "simulated_workers": len(workers), "selected_per_iteration": nnz_now,
                   "reduce_entries_in": E, "reduce_union_out": U,
                   "kernel_events_in_timed_region": not args.no_kernel_events},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "reduce_batch": reduce_batch,
        "two_call_path": two_call_path,
        "overlapped_path": overlapped_path,
        "global_stage": global_stage,
        "ceilings": ceilings,
        "sanity": sanity,
    }
    print(json.dumps(out), flush=True)


def read_traffic(call):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
    as recorded in profiles/hbm_traffic_cfg2.txt ("<call> <fetch_bytes> <write_bytes>")."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_cfg2.txt")
    try:
        with open(path) as fh:
            for line in fh:
                parts = line.split()
                if len(parts) >= 3 and parts[0] == call:
                    return float(parts[1]) + float(parts[2])
    except OSError:
        pass
    return None


def time_reduce_batch(args, torch, np, okt, wl, w, lo, hi):
    """The same reduce kernel over B independent regions of the workload's shape in
    one launch, B sized so that the input exceeds 1 GB (far beyond the caches)."""
    dev = "cuda:0"
    P, m, width = w.P, w.m, hi - lo
    E1 = P * m
    B = args.reduce_batch or max(1, int(1.0e9 // (8 * E1)) + 1)
    base_sets = min(B, 32)            # distinct index patterns; values differ per region
    t0 = time.time()
    sets = [wl.contributions(w, 0, width, stream=1000 + s) for s in range(base_sets)]
    idx_cat = np.empty(B * E1, dtype=np.uint32)
    off = np.empty(B * (P + 1), dtype=np.uint64)
    lohi = np.empty(2 * B, dtype=np.uint32)
    for j in range(B):
        ci, _, co = sets[j % base_sets]
        rlo = j * width
        if rlo + width > 0xFFFFFFFF:
            rlo = (j % 16) * width
        idx_cat[j * E1:(j + 1) * E1] = ci + np.uint32(rlo)
        off[j * (P + 1):(j + 1) * (P + 1)] = co + np.uint64(j * E1)
        lohi[2 * j], lohi[2 * j + 1] = rlo, rlo + width
    d_idx = torch.from_numpy(idx_cat.view(np.int32)).to(dev)
    d_val = torch.randn(B * E1, dtype=torch.float32, device=dev) * 1e-3   # values: any fp32
    d_off = torch.from_numpy(off.view(np.int64)).to(dev)
    d_lohi = torch.from_numpy(lohi.view(np.int32)).to(dev)
    out_idx = torch.zeros(B * E1, dtype=torch.int32, device=dev)
    out_val = torch.zeros(B * E1, dtype=torch.float32, device=dev)
    nnz = torch.zeros(2 * B, dtype=torch.int64, device=dev)
    ws = torch.empty(okt.okt_sparse_reduce_batch_workspace_bytes(B, P, width), dtype=torch.uint8,
                     device=dev)
    log(f"[bench] reduce batch: B={B} regions, {B * E1} entries uploaded ({time.time() - t0:.1f}s)")
    times = []
    for rep in range(8):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        okt.okt_sparse_reduce_batch(d_idx, d_val, d_off, d_lohi, B, P, width, out_idx, out_val,
                                    E1, nnz, ws)
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) * 1e3)
    us = float(np.median(times[2:]))
    U = int(nnz.cpu().numpy().view(np.uint64)[1::2].sum())
    nbytes = 8.0 * B * E1 + 8.0 * U
    return {"regions": B, "entries_in": B * E1, "union_out": U, "us_per_launch": round(us, 1),
            "algorithmic_bytes": nbytes, "achieved_GBs": round(nbytes / us * 1e-3, 1),
            "frac_of_hbm_peak": round(nbytes / us * 1e-3 / HBM_PEAK_GBS, 4),
            "entries_per_s": B * E1 / (us * 1e-6)}


def time_ceilings(torch, np, okt, w, workers):
    """What plain streaming reaches on this GPU at this vector length: the library's
    copy kernel (4 B in + 4 B out per element) and its read-only sum (4 B in), over
    buffers that rotate (40 sources, 3 destinations: no launch finds its data in
    the 256 MB last-level cache), timed by the library's own event pair around the
    kernel like the roofline figure."""
    dev = "cuda:0"
    srcs = [g for st in workers for g in st.grads]
    dsts = [torch.empty(w.n, dtype=torch.float32, device=dev) for _ in range(3)]
    parts = torch.zeros(okt.STREAM_SUM_PARTIALS, dtype=torch.float32, device=dev)
    reps = 24
    out = {"n": w.n}
    for name, nbytes in (("copy", 8.0 * w.n), ("read_sum", 4.0 * w.n)):
        pairs = []
        for r in range(reps):
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record(); b.record()
            okt.okt_time_next_kernel(a, b)
            if name == "copy":
                okt.okt_stream_copy(srcs[r % len(srcs)], dsts[r % len(dsts)])
            else:
                okt.okt_stream_sum(srcs[r % len(srcs)], parts)
            pairs.append((a, b))
        torch.cuda.synchronize()
        us = float(np.median([a.elapsed_time(b) * 1e3 for a, b in pairs[4:]]))
        out[name] = {"us_per_launch": round(us, 2), "bytes": nbytes,
                     "GBs": round(nbytes / us * 1e-3, 1),
                     "frac_of_hbm_peak": round(nbytes / us * 1e-3 / HBM_PEAK_GBS, 4)}
    return out


def time_global_stage(torch, np, okt, w, workers, red_idx, red_val, red_nnz):
    """The calls that follow the reduce (outside the step): global threshold over the
    reduced values of the own region, global selection on that region, and
    indexes = local ∩ global with the residual restore.  The global index list is
    synthetic: every other locally selected index of this worker plus the
    selection of another simulated worker, about 1.5 k ascending indices."""
    dev = "cuda:0"
    st, other = workers[0], workers[1 % len(workers)]
    U = int(red_nnz.cpu().numpy().view(np.uint64)[0])
    L = int(st.nnz.cpu().numpy().view(np.uint64)[0])
    Lo = int(other.nnz.cpu().numpy().view(np.uint64)[0])
    kg = max(w.k // w.P, 1)
    g_idx = torch.unique(torch.cat([st.idx[:L:2], other.idx[:Lo]]), sorted=True).contiguous()
    G = int(g_idx.numel())
    g_nnz = torch.tensor([G], dtype=torch.int64, device=dev)
    gth = torch.zeros(1, dtype=torch.float32, device=dev)
    gcnt = torch.zeros(1, dtype=torch.int64, device=dev)
    sel_idx = torch.zeros(max(U, 1), dtype=torch.int32, device=dev)
    sel_val = torch.zeros(max(U, 1), dtype=torch.float32, device=dev)
    sel_nnz = torch.zeros(2, dtype=torch.int64, device=dev)
    inter = torch.zeros(st.cap, dtype=torch.int32, device=dev)
    icnt = torch.zeros(1, dtype=torch.int64, device=dev)
    vals = red_val[:U]
    sel_idx2 = torch.zeros(st.cap, dtype=torch.int32, device=dev)
    sel_val2 = torch.zeros(st.cap, dtype=torch.float32, device=dev)
    sel_nnz2 = torch.zeros(2, dtype=torch.int64, device=dev)
    calls = {
        "global_threshold": lambda: okt.okt_topk_threshold_exact(vals, min(kg, U), gth, gcnt, st.ws),
        "global_select": lambda: okt.okt_coo_threshold_select(
            red_idx, red_val, red_nnz[:1], gth, sel_idx, sel_val, sel_nnz, st.ws, max_nnz=U),
        "intersect_restore": lambda: okt.okt_index_intersect_restore(
            st.residual, st.idx, st.val, st.nnz[:1], g_idx, g_nnz, icnt, st.ws, indexes_out=inter,
            max_local=L),
        "intersect_zero": lambda: okt.okt_index_intersect_zero(
            other.residual, st.idx, st.nnz[:1], g_idx, g_nnz, icnt, st.ws, indexes_out=inter,
            max_local=L),
        "select_copy": lambda: okt.okt_threshold_select_copy(
            workers[2 % len(workers)].residual, st.th, sel_idx2, sel_val2, sel_nnz2, st.ws),
    }
    out = {"reduced_entries": U, "region_k": min(kg, U), "local_entries": L, "global_entries": G}
    for name, fn in calls.items():
        times = []
        for rep in range(10):
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b) * 1e3)
        out[name + "_us"] = round(float(np.median(times[2:])), 2)
    out["global_selected"] = int(sel_nnz.cpu().numpy().view(np.uint64)[1])
    out["intersection"] = int(icnt.cpu().numpy().view(np.uint64)[0])
    return out


def cpu_baseline(np, w, grads, contrib, lo, hi, seconds=12.0):
    """The numpy oracle, as it stands, on whole steps (10 iterations each) of the
    same workload and the same inputs, repeated until about `seconds` of CPU work
    are done; the threads numpy's own routines use (none of these do)."""
    from oracle import okt_oracle as orc
    t0 = time.perf_counter()
    res = np.zeros(w.n, dtype=np.float32)
    steps = 0
    while True:
        th = None
        for it in range(ITERS_PER_STEP):
            acc = orc.residual_accumulate(grads[it], res, w.lr)
            if it == 0:
                th, _ = orc.topk_threshold_exact(acc, w.k, method="partition")
            idx, val, res, _ = orc.threshold_select(acc, th, capacity=4 * w.k)
            if it == 0:
                orc.region_partition(idx, w.n, w.P)
            orc.sparse_reduce(contrib[0], contrib[1], contrib[2], lo, hi)
        steps += 1
        dt = time.perf_counter() - t0
        if dt >= seconds or steps >= 64:
            break
    # the two steps that split trivially (accumulate, select), static chunks over the
    # host's threads: the same oracle functions, called on slices
    from concurrent.futures import ThreadPoolExecutor
    threads = max(1, min(16, os.cpu_count() or 1))
    cuts = np.linspace(0, w.n, threads + 1).astype(np.int64)
    pres = np.zeros(w.n, dtype=np.float32)

    def chunk(j, it):
        a, b = int(cuts[j]), int(cuts[j + 1])
        acc = orc.residual_accumulate(grads[it][a:b], pres[a:b], w.lr)
        idx, _, r, _ = orc.threshold_select(acc, th)
        pres[a:b] = r
        return idx.size

    t1 = time.perf_counter()
    piters = 0
    with ThreadPoolExecutor(threads) as pool:
        while time.perf_counter() - t1 < seconds / 4 and piters < 200:
            list(pool.map(lambda j: chunk(j, piters % ITERS_PER_STEP), range(threads)))
            piters += 1
    pdt = time.perf_counter() - t1
    parallel = {"value": piters * w.n / pdt, "unit": "elements/s", "threads": threads,
                "sample": f"{piters} iterations of accumulate + select only (the steps that split "
                          "into independent chunks), one static chunk per thread"}
    model = ""
    try:
        with open("/proc/cpuinfo") as fh:
            model = next((ln.split(":", 1)[1].strip() for ln in fh if ln.startswith("model name")), "")
    except OSError:
        pass
    return {"value": steps * ITERS_PER_STEP * w.n / dt, "unit": "elements/s", "cores": 1,
            "kind": "oracle", "seconds": round(dt, 2), "host_cpu": model,
            "host_threads_available": os.cpu_count(),
            "parallel_accumulate_select": parallel,
            "sample": f"{steps} full steps (10 iterations each, n=25,557,032, residual carried) of "
                      "the same workload, numpy oracle, np.partition for the exact threshold"}


if __name__ == "__main__":
    main()
