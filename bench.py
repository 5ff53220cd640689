#!/usr/bin/env python3
"""Decode throughput of the budgeted KV cache on one MI355X.

A "step" is one pass of the whole hot path over one batch: sc_decode_step (append + budgeted
attention + importance-record update, one kernel) followed by sc_compress whenever the cache
has reached its trigger size.  The workload is the OPT-6.7B-shaped single layer (batch 16,
32 heads, head_dim 128, fp16, 1024-token prompt put through sc_prefill, then decoding
under budget 1024).  Because one layer's cache (269 MB) is about the size of the chip's
last-level cache and is re-read every step, R independent cache instances are stepped
round-robin (as the layers of a model would be), so every step finds its cache cold in HBM.
tokens/s = batch * steps / wall time, a step being one layer-instance step.

Prints ONE JSON line: metric / value / unit (whole-job decode tokens/s, inputs resident in
HBM), ms_per_step, config (the workload), roofline (algorithmic bytes per decode-attention
launch / its average duration from HIP events on the launch stream, against the 8 TB/s HBM
peak; traffic = HBM bytes per launch from rocprofv3 counters where measured) and cpu_baseline
(the CPU oracle timed on the host cores on the same decode phase).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 matrix peak
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix peak
HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak

# HBM bytes per decode-attention launch measured with rocprofv3 counters (FETCH_SIZE x 2.000 +
# WRITE_SIZE x 1.000, factors from a copy of known size) for the headline workload in this
# launch configuration; see profiles/attn_rows_fp16_cfg2_hbm_traffic.md.  Other workloads: null.
MEASURED_TRAFFIC_BYTES = {"cfg2-opt6.7b-fp16": 253.59e6}


def algorithmic_bytes(wl, n: int) -> int:
    """Bytes one decode-attention launch must move when n rows are resident after the append:
    per unit, n rows of K and of V (plus their 4-bit scale/zero words), a 2-byte counter read
    and written per row, and the q / k_new / v_new / out vectors."""
    from paper_2305_17118_amd.workloads import KV_F32, KV_F16
    d = wl.head_dim
    if wl.kv_dtype == KV_F32:
        row, e_io = d * 4, 4
    elif wl.kv_dtype == KV_F16:
        row, e_io = d * 2, 2
    else:
        row, e_io = d // 2 + (d // 64) * 4, 2
    if isinstance(n, (list, tuple)):  # ragged batch: resident rows per sequence
        return wl.heads * sum(nb * (2 * row + 4) + 4 * d * e_io for nb in n)
    return wl.units * (n * (2 * row + 4) + 4 * d * e_io)


def ragged_prompt_lengths(wl):
    """The length mix of the ragged variant: prompts spread evenly from a quarter of the
    workload's prompt length up to all of it (sequence 0 the shortest), so that the sequences sit
    at different points of the compression cycle and see different thresholds."""
    lo, hi = wl.prompt // 4, wl.prompt
    if wl.batch == 1:
        return [hi]
    return [lo + (hi - lo) * b // (wl.batch - 1) for b in range(wl.batch)]


def rows_after_step(wl, t: int) -> int:
    """Resident rows of a sequence right after its step t (hard-cap trigger)."""
    n_trig, m = wl.budget + 1, wl.drop
    return t if t <= n_trig else n_trig - m + (t - n_trig - 1) % m + 1


def cpu_baseline(wl, sample_units: int, sample_steps: int) -> dict:
    """Time the CPU oracle, as it stands, on a bounded sample of the same workload: the first
    `sample_units` units, full streamed prompt (untimed), then `sample_steps` decode steps with
    their compressions (timed).  Scaled linearly to the full unit count (units are independent
    and identically distributed)."""
    from oracle.sco import Oracle, OracleConfig
    from paper_2305_17118_amd.workloads import streams

    units = list(range(min(sample_units, wl.units)))
    cores = os.cpu_count() or 1
    sample_steps = min(sample_steps, wl.decode)
    q, k, v = streams(wl, units, steps=wl.prompt + sample_steps, threads=min(cores, 16))
    o = Oracle(OracleConfig(1, len(units), wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history,
                            wl.drop), nthreads=cores)
    for s in range(wl.prompt):
        _, _, due = o.step(q[:, s], k[:, s], v[:, s], want_probs=False)
        if due:
            o.compress()
    t0 = time.perf_counter()
    for s in range(wl.prompt, wl.prompt + sample_steps):  # noqa: E501
        _, _, due = o.step(q[:, s], k[:, s], v[:, s], want_probs=False)
        if due:
            o.compress()
    dt = time.perf_counter() - t0
    frac = len(units) / wl.units
    return {
        "value": wl.batch * sample_steps / (dt / frac),
        "unit": "tokens/s",
        "cores": min(cores, len(units)),
        "kind": "oracle",
        "sample": "%d of %d units, %d decode steps after the full %d-token streamed prompt, "
                  "%.1f s of CPU time measured, scaled by unit count" % (
                      len(units), wl.units, sample_steps, wl.prompt, dt),
    }


def prefill_work(wl):
    """Algorithmic work of one prompt pass -> (flops, bytes).  The prompt is cut into runs that
    end at the steps t = n_trig + k*m (after which a compression is due); a run of c positions
    that finds n0 rows resident costs, per unit,
      flops: position i attends over n0 + i + 1 rows, 2*d multiply-adds for the score and 2*d
             for P.V per row (the recomputation of the scores in the counting pass is not
             counted);
      bytes: the n0 + c visible K and V rows read once, the c new K and V rows written, c query
             rows read and c output rows written, a 16-bit counter read and written per visible
             row when the run counts (4-bit storage: plus the run's fp16 rows read to be
             quantised).
    The traffic of the compressions between runs is not counted (it depends on which rows go)."""
    from paper_2305_17118_amd.workloads import KV_F16, KV_F32
    d = wl.head_dim
    e_io = 4 if wl.kv_dtype == KV_F32 else 2
    row = d * 4 if wl.kv_dtype == KV_F32 else d * 2 if wl.kv_dtype == KV_F16 else d // 2 + (d // 64) * 4
    n_trig, m, E = wl.budget + 1, wl.drop, wl.history // wl.drop
    t = n = 0
    rows_attended = 0
    nbytes = 0
    while t < wl.prompt:
        a = t + 1 - n_trig
        epoch = (a + m - 1) // m if a >= 0 else -((-a) // m)
        c = min(wl.prompt - t, n_trig + epoch * m - t)
        rows_attended += c * n + c * (c + 1) // 2
        nbytes += (n + c) * 2 * row + c * 2 * row + c * d * e_io * 2
        if wl.kv_dtype not in (KV_F16, KV_F32):
            nbytes += c * 2 * d * 2  # the run's fp16 rows are read once more, to be quantised
        if epoch > -E:
            nbytes += (n + c) * 4
        t += c
        n += c
        if n == n_trig:
            n -= m
    return 4.0 * d * rows_attended * wl.units, float(nbytes) * wl.units


def bench_prefill(args, wl, dev) -> int:
    """One step = one sc_prefill call over the whole prompt of the workload (dense causal runs
    on the matrix cores, a compression whenever one is due), on a cache reset to empty."""
    import torch

    from paper_2305_17118_amd import binding as B
    from paper_2305_17118_amd.workloads import KV_F16, KV_F32, streams

    cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history,
                        wl.drop)
    P, d, U = wl.prompt, wl.head_dim, wl.units
    K, W = min(args.steps, 50), min(args.warmup, 3)
    q, k, v = (torch.from_numpy(a).to(dev) for a in streams(wl, steps=P, threads=16))
    cache = B.BudgetCache(cfg, dev)
    out = torch.empty(U, P, d, dtype=cache.io_dtype, device=dev)
    mfma_peak = MFMA_F32_PEAK_TFLOPS if wl.kv_dtype == KV_F32 else MFMA_F16_PEAK_TFLOPS

    def one_pass():
        cache.reset()
        cache.prefill(q, k, v, P, 0, out)

    for _ in range(W):
        one_pass()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(K):
        one_pass()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dev_ms = e0.elapsed_time(e1) / K
    flops, nbytes = prefill_work(wl)
    # which roofline binds: a run offers only m queries per K/V row read, so with per-unit caches
    # the prompt phase is bound by HBM unless m is large
    t_mfma, t_hbm = flops / (mfma_peak * 1e12), nbytes / (HBM_PEAK_GBS * 1e9)
    hbm_bound = t_hbm >= t_mfma
    tflops = flops / (dev_ms * 1e-3) / 1e12
    gbs = nbytes / (dev_ms * 1e-3) / 1e9
    res = {
        "metric": "prompt tokens/s into a budgeted KV cache", "value": wl.batch * P * K / wall,
        "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {KV_F32: "f32", KV_F16: "f16"}.get(wl.kv_dtype, "i4+f16"), "data": "synthetic",
        "config": {"workload": wl.name, "phase": "prefill", "batch": wl.batch, "heads": wl.heads,
                   "head_dim": d, "prompt": P, "budget": wl.budget, "recent": wl.recent,
                   "history": wl.history, "drop": wl.drop, "trigger": "hard_cap"},
        # every launch of the call (attention, select, compact) is inside the timed span, so
        # this is a lower bound on the attention kernel's own rate
        "roofline": {"bound": "hbm" if hbm_bound else "mfma",
                     "achieved": gbs if hbm_bound else tflops,
                     "peak": HBM_PEAK_GBS if hbm_bound else mfma_peak,
                     "unit": "GB/s" if hbm_bound else "TFLOP/s",
                     "frac": gbs / HBM_PEAK_GBS if hbm_bound else tflops / mfma_peak,
                     "traffic": None,
                     "kernel": "prefill_chunk_kernel (whole sc_prefill call timed)",
                     "call_ms_avg": dev_ms, "algorithmic_flops_per_call": flops,
                     "algorithmic_bytes_per_call": nbytes, "tflops": tflops,
                     "mfma_frac": tflops / mfma_peak, "gbs": gbs,
                     "hbm_frac": gbs / HBM_PEAK_GBS},
    }
    print(json.dumps(res))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1500)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (2 = headline)")
    ap.add_argument("--rotate", type=int, default=0, help="cache instances stepped round-robin "
                    "(0 = enough to cover three times the 256 MB last-level cache)")
    ap.add_argument("--phase", choices=("decode", "prefill"), default="decode",
                    help="decode = the headline metric; prefill = the prompt phase (fp16 workloads)")
    ap.add_argument("--window", choices=("auto", "ring"), default="auto",
                    help="importance record: bucket counters (auto, when w is a multiple of m) or "
                         "the exact one-bit-per-step ring")
    ap.add_argument("--record", choices=("online", "recompute"), default="online",
                    help="importance record kept during the steps (headline) or rebuilt at each "
                         "compression by replaying the last w queries (fp16 workloads)")
    ap.add_argument("--ragged", action="store_true",
                    help="decode phase with prompts of different lengths (every sequence on its own "
                         "clock: sc_prefill_ragged / sc_decode_step_ragged / sc_compress_ragged)")
    ap.add_argument("--no-events", action="store_true", help="skip the per-launch HIP events")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-units", type=int, default=512)
    ap.add_argument("--cpu-steps", type=int, default=1024)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (units are independent, so sharding over "
              "GPUs needs no collective and is not part of this build); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch

    from paper_2305_17118_amd import binding as B
    from paper_2305_17118_amd.workloads import CONFIGS, KV_F32, KV_F16, streams

    wl = CONFIGS[args.config - 1]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.phase == "prefill":
        return bench_prefill(args, wl, dev)
    cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history,
                        wl.drop, window_mode=B.SC_WINDOW_RING if args.window == "ring" else B.SC_WINDOW_AUTO,
                        record_mode=B.SC_RECORD_RECOMPUTE if args.record == "recompute" else B.SC_RECORD_ONLINE)
    ws_bytes = B.sc_workspace_bytes(cfg)
    R = args.rotate or min(8, max(1, -(-3 * 256 * 2 ** 20 // ws_bytes)))
    T, d, U = wl.total, wl.head_dim, wl.units
    steps_avail = R * wl.decode
    K, W = args.steps, args.warmup
    if W + K > steps_avail:
        K = steps_avail - W
        print("bench.py: only %d decode steps exist for %d instances; timing %d" % (steps_avail, R, K),
              file=sys.stderr)

    q, k, v = (torch.from_numpy(a).to(dev) for a in streams(wl, threads=16))
    caches = [B.BudgetCache(cfg, dev) for _ in range(R)]
    outs = [torch.empty(U, d, dtype=caches[0].io_dtype, device=dev) for _ in range(R)]
    plens = ragged_prompt_lengths(wl) if args.ragged else None
    for c in caches:
        if args.ragged:
            c.prefill_ragged(q, k, v, plens, T * d, None)
        else:
            c.prefill(q, k, v, wl.prompt, T * d, None)
    torch.cuda.synchronize()

    cursor = [wl.prompt] * R
    n_log = []
    # The loop below talks to the C ABI with raw addresses (no tensor views per step): on the
    # small workload the host would otherwise be slower than the kernel.
    eb = q.element_size()
    qp, kp, vp = q.data_ptr(), k.data_ptr(), v.data_ptr()
    handles = [c.handle for c in caches]
    out_ptrs = [o.data_ptr() for o in outs]
    stream = int(torch.cuda.current_stream(dev).cuda_stream)
    step_ragged, step_lock = B.sc_decode_step_ragged, B.sc_decode_step
    compress_ragged, compress_lock = B.sc_compress_ragged, B.sc_compress

    def one_step(i):
        r = i % R
        s = cursor[r]
        cursor[r] = s + 1
        off = s * d * eb
        if args.ragged:  # all sequences take part, each at its own t_b and n_b
            due = step_ragged(handles[r], qp + off, kp + off, vp + off, T * d, out_ptrs[r], None, None, stream)
            n_log.append([rows_after_step(wl, p + s - wl.prompt + 1) for p in plens])
            if due:
                compress_ragged(handles[r], None, None, stream)
            return 1 if due else 0
        due = step_lock(handles[r], qp + off, kp + off, vp + off, T * d, out_ptrs[r], None, stream)
        n_log.append(rows_after_step(wl, s + 1))
        if due:
            compress_lock(handles[r], None, None, stream)
        return due

    for i in range(W):
        one_step(i)
    n_log.clear()
    # HIP events on the launch stream bracket groups of GROUP consecutive decode-attention
    # launches; groups in which a compression ran are left out of the kernel average.
    GROUP = 10
    use_events = not args.no_events
    groups = []  # (start_event, end_event, launches, clean)
    compress_events = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    i = 0
    while i < K:
        g = min(GROUP, K - i)
        if use_events:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        dirty = 0
        for j in range(g):
            dirty += one_step(W + i + j)
        if use_events:
            e1.record()
            groups.append((e0, e1, g, dirty == 0, list(n_log[-g:])))
        compress_events += dirty
        i += g
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    if use_events:
        clean = [gr for gr in groups if gr[3]] or groups
        launches = sum(gr[2] for gr in clean)
        kern_ms = sum(gr[0].elapsed_time(gr[1]) for gr in clean) / launches
        alg = sum(algorithmic_bytes(wl, n) for gr in clean for n in gr[4]) / launches
        achieved = alg / (kern_ms * 1e-3) / 1e9
    else:
        alg = sum(algorithmic_bytes(wl, n) for n in n_log) / len(n_log)
        kern_ms, achieved = None, None
    if wl.kv_dtype in (KV_F32, KV_F16):
        kernel_name = "attn_rows_kernel"
    else:
        kernel_name = "attn_i4_mfma_kernel" if wl.head_dim == 128 else "attn_i4_kernel"
    res = {
        "metric": "decode tokens/s with budgeted KV cache",
        "value": wl.batch * K / wall,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": wall / K * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {0: "f32", 1: "f16", 2: "i4+f16"}[wl.kv_dtype],
        "data": "synthetic",
        "config": {
            "workload": wl.name, "batch": wl.batch, "heads": wl.heads, "head_dim": wl.head_dim,
            "prompt": wl.prompt, "decode": wl.decode, "budget": wl.budget, "recent": wl.recent,
            "history": wl.history, "drop": wl.drop, "trigger": "hard_cap", "window": args.window, "record": args.record,
            "cache_instances_round_robin": R, "compressions_in_timed_region": compress_events,
            "resident_rows_avg": (sum(sum(x) / len(x) for x in n_log) if args.ragged else sum(n_log)) / len(n_log),
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": None if achieved is None else achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name) if R == 3 and not args.ragged else None,
            "kernel": kernel_name, "kernel_ms_avg": kern_ms, "algorithmic_bytes_per_launch": alg,
        },
    }
    if args.ragged:
        res["config"]["ragged_prompt_lengths"] = plens
    if not args.no_cpu_baseline and not args.ragged:
        res["cpu_baseline"] = cpu_baseline(wl, args.cpu_units, args.cpu_steps)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
