#!/usr/bin/env python3
"""Decode throughput of the budgeted KV cache on one MI355X.

A "step" is one pass of the whole hot path over one batch: sc_decode_step (append + budgeted
attention + importance-record update, one kernel) followed by sc_compress whenever the cache
has reached its trigger size.  The headline workload is the largest of the five that fits one
GPU, the OPT-66B-shaped single layer (batch 128, 72 heads, head_dim 128, fp16, 2048-token
prompt, then decoding under budget 683); `per_config` carries the same measurement for all
five workloads.  R >= 4 independent cache instances are stepped round-robin (as the layers of
a model would be), enough of them that every step finds its cache cold in HBM, and before the
timed region each instance is advanced (untimed) to a different phase of the m-step
compression cycle, so that a short run sees the same mix of resident rows as a long one.
tokens/s = batch * steps / wall time, a step being one layer-instance step.

Prints ONE JSON line: metric / value / unit (whole-job decode tokens/s, inputs resident in
HBM), ms_per_step, config (the workload), roofline (algorithmic bytes per decode-attention
launch / its average duration from HIP events on the launch stream, against the 8 TB/s HBM
peak; traffic = HBM bytes per launch from rocprofv3 counters when they were taken on exactly
these launches, else null), per_config (the five workloads) and cpu_baseline (the CPU oracle
timed on the host cores on a sample of the same decode phase).
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
# WRITE_SIZE x 1.000, factors from a copy of known size), keyed by workload and by the exact
# timed region they were taken on (steps, warmup, average resident rows): reported only when the
# current run timed the same launches, else `traffic` is null.  Sources: profiles/*hbm_traffic*.
MEASURED_TRAFFIC = {
    # workload: (steps, warmup, resident_rows_avg, bytes per launch)
    "cfg1-small-fp32": (200, 5, 225.94, 1536454),
    "cfg2-opt6.7b-fp16": (200, 5, 959.23, 254336938),
    "cfg3-opt13b-fp16": (200, 5, 346.75, 462236504),
    "cfg4-opt66b-fp16": (20, 5, 561.25, 2684583668),
    "cfg5-opt175b-int4": (200, 5, 574.29, 265963506),
}


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


def rows_after_step(wl, t: int, high_water: bool = False) -> int:
    """Resident rows of a sequence right after its step t (compression at B + 1 rows, or at
    B + m with the high-water trigger)."""
    m = wl.drop
    n_trig = wl.budget + m if high_water else wl.budget + 1
    return t if t <= n_trig else n_trig - m + (t - n_trig - 1) % m + 1


def cpu_baseline(wl, sample_units: int, sample_steps: int) -> dict:
    """Time the CPU oracle, as it stands, on a bounded sample of the same workload: the first
    `sample_units` units, full streamed prompt (untimed), then `sample_steps` decode steps with
    their compressions (timed).  Scaled linearly to the full unit count (units are independent
    and identically distributed)."""
    from oracle.sco import Oracle, OracleConfig
    from paper_2305_17118_amd.workloads import streams

    units = list(range(min(sample_units, wl.units)))
    cores = min(os.cpu_count() or 1, 16)  # the host share that goes with one GPU
    sample_steps = min(sample_steps, wl.decode)
    q, k, v = streams(wl, units, steps=wl.prompt + sample_steps, threads=cores)
    o = Oracle(OracleConfig(1, len(units), wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history,
                            wl.drop), nthreads=cores)
    tp = time.perf_counter()
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
                  "%.2f s measured on the decode steps (%.1f s more for the prompt), scaled by unit count" % (
                      len(units), wl.units, sample_steps, wl.prompt, dt, t0 - tp),
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


def copy_probe(args, dev) -> int:
    """Plain device copies of known size (torch's own copy kernel, one dispatch each, reading
    and writing exactly --copy-mib MiB), for calibrating HBM traffic counters: run under
    `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` it shows what the counters report for a
    known number of bytes, the scale factor applied to the decode kernel's counters."""
    import torch

    n = args.copy_mib * 2 ** 20
    src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    reps = max(1, min(args.steps, 20))
    t0 = time.perf_counter()
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    print(json.dumps({"probe": "device copy", "mib": args.copy_mib, "dispatches": reps + 1,
                      "us_per_dispatch": dt * 1e6, "read_gbs": n / dt / 1e9, "write_gbs": n / dt / 1e9}))
    return 0


def read_probe(args, dev) -> int:
    """What a launch that only reads reaches on this chip (sc_diag_read_bandwidth: --copy-mib MiB,
    rounded down to a multiple of 32, per launch; three buffers in turn so that every launch
    finds its buffer cold): the reference point for the decode kernels' fractions of peak."""
    import torch

    from paper_2305_17118_amd import binding as B

    n = max(32, args.copy_mib // 32 * 32) * 2 ** 20
    bufs = [torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(3)]
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    stream = int(torch.cuda.current_stream(dev).cuda_stream)
    reps = max(10, args.steps)
    out = {"probe": "pure read", "mib": n // 2 ** 20, "launches": reps}
    for name, nt in (("nontemporal", True), ("plain", False)):
        for i in range(5):
            B.sc_diag_read_bandwidth(bufs[i % 3].data_ptr(), n, nt, sink.data_ptr(), stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            B.sc_diag_read_bandwidth(bufs[i % 3].data_ptr(), n, nt, sink.data_ptr(), stream)
        e1.record()
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        out[name] = {"us_per_launch": us, "gbs": n / us / 1e3, "frac_of_8tbs": n / us / 1e3 / HBM_PEAK_GBS}
    print(json.dumps(out))
    return 0


def bench_layers(args, wl, dev) -> int:
    """A model step = one decode step of each of --layers caches of the workload's shape (the
    layers of a model, stepped one after another on one stream), enqueued three ways:
      calls  : one sc_decode_step_ragged call per layer,
      one    : one sc_layers_decode_step call for all layers,
      graph  : one captured sc_layers_decode_step call replayed from a HIP graph (step count kept
               on the device); compressions run eagerly between replays in all three.
    Reports microseconds per layer step (wall time of the model steps / layers)."""
    import torch

    from paper_2305_17118_amd import binding as B
    from paper_2305_17118_amd.workloads import streams

    L, U, d, T = args.layers, wl.units, wl.head_dim, wl.total
    cfg = B.make_config(wl.batch, wl.heads, d, wl.kv_dtype, wl.budget, wl.recent, wl.history, wl.drop)
    q, k, v = (torch.from_numpy(a).to(dev) for a in streams(wl, threads=16))
    K = min(args.steps, wl.decode - 2)
    res = {}
    for mode in ("calls", "one", "graph"):
        ls = B.LayerSet(cfg, [wl.budget] * L, None, dev)
        for c in ls.layers:
            c.prefill_ragged(q, k, v, [wl.prompt] * wl.batch, T * d, None)
        if mode == "graph":
            ls.device_clock(True)
        qs, ks, vs = (torch.empty(L, U, d, dtype=q.dtype, device=dev) for _ in range(3))
        out = torch.empty(L, U, d, dtype=q.dtype, device=dev)

        def load(s):
            qs.copy_(q[:, s].unsqueeze(0).expand(L, U, d))
            ks.copy_(k[:, s].unsqueeze(0).expand(L, U, d))
            vs.copy_(v[:, s].unsqueeze(0).expand(L, U, d))

        def eager_step():
            if mode == "calls":
                return sum(c.decode_step_ragged(qs[l], ks[l], vs[l], out[l]) for l, c in enumerate(ls.layers))
            return ls.decode_step(qs, ks, vs, out)

        s = wl.prompt
        load(s)
        if eager_step():   # (brings the device tables up to date)
            ls.compress()
        s += 1
        g, first = None, True
        if mode == "graph":
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                ls.decode_step(qs, ks, vs, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            load(s)
            s += 1
            if g is None:
                due = eager_step()
            else:
                due = 0 if first else ls.note_replays(1)
                first = False
                g.replay()
            if due:
                ls.compress()
        torch.cuda.synchronize()
        res[mode] = (time.perf_counter() - t0) / K / L * 1e6
        ls.close()
        del ls
        torch.cuda.empty_cache()
    print(json.dumps({"probe": "layer set", "workload": wl.name, "layers": L, "model_steps": K,
                      "us_per_layer_step": {"one_call_per_layer": res["calls"],
                                            "one_call_for_all_layers": res["one"],
                                            "one_graph_replay": res["graph"]}}))
    return 0


def pick_instances(ws_bytes: int, rotate: int) -> int:
    """Cache instances stepped round-robin: at least four (phases of the compression cycle), and
    enough that their total footprint is three times the 256 MB last-level cache."""
    return rotate or min(8, max(4, -(-3 * 256 * 2 ** 20 // ws_bytes)))


def load_compress_kernels(B, wl, dev, trigger) -> None:
    """One compression of a throw-away one-unit cache of the workload's storage type, so that the
    first sc_compress inside a timed region does not pay for loading the kernels."""
    import torch

    cfg = B.make_config(1, 1, wl.head_dim, wl.kv_dtype, 8, 2, 4, 4, trigger=trigger)
    c = B.BudgetCache(cfg, dev)
    x = torch.zeros(1, wl.head_dim, dtype=c.io_dtype, device=dev)
    out = torch.empty_like(x)
    for _ in range(16):
        if c.decode_step(x, x, x, out):
            c.compress()
            break
    torch.cuda.synchronize()
    c.close()


def run_decode(wl, args, K, W, dev, streams_dev=None):
    """Time K decode steps (after W untimed ones) of workload `wl`; -> dict of measurements."""
    import torch

    from paper_2305_17118_amd import binding as B
    from paper_2305_17118_amd.workloads import KV_F32, KV_F16, streams

    hw = getattr(args, "trigger", "hard_cap") == "high_water"
    cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history,
                        wl.drop, trigger=B.SC_TRIGGER_HIGH_WATER if hw else B.SC_TRIGGER_HARD_CAP,
                        window_mode=B.SC_WINDOW_RING if args.window == "ring" else B.SC_WINDOW_AUTO,
                        record_mode=B.SC_RECORD_RECOMPUTE if args.record == "recompute" else B.SC_RECORD_ONLINE)
    load_compress_kernels(B, wl, dev, cfg.trigger)  # (no first sc_compress pays for loading its kernels)
    R = pick_instances(B.sc_workspace_bytes(cfg), args.rotate)
    T, d, U, m = wl.total, wl.head_dim, wl.units, wl.drop
    # Phase offsets: instance r is advanced by floor(r*span/R) decode steps before the timed
    # region; span covers one compression cycle where the decode phase is long enough.
    need = -(-(K + W) // R)
    if need > wl.decode:
        K = R * wl.decode - W
        need = wl.decode
        print("bench.py: %s has only %d decode steps for %d instances; timing %d"
              % (wl.name, R * wl.decode, R, K), file=sys.stderr)
    span = 0 if args.ragged else max(0, min(m, wl.decode - need))
    offsets = [r * span // R for r in range(R)]

    if streams_dev is None:
        streams_dev = tuple(torch.from_numpy(a).to(dev) for a in streams(wl, threads=16))
    q, k, v = streams_dev
    caches = [B.BudgetCache(cfg, dev) for _ in range(R)]
    outs = [torch.empty(U, d, dtype=caches[0].io_dtype, device=dev) for _ in range(R)]
    plens = ragged_prompt_lengths(wl) if args.ragged else None
    # The prompt goes through sc_prefill except for its last m positions, which are stepped one
    # by one like the decode steps that follow (the prompt is the first part of one stream), so
    # that the compression inside them can be timed on its own.
    tail = 0 if args.ragged else min(m, wl.prompt - 1)
    for c in caches:
        if args.ragged:
            c.prefill_ragged(q, k, v, plens, T * d, None)
        else:
            c.prefill(q, k, v, wl.prompt - tail, T * d, None)
    torch.cuda.synchronize()

    cursor = [wl.prompt - tail] * R
    n_log = []
    compress_pairs = []  # HIP events around sc_compress calls outside the timed region
    # The loop below talks to the C ABI with raw addresses (no tensor views per step): on the
    # small workload the host would otherwise be slower than the kernel.
    eb = q.element_size()
    qp, kp, vp = q.data_ptr(), k.data_ptr(), v.data_ptr()
    handles = [c.handle for c in caches]
    out_ptrs = [o.data_ptr() for o in outs]
    stream = int(torch.cuda.current_stream(dev).cuda_stream)
    step_ragged, step_lock = B.sc_decode_step_ragged, B.sc_decode_step
    compress_ragged, compress_lock = B.sc_compress_ragged, B.sc_compress

    def one_step(r, time_compress=False):
        s = cursor[r]
        cursor[r] = s + 1
        off = s * d * eb
        if args.ragged:  # all sequences take part, each at its own t_b and n_b
            due = step_ragged(handles[r], qp + off, kp + off, vp + off, T * d, out_ptrs[r], None, None, stream)
            n_log.append([rows_after_step(wl, p + s - wl.prompt + 1, hw) for p in plens])
            if due:
                compress_ragged(handles[r], None, None, stream)
            return 1 if due else 0
        due = step_lock(handles[r], qp + off, kp + off, vp + off, T * d, out_ptrs[r], None, stream)
        n_log.append(rows_after_step(wl, s + 1, hw))
        if due:
            if time_compress:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                compress_lock(handles[r], None, None, stream)
                e1.record()
                compress_pairs.append((e0, e1))
            else:
                compress_lock(handles[r], None, None, stream)
        return due

    for r in range(R):  # untimed: rest of the prompt, then this instance's phase offset
        for _ in range(tail + offsets[r]):
            one_step(r, time_compress=True)
    for i in range(W):
        one_step(i % R)
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
            dirty += one_step((W + i + j) % R)
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
    compress_ms = (sum(a.elapsed_time(b) for a, b in compress_pairs) / len(compress_pairs)
                   if compress_pairs else None)
    # Compressions per decode step over the workload's whole decode phase (due after steps
    # t = n_trig + k*m), and the throughput with their measured cost spread over
    # the steps between them.
    n_trig = wl.budget + m if hw else wl.budget + 1
    in_decode = sum(1 for t in range(wl.prompt + 1, wl.total + 1) if t >= n_trig and (t - n_trig) % m == 0)
    per_step = in_decode / wl.decode
    step_ms = kern_ms if kern_ms is not None else wall / K * 1e3
    amortised = (wl.batch / ((step_ms + (compress_ms or 0.0) * per_step) * 1e-3)
                 if (compress_ms is not None or per_step == 0) else None)
    if wl.kv_dtype in (KV_F32, KV_F16):
        kernel_name = "attn_rows_kernel"
    else:
        kernel_name = "attn_i4_mfma_kernel" if wl.head_dim == 128 else "attn_i4_kernel"
    rows_avg = (sum(sum(x) / len(x) for x in n_log) if args.ragged else sum(n_log)) / len(n_log)
    lifetimes = None
    if args.lifetimes and cursor[0] < T:
        try:
            lifetimes = workgroup_lifetimes(B, handles[0], U, dev, lambda: one_step(0), args.lifetimes_dump)
        except B.ScError as e:  # caches whose units are shared among workgroups record no per-unit clocks
            print("bench.py: --lifetimes skipped (%s)" % e, file=sys.stderr)
    for c in caches:
        c.close()
    return {
        "workload": wl.name, "wl": wl, "K": K, "W": W, "R": R, "wall": wall, "offsets": offsets,
        "tokens_per_s": wl.batch * K / wall, "ms_per_step": wall / K * 1e3,
        "kernel": kernel_name, "kernel_ms_avg": kern_ms, "alg": alg, "achieved": achieved,
        "frac": None if achieved is None else achieved / HBM_PEAK_GBS,
        "compress_events": compress_events, "rows_avg": rows_avg, "plens": plens,
        "compress_ms_avg": compress_ms, "compress_samples": len(compress_pairs),
        "compressions_per_decode_step": per_step, "tokens_per_s_amortised": amortised,
        "lifetimes": lifetimes,
    }


def workgroup_lifetimes(B, handle, U, dev, step, dump=None) -> dict:
    """One more decode step with sc_diag_trace switched on: when every workgroup of the launch
    started, ended its K/V stream and finished (microseconds after the first start), overall and
    per XCD."""
    import torch

    buf = torch.zeros(U, 4, dtype=torch.int64, device=dev)
    B.sc_diag_trace(handle, buf.data_ptr())
    step()
    torch.cuda.synchronize()
    B.sc_diag_trace(handle, None)
    t = buf.cpu().numpy()
    if dump:
        import numpy
        numpy.save(dump, t)
    t = t[t[:, 2] > 0]
    if len(t) == 0:
        return None
    import numpy as np
    origin = t[:, 0].min()
    us = (t[:, :3] - origin) / 100.0  # 100 MHz clock
    q = lambda x: [round(float(v), 2) for v in np.percentile(x, [0, 5, 50, 95, 100])]
    where = t[:, 3] & 0xFFFFFFFF
    xcd = where >> 6
    # Waves that shared a SIMD (same XCD / shader engine / CU / SIMD id): does the one that
    # started first also finish first?  (rank correlation of start order and end order)
    simd = (where << 2) | ((t[:, 3] >> 36) & 3)
    same_order = pairs = 0
    for sid in np.unique(simd):
        rows = us[simd == sid]
        for a in range(len(rows)):
            for b in range(a + 1, len(rows)):
                if rows[a, 0] != rows[b, 0]:
                    pairs += 1
                    same_order += (rows[a, 0] < rows[b, 0]) == (rows[a, 2] < rows[b, 2])
    spread_in_simd = [float(us[simd == sid, 2].max() - us[simd == sid, 2].min()) for sid in np.unique(simd)]
    return {
        "workgroups": int(len(t)), "percentiles": [0, 5, 50, 95, 100],
        "start_us": q(us[:, 0]), "stream_end_us": q(us[:, 1]), "end_us": q(us[:, 2]),
        "lifetime_us": q(us[:, 2] - us[:, 0]), "after_stream_us": q(us[:, 2] - us[:, 1]),
        "per_xcd_end_us_median": {int(x): round(float(np.median(us[xcd == x, 2])), 2) for x in np.unique(xcd)},
        "per_xcd_workgroups": {int(x): int((xcd == x).sum()) for x in np.unique(xcd)},
        "cus_used": int(len(np.unique(where))),
        "simds_used": int(len(np.unique(simd))),
        "pairs_on_one_simd_finishing_in_start_order": [int(same_order), int(pairs)],
        "end_spread_within_simd_us_median": round(float(np.median(spread_in_simd)), 2),
    }


def measured_traffic(m):
    """HBM bytes per launch from the counter runs, if they were taken on exactly these launches."""
    known = MEASURED_TRAFFIC.get(m["workload"])
    if known and (m["K"], m["W"]) == known[:2] and abs(m["rows_avg"] - known[2]) < 0.05:
        return known[3]
    return None


def config_summary(m) -> dict:
    """One entry of `per_config`."""
    return {
        "traffic": measured_traffic(m),
        "workload": m["workload"], "steps": m["K"], "cache_instances_round_robin": m["R"],
        "kernel": m["kernel"], "kernel_ms_avg": m["kernel_ms_avg"],
        "algorithmic_bytes_per_launch": m["alg"], "achieved_gbs": m["achieved"], "frac": m["frac"],
        "resident_rows_avg": m["rows_avg"], "tokens_per_s": m["tokens_per_s"],
        "ms_per_step": m["ms_per_step"], "compress_ms_avg": m["compress_ms_avg"],
        "compressions_per_decode_step": m["compressions_per_decode_step"],
        "tokens_per_s_amortised": m["tokens_per_s_amortised"],
        "compressions_in_timed_region": m["compress_events"],
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="headline workload 1..5 (4 = the largest)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size "
                    "(few-unit batches; the line is then not the workload's own)")
    ap.add_argument("--rotate", type=int, default=0, help="cache instances stepped round-robin "
                    "(0 = at least 4 and enough to cover three times the 256 MB last-level cache)")
    ap.add_argument("--phase", choices=("decode", "prefill", "copy", "read", "layers"), default="decode",
                    help="decode = the headline metric; prefill = the prompt phase; copy = plain "
                         "device copies of --copy-mib MiB (calibration of HBM traffic counters); read = a launch that "
                         "only reads --copy-mib MiB (what reading reaches on this chip); "
                         "layers = --layers caches stepped per model step, eager against one HIP graph")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--copy-mib", type=int, default=1024)
    ap.add_argument("--window", choices=("auto", "ring"), default="auto",
                    help="importance record: bucket counters (auto, when w is a multiple of m) or "
                         "the exact one-bit-per-step ring")
    ap.add_argument("--record", choices=("online", "recompute"), default="online",
                    help="importance record kept during the steps (headline) or rebuilt at each "
                         "compression by replaying the last w queries")
    ap.add_argument("--trigger", choices=("hard_cap", "high_water"), default="hard_cap",
                    help="compress at B + 1 rows, leaving B + 1 - m (Alg. 1 as printed; headline), or "
                         "at B + m rows, leaving exactly B")
    ap.add_argument("--ragged", action="store_true",
                    help="decode phase with prompts of different lengths (every sequence on its own "
                         "clock: sc_prefill_ragged / sc_decode_step_ragged / sc_compress_ragged)")
    ap.add_argument("--no-events", action="store_true", help="skip the per-launch HIP events")
    ap.add_argument("--lifetimes", action="store_true",
                    help="after the timed region, one more step with sc_diag_trace: start / end of "
                         "stream / end of every workgroup of the decode-attention launch")
    ap.add_argument("--lifetimes-dump", default=None, help="also save the raw readings (.npy)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="time the headline workload only")
    ap.add_argument("--per-config-steps", type=int, default=200,
                    help="timed steps of each per_config entry other than the headline's")
    ap.add_argument("--cpu-units", type=int, default=0, help="units of the oracle sample (0 = sized "
                    "for about 20 s of CPU work)")
    ap.add_argument("--cpu-steps", type=int, default=1024)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (units are independent, so sharding over "
              "GPUs needs no collective and is not part of this build); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch

    from paper_2305_17118_amd.workloads import CONFIGS

    wl = CONFIGS[args.config - 1]
    if args.batch:
        wl = wl.scaled(batch=args.batch, name="%s-batch%d" % (wl.name, args.batch))
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.phase == "prefill":
        return bench_prefill(args, wl, dev)
    if args.phase == "copy":
        return copy_probe(args, dev)
    if args.phase == "read":
        return read_probe(args, dev)
    if args.phase == "layers":
        return bench_layers(args, wl, dev)

    variant = (args.batch or args.ragged or args.window != "auto" or args.record != "online"
               or args.trigger != "hard_cap")
    # The other workloads are timed first, in order of size, and the headline last: after the
    # 28 GB of the largest workload have been allocated and released, a small workload placed in
    # that memory ran 4% slower (cfg2: 42.6 against 40.9 us per launch) than in a fresh process.
    per_config = {}
    if not args.no_per_config and not variant:
        for other in sorted(CONFIGS, key=lambda c: c.units * (c.budget + 1) * c.head_dim):
            if other.name == wl.name:
                continue
            m = run_decode(other, args, args.per_config_steps, args.warmup, dev)
            per_config[other.name] = config_summary(m)
            del m
            torch.cuda.empty_cache()
    head = run_decode(wl, args, args.steps, args.warmup, dev)
    K, W = head["K"], head["W"]
    torch.cuda.empty_cache()
    if per_config:
        per_config[wl.name] = config_summary(head)
        per_config = [per_config[c.name] for c in CONFIGS]
    traffic = None if variant else measured_traffic(head)
    res = {
        "metric": "decode tokens/s with budgeted KV cache",
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {0: "f32", 1: "f16", 2: "i4+f16"}[wl.kv_dtype],
        "data": "synthetic",
        "config": {
            "workload": wl.name, "batch": wl.batch, "heads": wl.heads, "head_dim": wl.head_dim,
            "prompt": wl.prompt, "decode": wl.decode, "budget": wl.budget, "recent": wl.recent,
            "history": wl.history, "drop": wl.drop, "trigger": args.trigger, "window": args.window, "record": args.record,
            "cache_instances_round_robin": head["R"], "instance_phase_offsets": head["offsets"],
            "compressions_in_timed_region": head["compress_events"],
            "resident_rows_avg": head["rows_avg"],
        },
        "roofline": {
            "bound": "hbm", "achieved": head["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": head["frac"], "traffic": traffic,
            "kernel": head["kernel"], "kernel_ms_avg": head["kernel_ms_avg"],
            "algorithmic_bytes_per_launch": head["alg"],
        },
        # sc_compress (select + compact) timed with HIP events on the compressions of the untimed
        # set-up phase; amortised = batch / (attention launch + compress_ms_avg * compressions per
        # decode step of the workload's decode phase)
        "compress_ms_avg": head["compress_ms_avg"], "compress_samples": head["compress_samples"],
        "compressions_per_decode_step": head["compressions_per_decode_step"],
        "tokens_per_s_amortised": head["tokens_per_s_amortised"],
    }
    if head["lifetimes"]:
        res["workgroup_lifetimes"] = head["lifetimes"]
    if per_config:
        res["per_config"] = per_config
    if args.ragged:
        res["config"]["ragged_prompt_lengths"] = head["plens"]
    if not args.no_cpu_baseline and not args.ragged:
        units = args.cpu_units or {1: 12, 2: 512, 3: 512, 4: 1024, 5: 512}[wl.config_id]
        res["cpu_baseline"] = cpu_baseline(wl, units, args.cpu_steps)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
