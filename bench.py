#!/usr/bin/env python3
"""Benchmark of the FreeKV retrieval-decode path on one MI355X.

Workload (`config.workload`): the Llama-3-8B-shaped decode --
32 layers, 32 query / 8 KV heads, head_dim 128, bf16, batch 1, 32768 cached tokens, page 32,
budget 2048 (sink = window = 512), tau 0.8, step-correlated queries (rho = 0.9), KV resident
in HBM.  One "step" is one decode step: fkv_decode_step for each of the 32 layers, i.e. every
row of the hot path (append + summary update, correction test, page weights, softmax-mean
top-k, speculative reuse / correction, sparse attention) 32 times.  All inputs are generated
on the GPU beforehand and are resident in HBM when the timed region starts.

Prints one JSON line: `value` = layer-steps/s of the whole job; `roofline` = the layer kernel's
algorithmic HBM bytes per launch over its average launch duration (HIP events on the launch stream)
against the 8 TB/s peak, with the counter-measured traffic; `cpu_baseline` = the CPU oracle timed on
one layer of the same workload; `config.saturated_shape` = the same shape with 32 requests, where the
path is bound by bandwidth rather than by its chain of dependent memory round trips;
`config.host_pool_shape` = the same shape (16 layers of it) with the KV pool in pinned host memory, where the
loop runs at the rate of the host link; `config.other_workloads` = the other workload shapes, briefly.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM bytes per launch of the split attention kernel at this workload, from
# `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` runs scaled by a copy kernel of known
# size (profiles/layer_step_c2_pmc.txt).  None until measured.
MEASURED_TRAFFIC_BYTES = {"attn_kernel": 9419082, "layer_kernel": 14076847}
TRAFFIC_SOURCE = ("profiles/layer_step_c2_pmc.txt: rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE over this command with "
                  "--calibration-copy, KiB per dispatch scaled by what the same counters read for a 256 MiB copy")
# the same for the two kernels of the batch-32 shape (profiles/decode_step_c2_batch32_kernels_and_pmc.txt)
MEASURED_TRAFFIC_BYTES_B32 = {"attn_kernel": 273615139, "scan_kernel": 138655032}
TRAFFIC_SOURCE_B32 = "profiles/decode_step_c2_batch32_kernels_and_pmc.txt (same method, batch-32 shape)"


def algorithmic_bytes(wl):
    """Per layer-step: page summaries read by the scoring kernel and K/V read by attention."""
    n_full = wl.ctx // wl.page_size
    n_cand = n_full - wl.sink // wl.page_size - wl.window // wl.page_size
    score = n_cand * wl.n_kv_heads * wl.batch * 2 * wl.head_dim * 2
    pages = wl.budget // wl.page_size + 1          # sink + picked + window + the open page
    attn = pages * wl.n_kv_heads * wl.batch * 2 * wl.page_size * wl.head_dim * 2
    return score, attn


def gen_inputs(torch, wl, n_steps, device):
    """Seeded synthetic tensors on the GPU: N(0,1) K/V with 4 outlier channels x8, AR(1) queries."""
    g = torch.Generator(device=device)
    g.manual_seed(wl.seed)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float16
    outl = [7, 43, 71, 101]

    def kv(shape):
        x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        x[..., outl] *= 8.0
        return x.to(dt)

    noise = torch.randn((n_steps, wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim), generator=g,
                        device=device, dtype=torch.float32)
    q = torch.empty_like(noise)
    state = noise[0].clone()
    q[0] = state
    for t in range(1, n_steps):
        state = wl.rho * state + wl.q_noise * noise[t]
        q[t] = state
    q = q.to(dt).contiguous()
    k_new = kv((n_steps, wl.n_layers, wl.batch, wl.n_kv_heads, wl.head_dim)).contiguous()
    v_new = kv((n_steps, wl.n_layers, wl.batch, wl.n_kv_heads, wl.head_dim)).contiguous()
    return kv, q, k_new, v_new


def saturated_rate(torch, fkv, wl, batch, layers=2, steps=16, warmup=4):
    """The same shape with `batch` requests and few layers: enough bytes per launch for the path to be
    bound by HBM bandwidth instead of by its chain of dependent memory round trips."""
    ws = wl.scaled(batch=batch, n_layers=layers)
    dev = torch.device("cuda:0")
    p = ws.page_size
    n_steps = steps + warmup
    ctx = fkv.FreeKV(n_layers=layers, batch=batch, n_q_heads=ws.n_q_heads, n_kv_heads=ws.n_kv_heads,
                     max_ctx=((ws.ctx + n_steps + 16 + p - 1) // p) * p, budget=ws.budget, sink=ws.sink,
                     window=ws.window, tau=ws.tau, dtype=ws.dtype, placement=0)
    kv, q, k_new, v_new = gen_inputs(torch, ws, n_steps, dev)
    for layer in range(layers):
        ctx.load_prefix(layer, kv((batch, ws.ctx, ws.n_kv_heads, ws.head_dim)), kv((batch, ws.ctx, ws.n_kv_heads, ws.head_dim)))
    out = torch.empty((layers, batch, ws.n_q_heads, ws.head_dim), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def run(t0, t1):
        for t in range(t0, t1):
            for layer in range(layers):
                ctx.decode_step(layer, q[t, layer], k_new[t, layer], v_new[t, layer], out[layer], stream=stream)

    run(0, warmup)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    run(warmup, n_steps)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t_begin) / (steps * layers) * 1e6
    attn_ms, attn_n = ctx.profile_attn(q[n_steps - 1], out[0], 4, stream=stream)
    sel_ms, sel_n = ctx.profile_select(q[n_steps - 1], 4, stream=stream)
    for layer in range(layers):
        ctx.health(layer)
    launches = ctx.step_launches(0)
    ctx.close()
    score_b, attn_b = algorithmic_bytes(ws)
    attn_s, scan_s = attn_ms / attn_n * 1e-3, sel_ms / (4 * layers) * 1e-3
    # the two HBM readers of this shape, each timed back to back on its own between one HIP event pair on the launch
    # stream; the scan's time includes the selection launch that follows it (one block per KV head, no HBM stream)
    roof = [{"bound": "hbm", "kernel": "attn_kernel (split sparse decode attention)", "achieved": attn_b / attn_s / 1e9,
             "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": attn_b / attn_s / 1e9 / HBM_PEAK_GBPS,
             "traffic": MEASURED_TRAFFIC_BYTES_B32["attn_kernel"] if batch == 32 and wl.name == "c2" else None,
             "traffic_source": TRAFFIC_SOURCE_B32, "algorithmic_bytes_per_launch": attn_b, "avg_launch_us": attn_s * 1e6},
            {"bound": "hbm", "kernel": "scan_kernel (page-weight scan over the min-max summaries) + the selection launch behind it",
             "achieved": score_b / scan_s / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": score_b / scan_s / 1e9 / HBM_PEAK_GBPS,
             "traffic": MEASURED_TRAFFIC_BYTES_B32["scan_kernel"] if batch == 32 and wl.name == "c2" else None,
             "traffic_source": TRAFFIC_SOURCE_B32, "algorithmic_bytes_per_launch": score_b,
             "avg_launch_us": scan_s * 1e6, "launches_per_scan": sel_n // (4 * layers)}]
    return {"roofline": roof, "batch": batch, "layers": layers, "steps": steps, "launches_per_layer_step": launches,
            "us_per_layer_step": us, "algorithmic_MB_per_layer_step": (score_b + attn_b) / 1e6,
            "path_algorithmic_GBps": (score_b + attn_b) / us / 1e3,
            "path_frac_of_hbm_peak": (score_b + attn_b) / us / 1e3 / HBM_PEAK_GBPS,
            "attn_kernel_GBps": attn_b / (attn_ms / attn_n * 1e-3) / 1e9,
            "attn_kernel_frac_of_hbm_peak": attn_b / (attn_ms / attn_n * 1e-3) / 1e9 / HBM_PEAK_GBPS}


def host_pool_rate(torch, fkv, wl, layers=16, steps=32, warmup=8):
    """The same shape with the whole KV pool in pinned host memory (a few layers of it): recall of the picked pages
    that the GPU page cache does not hold, corrected heads inside their attention, the others deferred on a copy
    stream (Sec. 3.2, 3.3, 4.1).  Reports the loop's rate next to the host link's own."""
    from paper_2505_13109_amd import binding as B
    ws = wl.scaled(placement=1, n_layers=layers)
    dev = torch.device("cuda:0")
    p = ws.page_size
    n_probe = 8
    n_steps = steps + warmup + n_probe
    ctx = fkv.FreeKV(n_layers=layers, batch=ws.batch, n_q_heads=ws.n_q_heads, n_kv_heads=ws.n_kv_heads,
                     max_ctx=((ws.ctx + n_steps + 16 + p - 1) // p) * p, budget=ws.budget, sink=ws.sink,
                     window=ws.window, tau=ws.tau, dtype=ws.dtype, placement=1)
    kv, q, k_new, v_new = gen_inputs(torch, ws, n_steps, dev)
    for layer in range(layers):
        ctx.load_prefix(layer, kv((ws.batch, ws.ctx, ws.n_kv_heads, ws.head_dim)), kv((ws.batch, ws.ctx, ws.n_kv_heads, ws.head_dim)))
    out = torch.empty((layers, ws.batch, ws.n_q_heads, ws.head_dim), dtype=torch.float32, device=dev)
    stream, copy_stream = torch.cuda.current_stream(), torch.cuda.Stream()

    def run(t0, t1):
        for t in range(t0, t1):
            for layer in range(layers):
                ctx.decode_step(layer, q[t, layer], k_new[t, layer], v_new[t, layer], out[layer], stream=stream, copy_stream=copy_stream)

    run(0, warmup)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    run(warmup, warmup + steps)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t_begin) / (steps * layers) * 1e6
    launches = ctx.step_launches(0)
    miss = picked = 0
    for t in range(warmup + steps, n_steps):          # page-cache misses of a few more (untimed) steps
        for layer in range(layers):
            ctx.decode_step(layer, q[t, layer], k_new[t, layer], v_new[t, layer], out[layer], stream=stream, copy_stream=copy_stream)
            miss += int(ctx.debug_read(layer, B.DBG_MISS)[..., 0].sum())
            picked += ws.batch * ws.n_kv_heads * ws.k_pages
    for layer in range(layers):
        ctx.health(layer)
    ctx.close()
    src = torch.empty(1 << 29, dtype=torch.uint8, pin_memory=True)      # the host link's own rate: a plain pinned copy
    dst = torch.empty(1 << 29, dtype=torch.uint8, device=dev)
    dst.copy_(src, non_blocking=True)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    dst.copy_(src, non_blocking=True)
    c1.record()
    torch.cuda.synchronize()
    link = (1 << 29) / (c0.elapsed_time(c1) / 1e3) / 1e9
    recalled = miss / max(n_probe * layers, 1) * 16384
    return {"layers": layers, "steps": steps, "launches_per_layer_step_on_the_compute_stream": launches,
            "us_per_layer_step": us, "page_miss_rate": miss / max(picked, 1), "recall_bytes_per_layer_step": recalled,
            "recall_GBps_over_the_whole_step": recalled / us / 1e3, "pinned_copy_GBps": link}


def side_rate(torch, fkv, wl, steps, warmup):
    """Microseconds per layer-step of another workload shape, measured the same way (for the record beside the headline)."""
    dev = torch.device("cuda:0")
    p = wl.page_size
    n_steps = steps + warmup
    ctx = fkv.FreeKV(n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                     max_ctx=((wl.ctx + n_steps + 16 + p - 1) // p) * p, budget=wl.budget, sink=wl.sink,
                     window=wl.window, tau=wl.tau, dtype=wl.dtype, placement=0)
    kv, q, k_new, v_new = gen_inputs(torch, wl, n_steps, dev)
    for layer in range(wl.n_layers):
        ctx.load_prefix(layer, kv((wl.batch, wl.ctx, wl.n_kv_heads, wl.head_dim)), kv((wl.batch, wl.ctx, wl.n_kv_heads, wl.head_dim)))
    out = torch.empty((wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def run(t0, t1):
        for t in range(t0, t1):
            for layer in range(wl.n_layers):
                ctx.decode_step(layer, q[t, layer], k_new[t, layer], v_new[t, layer], out[layer], stream=stream)

    run(0, warmup)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    run(warmup, n_steps)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t_begin) / (steps * wl.n_layers) * 1e6
    launches = ctx.step_launches(0)
    for layer in range(wl.n_layers):
        ctx.health(layer)
    ctx.close()
    score_b, attn_b = algorithmic_bytes(wl)
    return {"workload": f"{wl.name}: {wl.n_layers} layers, {wl.n_q_heads}q/{wl.n_kv_heads}kv heads, {wl.dtype}, batch {wl.batch}, "
                        f"ctx {wl.ctx}, budget {wl.budget}, tau {wl.tau}, rho {wl.rho}, KV in HBM",
            "steps": steps, "launches_per_layer_step": launches, "us_per_layer_step": us,
            "path_algorithmic_GBps": (score_b + attn_b) / us / 1e3}


def handover_probe(pairs=4000):
    """What a dependency between two streams costs on this machine: pairs of tiny kernels (an in-place add on 4096 floats),
    (a) back to back on one stream, (b) the first on stream A, the second on stream B behind an event, A behind an event
    of B again.  Prints one JSON line; a side measurement for the design notes, not a benchmark of the path."""
    import torch
    dev = torch.device("cuda:0")
    x, y = torch.zeros(4096, device=dev), torch.zeros(4096, device=dev)
    a, b = torch.cuda.current_stream(), torch.cuda.Stream()
    ev = [(torch.cuda.Event(), torch.cuda.Event()) for _ in range(64)]

    def one_stream(n):
        for _ in range(n):
            x.add_(1.0)
            y.add_(1.0)

    def two_streams(n):
        for i in range(n):
            e, e2 = ev[i % 64]
            x.add_(1.0)
            e.record(a)
            b.wait_event(e)
            with torch.cuda.stream(b):
                y.add_(1.0)
            e2.record(b)
            a.wait_event(e2)

    def timed(fn):
        fn(100)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn(pairs)
        t1 = time.perf_counter()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / pairs * 1e6, (t1 - t0) / pairs * 1e6

    one, one_host = timed(one_stream)
    two, two_host = timed(two_streams)
    print(json.dumps({"probe": "stream hand-over", "pairs": pairs,
                      "us_per_pair_on_one_stream": one, "host_submit_us_per_pair_on_one_stream": one_host,
                      "us_per_pair_with_two_event_handovers": two, "host_submit_us_per_pair_with_two_event_handovers": two_host,
                      "us_per_cross_stream_dependency": (two - one) / 2}))


def _oracle_worker(job):
    """One layer of the workload through the oracle, one thread: (steps timed, seconds)."""
    wl, layer, budget_s = job
    from threadpoolctl import threadpool_limits
    import workloads as W
    from oracle import freekv_oracle as O
    with threadpool_limits(limits=1):
        (K, _), (V, _) = W.kv_prefix(wl, layer, 0)
        n_max = 400
        o = O.FreeKVOracle(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.page_size, wl.budget, wl.sink,
                           wl.window, wl.tau, wl.ctx + n_max + wl.page_size)
        o.load_prefix_bulk(K, V)
        q, _ = W.query_stream(wl, layer, 0, n_max)
        (k, _), (v, _) = W.kv_decode_tokens(wl, layer, 0, n_max)
        o.step(q[0], k[0], v[0])             # first step corrects every head: not representative, untimed
        t0 = time.perf_counter()
        n = 0
        while n + 1 < n_max and time.perf_counter() - t0 < budget_s:
            o.step(q[n + 1], k[n + 1], v[n + 1])
            n += 1
        return n, time.perf_counter() - t0


def cpu_baseline(wl, budget_s=12.0):
    """The oracle as it stands on a bounded sample of the same workload: layers are independent, so one
    single-threaded process per core takes a layer each, all at the same time.  Must run before this
    process touches the GPU (the workers are forked)."""
    import multiprocessing as mp
    workers = max(1, min(16, os.cpu_count() or 1, wl.n_layers))
    with mp.get_context("fork").Pool(workers) as pool:
        done = pool.map(_oracle_worker, [(wl, layer, budget_s) for layer in range(workers)])
    n_all = sum(n for n, _ in done)
    return {"value": sum(n / dt for n, dt in done), "unit": "layer-steps/s", "cores": workers, "kind": "oracle",
            "single_thread_value": max(n / dt for n, dt in done),
            "sample": f"layers 0..{workers - 1} of the same workload side by side, one single-threaded NumPy oracle "
                      f"process each, {n_all} decode steps in all after one untimed step per layer"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="c2", help="c2 is the benchmark workload; the others are for the design notes")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (stated in config.workload)")
    ap.add_argument("--recall-mode", type=int, default=0, help="placement 1: 0 gather kernel, 1 hipMemcpyAsync per unit")
    ap.add_argument("--placement", type=int, default=-1, help="override KV placement: 0 HBM, 1 pinned host pool")
    ap.add_argument("--batch", type=int, default=0, help="override the number of requests (stated in config.workload)")
    ap.add_argument("--tau", type=float, default=None, help="override the correction threshold (stated in config.workload)")
    ap.add_argument("--rho", type=float, default=None, help="override the adjacent-step query correlation (stated in config.workload)")
    ap.add_argument("--one-stream", action="store_true",
                    help="placement 1: the deferred recall on the compute stream instead of a copy stream (exposed; for the design notes)")
    ap.add_argument("--handover-probe", action="store_true",
                    help="measure what a dependency between two streams costs (empty kernels of the layer kernel's shape) and exit")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--standin-mb", type=int, default=0,
                    help="per layer-step, also stream this many MB through a plain reduction on the compute stream: "
                         "a labelled stand-in for the layer's QKV/FFN weight reads that recall overlaps with in a "
                         "real model (never part of the default run)")
    ap.add_argument("--saturation-batch", type=int, default=32,
                    help="also time the same shape with this many requests (2 layers, KV in HBM), where the path is "
                         "bandwidth-bound; reported as config.saturated_shape; 0 = skip")
    ap.add_argument("--real-layer", action="store_true",
                    help="design-note run: a Llama-shaped layer (QKV, RoPE, o_proj, SwiGLU FFN; random weights, "
                         "library GEMVs) around every layer-step, to see how much recall hides behind real compute")
    ap.add_argument("--nhd-stream", action="store_true",
                    help="placement 1: attach an NHD pool, so that every recalled unit is converted on its way in through "
                         "the recall kernel's two staging buffers (the paper's streamed recall, taken literally) and the "
                         "pages already on the GPU are converted in place every step")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="first run a plain elementwise kernel of known size (reads and writes 256 MiB) three "
                         "times: the yardstick for HBM byte counters collected over this command")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards over KV heads / requests "
              "with no exchange between GPUs); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.handover_probe:
        handover_probe()
        return

    import workloads as W

    wl = W.get_workload(args.workload)
    if args.layers > 0:
        wl = wl.scaled(n_layers=args.layers)
    if args.placement >= 0:
        wl = wl.scaled(placement=args.placement)
    if args.tau is not None:
        wl = wl.scaled(tau=args.tau)
    if args.batch > 0:
        wl = wl.scaled(batch=args.batch)
    if args.rho is not None:
        wl = wl.scaled(rho=args.rho, q_noise=math.sqrt(max(0.0, 1.0 - args.rho * args.rho)))
    # the CPU baseline first: its workers are forked, which has to happen before the GPU is initialised
    cpu = None
    if not args.no_cpu_baseline:
        try:
            cpu = cpu_baseline(wl)
        except Exception as e:               # noqa: BLE001 - a side measurement must not cost the result line
            cpu = {"value": None, "unit": "layer-steps/s", "cores": 0, "kind": "oracle", "sample": f"failed: {type(e).__name__}: {e}"}

    import torch                             # after the fork: the workers carry no torch threads
    import paper_2505_13109_amd as fkv
    if args.calibration_copy:
        a = torch.ones(64 * 1024 * 1024, dtype=torch.int32, device="cuda:0")
        for _ in range(3):
            b = a + 1          # vectorized_elementwise_kernel: 256 MiB read, 256 MiB written
        torch.cuda.synchronize()
        del a, b
    K, Wm = args.steps, args.warmup
    n_steps = K + Wm
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    p = wl.page_size
    long_run = K > 2048                        # a long generation: one pass, timed in segments, no per-launch event pass
    max_ctx = ((wl.ctx + (1 if long_run else 2) * n_steps + 16 + p - 1) // p) * p   # the steps are run twice (timed, then with kernel timers)
    ctx = fkv.FreeKV(n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                     max_ctx=max_ctx, budget=wl.budget, sink=wl.sink, window=wl.window, tau=wl.tau,
                     dtype=wl.dtype, placement=wl.placement, recall_mode=args.recall_mode)
    kv, q, k_new, v_new = gen_inputs(torch, wl, n_steps, dev)
    prefill_ms = 0.0
    for layer in range(wl.n_layers):
        Kp = kv((wl.batch, wl.ctx, wl.n_kv_heads, wl.head_dim))
        Vp = kv((wl.batch, wl.ctx, wl.n_kv_heads, wl.head_dim))
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        ctx.load_prefix(layer, Kp, Vp)          # bulk paging + min-max summaries (+ offload to the host pool)
        p1.record()
        torch.cuda.synchronize()
        if layer > 0 or wl.n_layers == 1:
            prefill_ms += p0.elapsed_time(p1)
        del Kp, Vp
    kv_bytes = 2 * wl.batch * wl.ctx * wl.n_kv_heads * wl.head_dim * 2
    prefill_layers = max(wl.n_layers - 1, 1)
    prefill = {"prefill_us_per_layer": prefill_ms / prefill_layers * 1e3,
               # K and V read once, written once as pages, plus the summaries (2 of 32 rows of K per page)
               "prefill_GBps_read_plus_written": (2 * kv_bytes + kv_bytes // 32) / (prefill_ms / prefill_layers / 1e3) / 1e9}
    out = torch.empty((wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    copy_stream = stream if args.one_stream else torch.cuda.Stream()

    nhd_attached = None
    if args.nhd_stream and wl.placement == 1:
        ns = wl.budget // p + 1
        nhd_attached = (torch.zeros((wl.batch, ns, 2, p, wl.n_kv_heads, wl.head_dim), dtype=ctx.torch_dtype, device=dev),
                        torch.zeros((wl.batch, wl.n_kv_heads, ns), dtype=torch.int32, device=dev))
        ctx.attach_nhd_pool(*nhd_attached)

    standin = None
    if args.standin_mb > 0:
        standin = torch.ones(args.standin_mb * 1000 * 1000 // 2, dtype=torch.bfloat16, device=dev)
        sink_val = torch.zeros((1,), dtype=torch.float32, device=dev)

    stack = None
    if args.real_layer:
        # The rest of a decoder layer, for its cost and its place on the stream (paper_2505_13109_amd/layer_loop.py):
        # hidden = n_q * d, FFN 3.5 x hidden (Llama-3.1-8B: 4096 / 14336, 436 MB of weights per layer), random
        # weights, distinct per layer.  The loop's own q, k, v stay the seeded synthetic streams, so that the reuse
        # and correction statistics remain the workload's; the projections are computed and dropped.
        from paper_2505_13109_amd.layer_loop import DecoderStack
        stack = DecoderStack(ctx, copy_stream=copy_stream)
        stack.out = out
        x_in = (torch.randn((wl.batch, stack.hidden), device=dev) ).to(ctx.torch_dtype)

    def run(t0, t1):
        for t in range(t0, t1):
            if stack is not None:
                stack.step(x_in, external_qkv=[(q[t, layer], k_new[t, layer], v_new[t, layer]) for layer in range(wl.n_layers)],
                           stream=stream)
                continue
            for layer in range(wl.n_layers):
                ctx.decode_step(layer, q[t, layer], k_new[t, layer], v_new[t, layer], out[layer],
                                stream=stream, copy_stream=copy_stream)
                if standin is not None:
                    torch.sum(standin, dim=(0,), keepdim=True, dtype=torch.float32, out=sink_val)

    run(0, Wm)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_begin = time.perf_counter()
    ev0.record(stream)                     # HIP events on the launch stream, around the timed region
    if not long_run:
        run(Wm, n_steps)
    seg_events = []
    if long_run:                               # the timed steps in 16 segments, an event at every boundary
        seg = max(1, K // 16)
        t0 = Wm
        while t0 < n_steps:
            t1 = min(n_steps, t0 + seg)
            run(t0, t1)
            e = torch.cuda.Event(enable_timing=True)
            e.record(stream)
            seg_events.append((t1 - t0, e))
            t0 = t1
            print(f"bench.py: {t0 - Wm} of {K} timed steps enqueued, {time.perf_counter() - t_begin:.0f} s", file=sys.stderr, flush=True)
    ev1.record(stream)
    t_enqueued = time.perf_counter() - t_begin     # the host is done submitting; the GPU may still be working
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_begin
    region_ms = ev0.elapsed_time(ev1)
    one_launch = ctx.step_launches(0) == 1
    assert torch.isfinite(out).all()

    # second pass over the same step inputs with a HIP event pair around every launch of the
    # split attention kernel (the dominant HBM reader), on the stream it is launched on
    pair_ms, pair_n = 0.0, 0
    if not long_run:
        ctx.profile_enable(K * wl.n_layers)
        run(Wm, n_steps)
        pair_ms, pair_n = ctx.profile_read()
        ctx.profile_enable(0)
    segments = {}
    if seg_events:
        prev, ctx_at, rows = ev0, wl.ctx + Wm, []
        for n, e in seg_events:
            ctx_at += n
            rows.append({"ctx_at_end": ctx_at, "ms_per_step": prev.elapsed_time(e) / n})
            prev = e
        segments = {"ms_per_step_by_segment": rows}
    # and the same kernel launched back to back for every layer in turn between ONE event
    # pair: no marker sits between a launch and the next, so the average is the kernel's
    # duration plus the dispatch gap, the figure a kernel trace reports
    attn_ms, attn_n = ctx.profile_attn(q[n_steps - 1], out[0], max(1, K // 4), stream=stream)

    if nhd_attached is not None:
        ctx.attach_nhd_pool(None, None)
    # what the paper's literal GPU layout would add per layer-step: the attended pages converted
    # to an NHD pool (tokens with all KV heads side by side) for a kernel that wants that layout
    n_slots = wl.budget // p + 1
    nhd_pool = torch.empty((wl.batch, n_slots, 2, p, wl.n_kv_heads, wl.head_dim), dtype=ctx.torch_dtype, device=dev)
    nhd_pages = torch.empty((wl.batch, wl.n_kv_heads, n_slots), dtype=torch.int32, device=dev)
    reps = 8
    with torch.cuda.stream(stream):
        for layer in range(wl.n_layers):
            ctx.export_nhd(layer, nhd_pool, nhd_pages, stream=stream)
        x0, x1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        x0.record(stream)
        for _ in range(reps):
            for layer in range(wl.n_layers):
                ctx.export_nhd(layer, nhd_pool, nhd_pages, stream=stream)
        x1.record(stream)
    torch.cuda.synchronize()
    nhd_us = x0.elapsed_time(x1) * 1e3 / (reps * wl.n_layers)
    nhd = {"nhd_export_us_per_layer_step": nhd_us,
           "nhd_export_GBps_read_plus_written": 2 * nhd_pool.numel() * 2 / (nhd_us * 1e-6) / 1e9}
    del nhd_pool, nhd_pages

    extra = {}
    floor = {}
    if one_launch:
        # what a launch of that shape costs when its blocks return at once, and the roofline fraction of the time
        # that is left when that cost is taken out (the launch cost is paid whatever the kernel does)
        f_ms, f_grid, f_lds = ctx.profile_launch_floor(0, 2048, stream=stream)
        floor = {"empty_launch_same_shape_us": f_ms / 2048 * 1e3, "grid_blocks": f_grid, "dynamic_lds_bytes": f_lds}
    if wl.placement == 1:
        # page-cache misses of a few more (untimed) steps, read back per layer
        from paper_2505_13109_amd import binding as B
        n_probe = min(8, Wm)
        miss = picked = 0
        for t in range(n_probe):
            for layer in range(wl.n_layers):
                ctx.decode_step(layer, q[Wm + t, layer], k_new[Wm + t, layer], v_new[Wm + t, layer], out[layer],
                                stream=stream, copy_stream=copy_stream)
                m = ctx.debug_read(layer, B.DBG_MISS)
                miss += int(m[..., 0].sum())
                picked += wl.batch * wl.n_kv_heads * wl.k_pages
        extra = {"recall_mode": "hipMemcpyAsync per unit" if args.recall_mode else
                 ("gather kernel, streamed into an NHD pool through two LDS staging buffers" if args.nhd_stream else "gather kernel"),
                 "page_miss_rate": miss / max(picked, 1),
                 "recall_bytes_per_layer_step": miss / max(n_probe * wl.n_layers, 1) * 16384}
        extra["recall_GBps_if_exposed"] = extra["recall_bytes_per_layer_step"] / (elapsed / (K * wl.n_layers)) / 1e9
        # the host link's own rate: a plain 1 GiB pinned -> device copy
        src = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
        dst = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        dst.copy_(src, non_blocking=True)
        c1.record()
        torch.cuda.synchronize()
        extra["pinned_copy_GBps"] = (1 << 30) / (c0.elapsed_time(c1) / 1e3) / 1e9
        del src, dst

    layer_steps = K * wl.n_layers
    score_b, attn_b = algorithmic_bytes(wl)
    if one_launch:
        # the whole layer-step is ONE kernel (layer_kernel): the timed region is K x n_layers
        # back-to-back launches of it, so the event time over the region divided by the launches
        # is its average launch-to-launch duration
        kernel = "layer_kernel (append + correction test + page weights + top-k + sparse attention, one launch)"
        kern_b = score_b + attn_b
        kern_s = region_ms / 1e3 / layer_steps
        kern_n = layer_steps
    else:
        kernel = "attn_kernel (split sparse decode attention)"
        kern_b = attn_b
        kern_s = attn_ms / 1e3 / max(attn_n, 1)
        kern_n = attn_n
    achieved = kern_b / kern_s / 1e9
    res = {
        "metric": "retrieval-decode layer-steps/s at 32K ctx",
        "value": layer_steps / elapsed,
        "unit": "layer-steps/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": elapsed / K * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.n_layers} layers, {wl.n_q_heads}q/{wl.n_kv_heads}kv heads, d128, "
                               f"{wl.dtype}, batch {wl.batch}, ctx {wl.ctx}, page {p}, budget {wl.budget} "
                               f"(sink {wl.sink}, window {wl.window}), tau {wl.tau}, rho {wl.rho}, "
                               f"KV {'in HBM' if wl.placement == 0 else 'in pinned host memory'}",
                   "layer_steps_per_step": wl.n_layers,
                   "us_per_layer_step": elapsed / layer_steps * 1e6,
                   "host_submit_us_per_layer_step": t_enqueued / layer_steps * 1e6,
                   "path_algorithmic_GBps": (score_b + attn_b) * layer_steps / elapsed / 1e9,
                   **({"standin_MB_per_layer_step": args.standin_mb} if args.standin_mb else {}),
                   **({"real_layer": "QKV + RoPE + o_proj + SwiGLU FFN GEMVs with random weights around every layer-step "
                                     "(library GEMVs; the loop's q, k, v stay the synthetic streams)",
                       "real_layer_weight_MB": stack.weight_bytes_per_layer / 1e6} if stack else {}), **segments, **extra, **prefill, **nhd},
        "roofline": {"bound": "hbm", "kernel": kernel,
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES["layer_kernel" if one_launch else "attn_kernel"] if wl.name == "c2" else None,
                     "traffic_source": TRAFFIC_SOURCE if wl.name == "c2" else None,
                     "algorithmic_bytes_per_launch": kern_b, "avg_launch_us": kern_s * 1e6,
                     "launches_timed": kern_n,
                     "standalone_attn_kernel_us": attn_ms / max(attn_n, 1) * 1e3,
                     "event_pair_per_launch_us": pair_ms / max(pair_n, 1) * 1e3, **floor,
                     **({"frac_of_peak_with_the_empty_launch_taken_out":
                         kern_b / max(kern_s - floor["empty_launch_same_shape_us"] * 1e-6, 1e-9) / 1e9 / HBM_PEAK_GBPS} if floor else {})},
    }
    for layer in range(wl.n_layers):
        ctx.health(layer)                # no kernel gave up a bounded wait
    ctx.close()
    del kv, q, k_new, v_new, out
    torch.cuda.empty_cache()
    if args.saturation_batch > 0 and wl.name == "c2" and args.batch == 0 and not args.real_layer and not args.standin_mb:
        try:                             # a side measurement: it must not cost the line above
            sat = saturated_rate(torch, fkv, wl, args.saturation_batch)
            res["roofline_saturated_shape"] = sat.pop("roofline")
            res["config"]["saturated_shape"] = sat
        except Exception as e:           # noqa: BLE001
            res["config"]["saturated_shape"] = {"error": f"{type(e).__name__}: {e}"}
        try:                             # and the same shape with the KV pool in pinned host memory
            res["config"]["host_pool_shape"] = host_pool_rate(torch, fkv, wl)
        except Exception as e:           # noqa: BLE001
            res["config"]["host_pool_shape"] = {"error": f"{type(e).__name__}: {e}"}
        try:                             # the other workload shapes, briefly (a few layers of the big ones)
            import workloads as W
            res["config"]["other_workloads"] = [
                side_rate(torch, fkv, W.get_workload("c1"), 64, 8),
                side_rate(torch, fkv, W.get_workload("c4").scaled(n_layers=8), 32, 8),
                side_rate(torch, fkv, W.get_workload("c5"), 128, 16),
                side_rate(torch, fkv, W.get_workload("c5").scaled(tau=0.65), 128, 16),
                side_rate(torch, fkv, W.get_workload("c3").scaled(placement=0, n_layers=4), 16, 4)]
        except Exception as e:           # noqa: BLE001
            res["config"]["other_workloads"] = {"error": f"{type(e).__name__}: {e}"}
    if cpu is not None:
        res["cpu_baseline"] = cpu
    print(json.dumps(res))


if __name__ == "__main__":
    main()
