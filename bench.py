#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A "step" is one pass of the whole layer (gate -> Top-k -> dispatch -> grouped SwiGLU GEMM ->
down GEMM -> weighted combine) over one batch of synthetic tokens, through the C ABI, with all
inputs already in HBM (experts resident: the kernel regime).  The headline workload is the
Mixtral-8x7B-shaped prefill layer (d=4096, I=14336, 8 experts, top-2, 2048 tokens, bf16).

Also reported on the same JSON line:
  roofline      the dominant kernel (gate/up grouped GEMM + SwiGLU) against the bf16 MFMA peak,
                from HIP events recorded on the compute stream around each launch
  offloaded     the same layer with the GPU expert cache capped at 2 slots: experts stream from
                pinned host memory on the copy stream while a stand-in attention block runs
  decode        Mixtral-shaped decode (batch 1): per-layer latency and expert-GEMV HBM GB/s
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
PEAK_PCIE_GBS = 64.0        # PCIe Gen5 x16 per direction
# HBM bytes per launch of the gate/up GEMM on the headline workload.  NOT measured by this run: hardware
# counters need the profiler.  The figure comes from two rocprofv3 --pmc runs of this same command
# (FETCH_SIZE, WRITE_SIZE), each scaled by what the same counter reads for a plain 256 MiB device copy
# (x2.000 and x1.000); the summary with the commands is the file named here.
# Algorithmic bytes of that launch: 1879 MB of weights + 16.8 MB of activations read, 117.4 MB written.
TRAFFIC_PROFILE = "profiles/prefill_c2_mixtral_gemm_counters.txt"
MEASURED_TRAFFIC_BYTES = {"c2_mixtral_prefill": 2352.6e6 + 117.4e6}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def prefill_resident(args, torch, B, H, S, w, compute, copy):
    """Kernel regime of the prefill layer: S = E slots, every expert resident."""
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E, w.I_shared)
    t0 = time.time()
    pool = H.HostPool(w, 0)
    log(f"[bench] host pool {w.E * w.blob_bytes / 1e9:.2f} GB generated in {time.time() - t0:.1f}s")
    lay = H.DeviceLayer(ctx, w, 0, pool, list(range(w.E)))
    buf = H.Buffers(ctx, w.T)
    x_np = S.activations(w)
    x = H.np_to_dev(x_np)
    bias = None
    if w.zipf_s > 0:
        bias = torch.from_numpy(S.zipf_route_bias(w, 0)).cuda()

    def step():
        ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, compute, copy, bias, 0)

    # The device needs a fraction of a second of work after idling before its clocks settle (the first
    # ~15 layer calls run 15-40 % slower), whatever --warmup says: untimed steps for settle_s seconds,
    # then the W warm-up steps, then exactly K timed steps.
    t0 = time.perf_counter()
    settle_steps = 0
    while time.perf_counter() - t0 < args.settle_s:
        for _ in range(8):
            step()
        torch.cuda.synchronize()
        settle_steps += 8
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-kernel durations from HIP events on the compute stream
    ctx.moe_set_profiling(True)
    nprof = max(3, min(args.steps, 10))
    for _ in range(nprof):
        step()
    torch.cuda.synchronize()
    times = ctx.moe_get_kernel_times()
    ctx.moe_set_profiling(False)
    kern = {k: (v[0] / v[1] if v[1] else 0.0) for k, v in times.items()}
    routing = buf.routing(ctx, compute)
    return dict(ms=ms, kern_ms=kern, ctx=ctx, pool=pool, lay=lay, buf=buf, x=x, x_np=x_np, bias=bias,
                routing=routing, compute=compute, copy=copy, settle_steps=settle_steps)


def prefill_large_batch(args, torch, B, H, S, w, res, rep):
    """The same layer on rep x the tokens (the batch of rep sequences prefilled together): more row
    tiles per expert, so the GEMMs run at the rate the kernel reaches when tiles are plentiful."""
    from dataclasses import replace
    wl = replace(w, T=w.T * rep)
    ctx = B.MoeContext(wl.d, wl.I, wl.E, wl.k, 1, wl.E, wl.I_shared)
    lay = H.DeviceLayer(ctx, wl, 0, res["pool"], list(range(wl.E)))
    buf = H.Buffers(ctx, wl.T)
    x = res["x"].repeat(rep, 1).contiguous()
    compute, copy = res["compute"], res["copy"]

    def step():
        ctx.moe_prefill_layer(0, x, wl.T, buf.y, buf.ws, compute, copy, res["bias"], 0)

    n = 4
    for _ in range(n):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / n
    ctx.moe_set_profiling(True)
    for _ in range(3):
        step()
    torch.cuda.synchronize()
    times = ctx.moe_get_kernel_times()
    ctx.close()
    g1 = times["gemm1"][0] / times["gemm1"][1]
    g2 = times["gemm2"][0] / times["gemm2"][1]
    rows = wl.T * wl.k
    return {"workload": f"{w.name} shape with T={wl.T}", "ms_per_layer": ms, "tokens_per_s": wl.T / (ms * 1e-3),
            "gemm1_TFLOPs": 4.0 * rows * wl.d * wl.I / (g1 * 1e-3) / 1e12,
            "gemm1_frac_of_mfma_peak": 4.0 * rows * wl.d * wl.I / (g1 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "gemm2_TFLOPs": 2.0 * rows * wl.d * wl.I / (g2 * 1e-3) / 1e12}


def prefill_offloaded(args, torch, B, H, S, w, pool, x, compute, copy, steps=6, fmt=0):
    """Offloaded regime: S = w.S slots, experts fetched from pinned memory on the copy stream; a
    stand-in attention block (4 bf16 GEMMs T x d x d) runs on the compute stream while the first
    experts are prefetched.  Returns T_copy-alone, T_compute-alone and T_pipelined per layer.
    fmt 1 / 3: the CPU expert cache holds the same experts as e4m3 codes with per-row scales / as MXFP4
    (half / about a quarter of the bytes on the link; the slots hold those blobs and every kernel reads
    the codes); fmt 2: as 4-bit integer codes in groups of 128, expanded into bf16 slots by a kernel
    behind each copy."""
    q8 = fmt != 0
    if q8:
        t0 = time.time()
        pool = H.HostPool(w, 0, fmt=fmt)
        log(f"[bench] {8 if fmt == 1 else 4}-bit host pool (format {fmt}) {w.E * pool.bytes_per_expert / 1e9:.2f} GB quantised in {time.time() - t0:.1f}s")
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.S, w.I_shared, host_format=fmt)
    lay = H.DeviceLayer(ctx, w, 0, pool, None)
    buf = H.Buffers(ctx, w.T)
    wa = H.np_to_dev(S.normal_bf16((4, w.d, w.d), w.seed, S.stream_id(S.KIND_ATTN), 0.02))
    act = [torch.empty((w.T, w.d), dtype=torch.int16, device="cuda") for _ in range(2)]
    act[0].copy_(x)

    def attention():
        src = 0
        for i in range(4):
            B.moe_dense_gemm_bf16(act[src], wa[i], act[1 - src], w.T, w.d, w.d, compute)
            src = 1 - src

    def pipelined():
        # a new layer: its experts are not in the slots yet (copies still wait for the readers
        # of the previous pass)
        ctx.moe_cache_invalidate(0)
        ctx.expert_cache_prefetch(0, list(range(w.S)), copy)
        attention()
        ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, compute, copy)

    def timed(fn, n):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    t_p = timed(pipelined, steps)
    st = ctx.moe_get_stats(0)
    bytes_per_layer = st["bytes_h2d"] / st["layer_calls"]

    # copies alone: the same blobs through the same slots, nothing else running
    raw = lay.cache.view(torch.uint8)
    hb = pool.bytes_per_expert
    stage = (hb + 255) // 256 * 256

    def copies():
        for e in range(w.E):
            s = e % w.S
            off = (s * stage if fmt in (1, 3) else w.S * w.blob_bytes + s * stage) if q8 else s * w.blob_bytes
            raw[off:off + hb].copy_(pool.buf[e], non_blocking=True)

    with torch.cuda.stream(copy):
        t_c = timed(copies, steps)
    ctx.close()
    out = dict(t_pipelined_ms=t_p, t_copy_ms=t_c, bytes_per_layer=bytes_per_layer, attention=attention, timed=timed)
    if fmt in (1, 3):
        # the same layer with every expert resident in its quantised form: the GEMMs that expand code tiles
        # on their way into LDS, nothing fetched
        ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E, w.I_shared, host_format=fmt)
        lay = H.DeviceLayer(ctx, w, 0, pool, list(range(w.E)))
        buf = H.Buffers(ctx, w.T)
        layer = lambda: ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, compute, copy)
        for _ in range(150):      # clocks settle under the GEMMs' load, as in the bf16 leg
            layer()
        out["t_resident_ms"] = timed(layer, 20)
        ctx.close()
    return out


def decode_batch_us(torch, H, S, ctx, wl, n_layers, batch, compute, copy, bytes_per_expert, steps=8):
    """Per-layer latency of the same resident layers at a decode batch of `batch` tokens (the paper's
    batching study, Section VI): one warm-up pass over the trace (every launch variant loaded), one timed."""
    from dataclasses import replace
    import numpy as np
    wb = replace(wl, T=batch, steps=steps)
    trace = S.markov_trace(wb)
    buf = H.Buffers(ctx, batch)
    xs = [H.np_to_dev(S.activations(wb, l, 0)) for l in range(n_layers)]
    biases = [[H.np_to_dev(S.trace_route_bias(trace[s, l], wb.E)) for l in range(n_layers)] for s in range(steps)]

    def one_pass():
        for s in range(steps):
            for l in range(n_layers):
                ctx.moe_decode_layer(l, xs[l], batch, buf.y, buf.ws, compute, copy, biases[s][l], wb.E)
        torch.cuda.synchronize()

    one_pass()
    t0 = time.perf_counter()
    one_pass()
    us = (time.perf_counter() - t0) * 1e6 / (steps * n_layers)
    distinct = float(np.mean([len(set(trace[s, l].ravel().tolist())) for s in range(steps) for l in range(n_layers)]))
    # the distinct experts' weights (in the form the mat-vecs read) once per layer, over the whole layer time
    return {"us_per_layer": us, "distinct_experts_per_layer": distinct,
            "layer_HBM_GBps": distinct * bytes_per_expert / (us * 1e-6) / 1e9}


def decode_regime(args, torch, B, H, S, w, n_layers, steps, compute, copy, pred):
    """Decode: per-layer latency with the predictor-guided cache (S slots per layer) and with all
    experts resident (hit path only); expert-GEMV HBM GB/s from HIP events."""
    import numpy as np
    from dataclasses import replace
    wl = replace(w, L=n_layers, steps=steps)
    t0 = time.time()
    pools = [H.HostPool(wl, l) for l in range(n_layers)]
    log(f"[bench] decode host pools {n_layers * wl.E * wl.blob_bytes / 1e9:.1f} GB in {time.time() - t0:.1f}s")
    trace = S.markov_trace(wl)
    out = {}
    # "cached": S slots per layer (the configuration named in BASELINE.json); "shared_k": the paper's
    # cache, ONE set of k slots for all layers, predictor top-k; "resident": kernels only
    xs0 = [H.np_to_dev(S.activations(wl, l, 0)) for l in range(n_layers)]
    biases0 = [[H.np_to_dev(S.trace_route_bias(trace[s, l], wl.E)) for l in range(n_layers)] for s in range(steps)]
    out["cached"] = decode_cached(torch, B, H, S, wl, pools, trace, xs0, biases0, compute, copy, pred)
    for label, slots in (("shared_k", wl.k), ("resident", wl.E)):
        shared = label == "shared_k"
        ctx = B.MoeContext(wl.d, wl.I, wl.E, wl.k, n_layers, slots, wl.I_shared, True, shared_slots=shared)
        init = None if shared else list(range(slots))
        cache = torch.empty((slots, wl.blob_elems), dtype=torch.int16, device="cuda") if shared else None
        layers = [H.DeviceLayer(ctx, wl, l, pools[l], init, slots=cache) for l in range(n_layers)]
        top_m = wl.k if shared else wl.top_m
        wps = [H.np_to_dev(S.predictor_weight(wl, l)) for l in range(n_layers)]
        buf = H.Buffers(ctx, wl.T)
        xs = [H.np_to_dev(S.activations(wl, l, 0)) for l in range(n_layers)]
        biases = [[torch.from_numpy(S.trace_route_bias(trace[s, l], wl.E)).cuda() for l in range(n_layers)]
                  for s in range(steps)]
        top = torch.zeros(max(1, top_m), dtype=torch.int32).pin_memory()
        predict = label != "resident"

        def one_step(s):
            for l in range(n_layers):
                if predict and l + 1 < n_layers:
                    # predictor for the next layer on its own stream (Section V-C)
                    ctx.predictor_score(l + 1, xs[l], wl.T, wps[l + 1], top_m, top, pred)
                ctx.moe_decode_layer(l, xs[l], wl.T, buf.y, buf.ws, compute, copy, biases[s][l], wl.E)
                if predict and l + 1 < n_layers:
                    pred.synchronize()
                    ctx.expert_cache_prefetch(l + 1, top.tolist(), copy)

        one_step(0)
        torch.cuda.synchronize()
        ctx.moe_reset_stats()
        t0 = time.perf_counter()
        for s in range(steps):
            one_step(s)
        torch.cuda.synchronize()
        us_layer = (time.perf_counter() - t0) * 1e6 / (steps * n_layers)
        st = ctx.moe_get_stats(-1)
        ctx.moe_set_profiling(True)
        for s in range(min(steps, 8)):
            one_step(s)
        torch.cuda.synchronize()
        kt = ctx.moe_get_kernel_times()
        ctx.moe_set_profiling(False)
        g1 = kt["gemv1"][0] / max(1, kt["gemv1"][1])
        g2 = kt["gemv2"][0] / max(1, kt["gemv2"][1])
        out[label] = dict(us_per_layer=us_layer, stats=st, gemv1_ms=g1, gemv2_ms=g2,
                          launches=(kt["gemv1"][1], kt["gemv2"][1]))
        if label == "resident":
            out[label]["batch8"] = decode_batch_us(torch, H, S, ctx, wl, n_layers, 8, compute, copy, wl.blob_bytes)
        ctx.close()
        del layers, cache
    return out


def decode_resident_q8(args, torch, B, H, S, w, n_layers, steps, compute, copy, fmt=1):
    """Kernel regime of decode with a quantised host pool (fmt 1: e4m3 rows, 3: MXFP4): every expert
    fetched once through the library into a slot of its own, then steady-state steps in which the
    mat-vec kernels stream the quantised blobs."""
    from dataclasses import replace
    wl = replace(w, L=n_layers, steps=steps)
    t0 = time.time()
    pools = [H.HostPool(wl, l, fmt=fmt) for l in range(n_layers)]
    log(f"[bench] decode host pools in format {fmt}: {n_layers * wl.E * pools[0].bytes_per_expert / 1e9:.1f} GB in {time.time() - t0:.1f}s")
    trace = S.markov_trace(wl)
    ctx = B.MoeContext(wl.d, wl.I, wl.E, wl.k, n_layers, wl.E, wl.I_shared, True, host_format=fmt)
    layers = [H.DeviceLayer(ctx, wl, l, pools[l], None) for l in range(n_layers)]
    for l in range(n_layers):
        ctx.expert_cache_prefetch(l, list(range(wl.E)), copy)
    torch.cuda.synchronize()
    buf = H.Buffers(ctx, wl.T)
    xs = [H.np_to_dev(S.activations(wl, l, 0)) for l in range(n_layers)]
    biases = [[torch.from_numpy(S.trace_route_bias(trace[s, l], wl.E)).cuda() for l in range(n_layers)]
              for s in range(steps)]

    def one_step(s):
        for l in range(n_layers):
            ctx.moe_decode_layer(l, xs[l], wl.T, buf.y, buf.ws, compute, copy, biases[s][l], wl.E)

    one_step(0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        one_step(s)
    torch.cuda.synchronize()
    us_layer = (time.perf_counter() - t0) * 1e6 / (steps * n_layers)
    ctx.moe_set_profiling(True)
    for s in range(min(steps, 8)):
        one_step(s)
    torch.cuda.synchronize()
    kt = ctx.moe_get_kernel_times()
    ctx.moe_set_profiling(False)
    batch8 = decode_batch_us(torch, H, S, ctx, wl, n_layers, 8, compute, copy, pools[0].bytes_per_expert)
    ctx.close()
    g = kt["gemv1"][0] / max(1, kt["gemv1"][1]) + kt["gemv2"][0] / max(1, kt["gemv2"][1])
    code_bytes = wl.k * pools[0].bytes_per_expert
    out = {"us_per_layer": us_layer, "gemv_us_per_layer": g * 1e3, "layers": n_layers,
           "gemv_HBM_GBps": code_bytes / (g * 1e-3) / 1e9 if g else 0.0,
           "gemv_frac_of_hbm_peak": code_bytes / (g * 1e-3) / 1e9 / PEAK_HBM_GBS if g else 0.0,
           "batch8": batch8}
    del layers

    # the paper's decode flow on the same 8-bit pools: one cache of k slots for all layers, first layer
    # on demand, the next layer's experts predicted and prefetched, wrong guesses fetched again
    ctx = B.MoeContext(wl.d, wl.I, wl.E, wl.k, n_layers, wl.k, wl.I_shared, True, shared_slots=True, host_format=fmt)
    cache = torch.empty(ctx.moe_cache_bytes() // 2, dtype=torch.int16, device="cuda")
    layers = [H.DeviceLayer(ctx, wl, l, pools[l], None, slots=cache) for l in range(n_layers)]
    wps = [H.np_to_dev(S.predictor_weight(wl, l)) for l in range(n_layers)]
    top = torch.zeros(wl.k, dtype=torch.int32).pin_memory()
    pred = torch.cuda.Stream()

    def flow_step(s):
        for l in range(n_layers):
            if l + 1 < n_layers:
                ctx.predictor_score(l + 1, xs[l], wl.T, wps[l + 1], wl.k, top, pred)
            ctx.moe_decode_layer(l, xs[l], wl.T, buf.y, buf.ws, compute, copy, biases[s][l], wl.E)
            if l + 1 < n_layers:
                pred.synchronize()
                ctx.expert_cache_prefetch(l + 1, top.tolist(), copy)

    flow_step(0)
    torch.cuda.synchronize()
    ctx.moe_reset_stats()
    t0 = time.perf_counter()
    for s in range(steps):
        flow_step(s)
    torch.cuda.synchronize()
    out["shared_k_us_per_layer"] = (time.perf_counter() - t0) * 1e6 / (steps * n_layers)
    out["shared_k_stats"] = ctx.moe_get_stats(-1)
    ctx.close()
    return out


def mlp_predictor_latency(torch, B, H, S, w, pred):
    """One ExpertMLP prediction (Section IV-B) for the decode workload's model: state vector in pinned
    memory, eight fully connected layers and the top-k on the prediction stream; microseconds each."""
    import numpy as np
    dims = S.mlp_dims(w.L, w.E, w.k)
    ws, bs, sc, sh = S.mlp_params(dims, w.seed)
    dev = lambda arrs: [H.np_to_dev(a) for a in arrs]
    dws, dbs, dsc, dsh = dev(ws), dev(bs), dev(sc), dev(sh)
    act = torch.empty(2 * max(dims), dtype=torch.float32, device="cuda")
    state = torch.from_numpy(np.abs(S.normal_f32((dims[0],), w.seed, 12345, 0.3))).pin_memory()
    top = torch.zeros(w.k, dtype=torch.int32).pin_memory()
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E)
    for _ in range(10):
        ctx.predictor_mlp_score(state, dims, dws, dbs, dsc, dsh, act, w.k, top, pred)
    pred.synchronize()
    t0 = time.perf_counter()
    n = 200
    for _ in range(n):
        ctx.predictor_mlp_score(state, dims, dws, dbs, dsc, dsh, act, w.k, top, pred)
    pred.synchronize()
    us = (time.perf_counter() - t0) * 1e6 / n
    ctx.close()
    params_mb = sum(a.nbytes for a in ws + bs + sc + sh) / 1e6
    return {"us_per_prediction": us, "layers": dims, "parameter_MB": params_mb}


def prefill_c4(args, torch, B, H, S, compute, copy, steps=20, n_check=32):
    """DeepSeek-MoE-shaped prefill layer (64 routed experts top-6 with Zipf popularity, 2 shared experts,
    4096 tokens): kernel regime with every expert resident, then the configured 16 slots with the
    experts streaming from pinned memory.  Sampled tokens are checked against the oracle."""
    import numpy as np
    import oracle
    w = S.WORKLOADS["c4_deepseek_prefill"]
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E, w.I_shared)
    pool = H.HostPool(w, 0)
    lay = H.DeviceLayer(ctx, w, 0, pool, list(range(w.E)))
    buf = H.Buffers(ctx, w.T)
    x_np = S.activations(w)
    x = H.np_to_dev(x_np)
    bias_np = S.zipf_route_bias(w, 0)
    bias = H.np_to_dev(bias_np)

    def step():
        ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, compute, copy, bias, 0)

    t0 = time.perf_counter()
    warm = 0
    while warm < 10 or time.perf_counter() - t0 < args.settle_s:   # (clock settling, as in the main leg)
        for _ in range(5):
            step()
        torch.cuda.synchronize()
        warm += 5
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    ctx.moe_set_profiling(True)
    for _ in range(5):
        step()
    torch.cuda.synchronize()
    kt = ctx.moe_get_kernel_times()
    ctx.moe_set_profiling(False)
    kern = {k: v[0] / 5 for k, v in kt.items() if v[1]}          # ms per layer call (routed + shared launches)
    routing = buf.routing(ctx, compute)
    counts = routing["counts"]
    sel = np.linspace(0, w.T - 1, n_check).astype(np.int32)
    ref = oracle.moe_layer(x_np, lay.router_np, [pool.ptr(e) for e in range(w.E)], w.k, bias=bias_np, sel=sel,
                           shared_blob=lay.shared_np, I=w.I, I_shared=w.I_shared)
    got = S.bf16_to_f32(H.dev_to_np_u16(buf.y)[sel]).astype(np.float64)
    err = np.abs(got - ref["out_f64"])
    ok = bool(np.all(err <= 1e-2 + 2e-2 * np.abs(ref["out_f64"])) and np.array_equal(ref["ids"], routing["ids"]))
    ctx.close()
    rows = w.T * w.k
    fl_routed, fl_shared = 6.0 * rows * w.d * w.I, 6.0 * w.T * w.d * w.I_shared
    out = {"workload": f"{w.name}: d={w.d} I={w.I} E={w.E} top-{w.k} + shared I={w.I_shared}, T={w.T}, Zipf s={w.zipf_s}, "
                       f"layer 0 of {w.L}, experts resident",
           "ms_per_layer": ms, "tokens_per_s": w.T / (ms * 1e-3), "kernels_ms_per_layer": kern,
           "flops_per_layer": fl_routed + fl_shared,
           "mfma_frac_layer": (fl_routed + fl_shared) / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
           # the shared experts' two GEMM launches run on the library's side stream beside the gate, the
           # grouping and the routed launches, so the stage timers above overlap; the GEMM phase is the
           # layer without its weighted sum
           "gemm_phase_ms": ms - kern["combine"],
           "gemm_phase_frac_of_mfma_peak": (fl_routed + fl_shared) / ((ms - kern["combine"]) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
           "rows_per_expert": {"max": int(counts.max()), "median": int(np.median(counts)), "min": int(counts.min()),
                               "below_256": int((counts < 256).sum())},
           "parity_on_sample": ok, "sample_tokens": n_check, "max_abs_err_on_sample": float(err.max())}

    if args.no_offloaded:
        return out
    # the configured cache of 16 slots: every expert streams through it once per layer; in bf16, and
    # (unless --no-q8) with the experts held and fetched as MXFP4 blobs, for which the layer with every
    # expert resident is timed as well
    for fmt, key in ((0, "offloaded"),) + (() if args.no_q8 else ((3, "offloaded_mxfp4"),)):
        qpool = pool if fmt == 0 else H.HostPool(w, 0, fmt=fmt)
        ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.S, w.I_shared, host_format=fmt)
        lay2 = H.DeviceLayer(ctx, w, 0, qpool, None)

        def pipelined():
            ctx.moe_cache_invalidate(0)
            ctx.expert_cache_prefetch(0, list(range(w.S)), copy)
            ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, compute, copy, bias, 0)

        pipelined()
        torch.cuda.synchronize()
        ctx.moe_reset_stats()
        t0 = time.perf_counter()
        for _ in range(3):
            pipelined()
        torch.cuda.synchronize()
        t_p = (time.perf_counter() - t0) * 1e3 / 3
        st = ctx.moe_get_stats(0)
        ctx.close()
        del lay2
        out[key] = {"slots": w.S, "ms_per_layer": t_p, "bytes_per_layer": st["bytes_h2d"] / st["layer_calls"],
                    "link_GBps_over_the_layer": st["bytes_h2d"] / st["layer_calls"] / (t_p * 1e-3) / 1e9}
        if fmt:
            ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E, w.I_shared, host_format=fmt)
            lay3 = H.DeviceLayer(ctx, w, 0, qpool, list(range(w.E)))
            layer = lambda: ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, compute, copy, bias, 0)
            for _ in range(100):
                layer()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                layer()
            torch.cuda.synchronize()
            out[key]["resident_ms_per_layer"] = (time.perf_counter() - t0) * 1e3 / steps
            ctx.close()
            del lay3
    return out


def decode_c5(args, torch, B, H, S, compute, copy, pred, n_layers=4, steps=32):
    """Qwen1.5-MoE-shaped decode (60 routed experts top-4, one shared expert of 5632, batch 8): per-layer
    latency with every expert resident (kernel regime, HBM fraction of the distinct experts' bytes) and
    with the configured 15 slots per layer and the linear predictor's top-8 prefetched a layer ahead."""
    import numpy as np
    from dataclasses import replace
    w = replace(S.WORKLOADS["c5_qwen_decode"], L=n_layers, steps=steps)
    pools = [H.HostPool(w, l) for l in range(n_layers)]
    trace = S.markov_trace(w)
    distinct = float(np.mean([len(set(trace[s, l].ravel().tolist())) for s in range(steps) for l in range(n_layers)]))
    xs = [H.np_to_dev(S.activations(w, l, 0)) for l in range(n_layers)]
    biases = [[H.np_to_dev(S.trace_route_bias(trace[s, l], w.E)) for l in range(n_layers)] for s in range(steps)]
    out = {"workload": f"{w.name}: d={w.d} I={w.I} E={w.E} top-{w.k} + shared I={w.I_shared}, batch {w.T}, "
                       f"{n_layers} of {S.WORKLOADS['c5_qwen_decode'].L} layers in memory, {steps} steps",
           "distinct_experts_per_layer": distinct}

    # kernel regime
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, n_layers, w.E, w.I_shared)
    layers = [H.DeviceLayer(ctx, w, l, pools[l], list(range(w.E))) for l in range(n_layers)]
    buf = H.Buffers(ctx, w.T)

    def resident_pass():
        for s in range(steps):
            for l in range(n_layers):
                ctx.moe_decode_layer(l, xs[l], w.T, buf.y, buf.ws, compute, copy, biases[s][l], w.E)
        torch.cuda.synchronize()

    resident_pass()
    t0 = time.perf_counter()
    resident_pass()
    us = (time.perf_counter() - t0) * 1e6 / (steps * n_layers)
    ctx.moe_set_profiling(True)
    resident_pass()
    kt = ctx.moe_get_kernel_times()
    ctx.moe_set_profiling(False)
    calls = steps * n_layers
    kern_us = {k: v[0] * 1e3 / calls for k, v in kt.items() if v[1]}
    bytes_layer = distinct * w.blob_bytes + w.shared_blob_bytes
    out.update({"resident_us_per_layer": us, "kernels_us_per_layer": kern_us,
                "bytes_per_layer": bytes_layer,
                "layer_HBM_GBps": bytes_layer / (us * 1e-6) / 1e9,
                "layer_frac_of_hbm_peak": bytes_layer / (us * 1e-6) / 1e9 / PEAK_HBM_GBS})
    ctx.close()
    del layers

    if args.no_offloaded:
        return out
    # the configured cache: 15 of 60 experts per layer, predictor top-8 one layer ahead
    out["cached"] = decode_cached(torch, B, H, S, w, pools, trace, xs, biases, compute, copy, pred)
    return out


def decode_cached(torch, B, H, S, w, pools, trace, xs, biases, compute, copy, pred):
    """Decode through the configured per-layer slots with predictor-guided prefetch (Section V-C): whole-run
    latency, counters, the share of used prefetches that had landed when compute asked for them, and the
    per-layer latency of calls without and with a miss (each call timed to its completion on the host)."""
    n_layers, steps = len(pools), len(biases)
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, n_layers, w.S, w.I_shared)
    layers = [H.DeviceLayer(ctx, w, l, pools[l], list(range(w.S))) for l in range(n_layers)]
    wps = [H.np_to_dev(S.predictor_weight(w, l)) for l in range(n_layers)]
    buf = H.Buffers(ctx, w.T)
    top = torch.zeros(w.top_m, dtype=torch.int32).pin_memory()

    def one_step(s, per_call=None):
        for l in range(n_layers):
            if l + 1 < n_layers:
                ctx.predictor_score(l + 1, xs[l], w.T, wps[l + 1], w.top_m, top, pred)
            t0 = time.perf_counter()
            st = ctx.moe_decode_layer(l, xs[l], w.T, buf.y, buf.ws, compute, copy, biases[s][l], w.E,
                                      want_stats=per_call is not None)
            if per_call is not None:
                compute.synchronize()
                per_call.append(((time.perf_counter() - t0) * 1e6, st["misses"]))
            if l + 1 < n_layers:
                pred.synchronize()
                ctx.expert_cache_prefetch(l + 1, top.tolist(), copy)

    one_step(0)
    torch.cuda.synchronize()
    ctx.moe_reset_stats()
    t0 = time.perf_counter()
    for s in range(steps):
        one_step(s)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) * 1e6 / (steps * n_layers)
    st = ctx.moe_get_stats(-1, full=True)
    per_call = []
    for s in range(steps):
        one_step(s, per_call)
    torch.cuda.synchronize()
    ctx.close()
    del layers
    hit_calls = [t for t, m in per_call if m == 0]
    miss_calls = [t for t, m in per_call if m > 0]
    used = st["prefetch_ready"] + st["prefetch_stalled"]
    mean = lambda v: float(sum(v) / len(v)) if v else None
    return {"slots": w.S, "predictor_top_m": w.top_m, "us_per_layer": us, "stats": st,
            "hit_rate": st["hits"] / max(1, st["hits"] + st["misses"]),
            # of the prefetched experts that were used: landed before compute asked for them (no stall)
            "prefetch_no_stall_frac": st["prefetch_ready"] / used if used else None,
            "host_wait_for_gate_ms_per_layer": st["wait_ms"] / max(1, st["layer_calls"]),
            "calls_without_miss": len(hit_calls), "hit_path_us_per_layer": mean(hit_calls),
            "calls_with_miss": len(miss_calls), "miss_path_us_per_layer": mean(miss_calls),
            "misses_per_miss_call": mean([m for _, m in per_call if m > 0])}


def batch_sweep(torch, B, H, S, compute, copy, batches=(1, 2, 4, 8, 12), n_layers=2, steps=8):
    """The paper's batching study (Section VI: batch sizes 1-12 activate more distinct experts per layer):
    per-layer decode latency of the Mixtral- and the Qwen-shaped layers at each batch size, with every
    expert resident and through the configured slots per layer without a predictor (every miss a fetch)."""
    import numpy as np
    from dataclasses import replace
    table = {}
    for name in ("c3_mixtral_decode", "c5_qwen_decode"):
        w0 = replace(S.WORKLOADS[name], L=n_layers, steps=steps)
        pools = [H.HostPool(w0, l) for l in range(n_layers)]
        rows = []
        for slots in (w0.E, w0.S):
            ctx = B.MoeContext(w0.d, w0.I, w0.E, w0.k, n_layers, slots, w0.I_shared)
            layers = [H.DeviceLayer(ctx, w0, l, pools[l], list(range(slots))) for l in range(n_layers)]
            for bi, batch in enumerate(batches):
                w = replace(w0, T=batch)
                trace = S.markov_trace(w)
                buf = H.Buffers(ctx, batch)
                xs = [H.np_to_dev(S.activations(w, l, 0)) for l in range(n_layers)]
                biases = [[H.np_to_dev(S.trace_route_bias(trace[s, l], w.E)) for l in range(n_layers)]
                          for s in range(steps)]

                def one_pass():
                    for s in range(steps):
                        for l in range(n_layers):
                            ctx.moe_decode_layer(l, xs[l], batch, buf.y, buf.ws, compute, copy, biases[s][l], w.E)
                    torch.cuda.synchronize()

                one_pass()
                # a pass is 16 layer calls (a millisecond at the small batches): the median of three, so
                # that one hiccup of the host does not become a table entry; counters from the first
                ctx.moe_reset_stats()
                times = []
                for rep in range(3 if slots == w0.E else 1):
                    t0 = time.perf_counter()
                    one_pass()
                    times.append((time.perf_counter() - t0) * 1e6 / (steps * n_layers))
                    if rep == 0:
                        st = ctx.moe_get_stats(-1)
                us = sorted(times)[len(times) // 2]
                distinct = float(np.mean([len(set(trace[s, l].ravel().tolist()))
                                          for s in range(steps) for l in range(n_layers)]))
                if slots == w0.E:
                    rows.append({"batch": batch, "distinct_experts": distinct, "resident_us": us})
                else:
                    rows[bi][f"slots_{slots}_us"] = us
                    rows[bi][f"slots_{slots}_misses_per_layer"] = st["misses"] / st["layer_calls"]
            ctx.close()
            del layers
        table[name] = rows
    return table


def oracle_single_thread_c1(S):
    """The oracle on config 1 in full (64 tokens, 8 experts, top-2) on ONE thread: tokens per second."""
    import ctypes
    import oracle
    omp = ctypes.CDLL("libgomp.so.1")
    before = omp.omp_get_max_threads()
    w = S.WORKLOADS["c1_tiny"]
    x = S.activations(w)
    wr = S.router_weight(w, 0)
    blobs = [S.expert_blob(w, 0, e) for e in range(w.E)]
    omp.omp_set_num_threads(1)
    try:
        oracle.moe_layer(x, wr, blobs, w.k)
        t0 = time.perf_counter()
        n = 3
        for _ in range(n):
            oracle.moe_layer(x, wr, blobs, w.k)
        dt = (time.perf_counter() - t0) / n
    finally:
        omp.omp_set_num_threads(before)
    return {"workload": "c1_tiny in full", "threads": 1, "seconds": dt, "tokens_per_s": w.T / dt}


def host_cores():
    """(threads the OpenMP oracle uses, physical cores, logical CPUs) of this host."""
    import ctypes
    logical = os.cpu_count()
    phys = set()
    try:
        pid = cid = None
        for line in open("/proc/cpuinfo"):
            if line.startswith("physical id"):
                pid = line.split(":")[1].strip()
            elif line.startswith("core id"):
                cid = line.split(":")[1].strip()
            elif not line.strip():
                if pid is not None and cid is not None:
                    phys.add((pid, cid))
                pid = cid = None
    except OSError:
        pass
    try:
        threads = int(ctypes.CDLL("libgomp.so.1").omp_get_max_threads())
    except OSError:
        threads = int(os.environ.get("OMP_NUM_THREADS", logical))
    return threads, (len(phys) or None), logical


def cpu_baseline(args, S, w, res, n_tokens):
    """The CPU oracle on a bounded sample: full routing + dispatch, expert math on n_tokens tokens."""
    import numpy as np
    import oracle
    pool, lay = res["pool"], res["lay"]
    blobs = [pool.ptr(e) for e in range(w.E)]
    bias = None if res["bias"] is None else res["bias"].cpu().numpy()
    sel = np.linspace(0, w.T - 1, n_tokens).astype(np.int32)
    t0 = time.perf_counter()
    logits = oracle.router_logits(res["x_np"], lay.router_np, bias)
    ids, wts = oracle.topk_weights(logits, w.k)
    oracle.dispatch(ids, w.E)
    t_route = time.perf_counter() - t0
    t0 = time.perf_counter()
    out16, out64 = oracle.moe_tokens(res["x_np"], blobs, ids, wts, sel, lay.shared_np, w.I, w.I_shared)
    t_exp = time.perf_counter() - t0
    tok_s = 1.0 / (t_route / w.T + t_exp / n_tokens)
    return dict(value=tok_s, t_route_s=t_route, t_expert_s=t_exp, sel=sel, out64=out64, ids=ids)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps; the device needs ~15 layer calls after idle to settle its clocks")
    ap.add_argument("--workload", default="c2_mixtral_prefill")
    ap.add_argument("--cpu-tokens", type=int, default=1536, help="tokens of the workload the CPU oracle computes")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (a reference for hardware byte counters)")
    ap.add_argument("--large-batch", type=int, default=16,
                    help="also time the layer on this many times the workload's tokens (0 or 1: skip)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-offloaded", action="store_true")
    ap.add_argument("--no-q8", action="store_true", help="skip the legs with quantised host pools")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--decode-layers", type=int, default=8, help="layers of the decode workload held in memory")
    ap.add_argument("--decode-steps", type=int, default=32)
    ap.add_argument("--settle-s", type=float, default=0.5,
                    help="seconds of untimed steps before the warm-up steps (clock ramp after idle)")
    ap.add_argument("--no-c4", action="store_true", help="skip the DeepSeek-shaped prefill leg")
    ap.add_argument("--no-c5", action="store_true", help="skip the Qwen-shaped batch-8 decode leg")
    ap.add_argument("--no-batch-sweep", action="store_true", help="skip the batch 1-12 decode table")
    ap.add_argument("--only", choices=["c4", "c5"], default=None,
                    help="run just the DeepSeek-shaped prefill leg or the Qwen-shaped decode leg and print it "
                         "(for profiler runs: rocprofv3 --kernel-trace / --pmc around a short command)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2509_07379_amd import binding as B, harness as H, synth as S
    B.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = S.WORKLOADS[args.workload]

    # one compute, one copy and one prediction stream for the whole run: HIP multiplexes streams
    # onto 4 hardware queues, and two streams that land on the same queue serialise
    compute, copy, pred = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    def calibration_copy():
        # a copy kernel of known size: FETCH_SIZE / WRITE_SIZE of the library's launches are scaled by what
        # the same counters read for these 256 MiB in and 256 MiB out
        src = torch.full((64 << 20,), 3, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    if args.only:
        leg = (prefill_c4(args, torch, B, H, S, compute, copy) if args.only == "c4"
               else decode_c5(args, torch, B, H, S, compute, copy, pred))
        if args.calibration_copy:
            calibration_copy()
        print(json.dumps({"leg": args.only, **leg}), flush=True)
        return
    res = prefill_resident(args, torch, B, H, S, w, compute, copy)
    if args.calibration_copy:
        calibration_copy()
    ms = res["ms"]
    tok_s = w.T / (ms * 1e-3)
    k = res["kern_ms"]
    n_assign = w.T * w.k
    flops1 = 4.0 * n_assign * w.d * w.I            # gate + up projections
    flops2 = 2.0 * n_assign * w.d * w.I            # down projection
    tf1 = flops1 / (k["gemm1"] * 1e-3) / 1e12 if k["gemm1"] else 0.0
    tf2 = flops2 / (k["gemm2"] * 1e-3) / 1e12 if k["gemm2"] else 0.0
    log(f"[bench] {w.name}: {ms:.3f} ms/step, {tok_s:,.0f} tok/s; kernels(ms) {k}")
    log(f"[bench] gemm1 {tf1:.0f} TFLOP/s ({tf1 / PEAK_BF16_TFLOPS:.1%}), gemm2 {tf2:.0f} TFLOP/s "
        f"({tf2 / PEAK_BF16_TFLOPS:.1%})")

    line = {
        "metric": "MoE-layer prefill tokens/s (MFMA util %) + decode per-layer latency us (HBM GB/s)",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "settle_steps_before_warmup": res["settle_steps"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: d={w.d} I={w.I} E={w.E} top-{w.k} T={w.T}, one MoE layer, "
                               f"experts resident in HBM (S=E)", "counts": res["routing"]["counts"].tolist()},
        "roofline": {"bound": "mfma", "kernel": "grouped_gemm SwiGLU (gate+up)", "achieved": tf1,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tf1 / PEAK_BF16_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(w.name), "traffic_unit": "bytes/launch",
                     "traffic_source": f"{TRAFFIC_PROFILE} (rocprofv3 --pmc of this command; not measured by this run)",
                     "flops_per_launch": flops1, "avg_launch_ms": k["gemm1"]},
        "kernels_ms": k,
        "gemm2": {"achieved": tf2, "unit": "TFLOP/s", "frac": tf2 / PEAK_BF16_TFLOPS},
        "mfma_util_layer": (flops1 + flops2) / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
    }

    if args.large_batch > 1:
        line["large_batch"] = prefill_large_batch(args, torch, B, H, S, w, res, args.large_batch)
        log(f"[bench] large batch: {line['large_batch']}")

    if not args.no_offloaded and w.S and w.S < w.E:
        off = prefill_offloaded(args, torch, B, H, S, w, res["pool"], res["x"], compute, copy)
        t_attn = off["timed"](off["attention"], 5)
        t_k = ms + t_attn
        t_c, t_p = off["t_copy_ms"], off["t_pipelined_ms"]
        line["offloaded"] = {
            "slots": w.S, "ms_per_layer": t_p, "tokens_per_s": w.T / (t_p * 1e-3),
            "t_copy_alone_ms": t_c, "t_compute_alone_ms": t_k, "attention_standin_ms": t_attn,
            "h2d_GBps": off["bytes_per_layer"] / (t_c * 1e-3) / 1e9,
            "h2d_frac_of_pcie5_x16": off["bytes_per_layer"] / (t_c * 1e-3) / 1e9 / PEAK_PCIE_GBS,
            "overlap": (t_c + t_k - t_p) / min(t_c, t_k), "exposed_copy_frac": (t_p - t_k) / t_c,
            # share of the pipelined layer during which the host link moves expert bytes at its measured rate
            "link_busy_frac": t_c / t_p,
        }
        log(f"[bench] offloaded: {line['offloaded']}")
        formats = {"offloaded_q8": (1, "e4m3 codes + fp32 scale per row"),
                   "offloaded_mxfp4": (3, "MXFP4: e2m1 codes + one power-of-two scale byte per 32 weights"),
                   "offloaded_q4": (2, "4-bit codes in groups of 128 + fp32 scale and zero point per group")}
        for key, (fmt, what) in ({} if args.no_q8 else formats).items():
            oq = prefill_offloaded(args, torch, B, H, S, w, None, res["x"], compute, copy, fmt=fmt)
            t_c, t_p = oq["t_copy_ms"], oq["t_pipelined_ms"]
            line[key] = {
                "host_format": what + (": the cache holds the quantised blobs, the GEMMs expand tiles on their way into LDS"
                                       if fmt in (1, 3) else ", expanded into the bf16 slots by a kernel behind each copy"),
                "slots": w.S, "ms_per_layer": t_p, "tokens_per_s": w.T / (t_p * 1e-3), "t_copy_alone_ms": t_c,
                "bytes_per_layer": oq["bytes_per_layer"], "h2d_GBps": oq["bytes_per_layer"] / (t_c * 1e-3) / 1e9,
                "overlap": (t_c + t_k - t_p) / min(t_c, t_k), "link_busy_frac": t_c / t_p,
            }
            if "t_resident_ms" in oq:
                # overlap above is against the bf16 layer's compute time; this is the quantised layer's own
                own = oq["t_resident_ms"] + t_attn
                line[key]["resident_ms_per_layer"] = oq["t_resident_ms"]
                line[key]["overlap_own_compute"] = (t_c + own - t_p) / min(t_c, own)
            log(f"[bench] {key}: {line[key]}")

    if not args.no_c4:
        line["prefill_c4"] = prefill_c4(args, torch, B, H, S, compute, copy)
        log(f"[bench] prefill_c4: {line['prefill_c4']}")
    if not args.no_c5:
        line["decode_c5"] = decode_c5(args, torch, B, H, S, compute, copy, pred)
        log(f"[bench] decode_c5: {line['decode_c5']}")
    if not args.no_batch_sweep:
        line["batch_sweep"] = batch_sweep(torch, B, H, S, compute, copy)
        log(f"[bench] batch_sweep: {line['batch_sweep']}")

    if not args.no_decode:
        wd = S.WORKLOADS["c3_mixtral_decode"]
        dec = decode_regime(args, torch, B, H, S, wd, args.decode_layers, args.decode_steps, compute, copy, pred)
        bytes_layer = wd.k * wd.blob_bytes  # batch 1: k distinct experts streamed once
        r = dec["resident"]
        gemv_ms = r["gemv1_ms"] + r["gemv2_ms"]
        line["decode"] = {
            "workload": f"{wd.name}: d={wd.d} I={wd.I} E={wd.E} top-{wd.k} batch {wd.T}, "
                        f"{args.decode_layers} of {wd.L} layers in memory, {args.decode_steps} steps",
            "resident_us_per_layer": r["us_per_layer"],
            "gemv_us_per_layer": gemv_ms * 1e3,
            "gemv_HBM_GBps": bytes_layer / (gemv_ms * 1e-3) / 1e9 if gemv_ms else 0.0,
            "gemv_frac_of_hbm_peak": bytes_layer / (gemv_ms * 1e-3) / 1e9 / PEAK_HBM_GBS if gemv_ms else 0.0,
            "layer_HBM_GBps": bytes_layer / (r["us_per_layer"] * 1e-6) / 1e9,
            "resident_batch8": r["batch8"],
            "cached_us_per_layer": dec["cached"]["us_per_layer"], "cached_slots": wd.S,
            "cached_stats": dec["cached"]["stats"], "cached": dec["cached"],
            # the paper's cache: one set of k slots for all layers, predictor top-k, first layer on demand
            "shared_k_us_per_layer": dec["shared_k"]["us_per_layer"], "shared_k_slots": wd.k,
            "shared_k_stats": dec["shared_k"]["stats"],
            "mlp_predictor": mlp_predictor_latency(torch, B, H, S, wd, pred),
        }
        if not args.no_q8:
            # the same kernel regime with experts fetched from an 8-bit host pool: the mat-vecs stream the codes
            line["decode"]["resident_q8"] = decode_resident_q8(args, torch, B, H, S, wd, min(2, args.decode_layers),
                                                               args.decode_steps, compute, copy)
            # and from an MXFP4 pool (the mat-vecs stream 4-bit codes and block scales)
            line["decode"]["resident_mxfp4"] = decode_resident_q8(args, torch, B, H, S, wd, min(2, args.decode_layers),
                                                                  args.decode_steps, compute, copy, fmt=3)
        log(f"[bench] decode: {line['decode']}")

    if not args.no_cpu_baseline:
        cb = cpu_baseline(args, S, w, res, args.cpu_tokens)
        # the sampled outputs double as a full-size parity spot check of this very run
        got = S.bf16_to_f32(H.dev_to_np_u16(res["buf"].y)[cb["sel"]]).astype(np.float64)
        err = np.abs(got - cb["out64"])
        ok = bool(np.all(err <= 1e-2 + 2e-2 * np.abs(cb["out64"])) and
                  np.array_equal(cb["ids"], res["routing"]["ids"]))
        threads, physical, logical = host_cores()
        line["cpu_baseline"] = {
            "value": cb["value"], "unit": "tokens/s", "cores": threads, "physical_cores": physical,
            "logical_cpus": logical, "kind": "oracle", "single_thread": oracle_single_thread_c1(S),
            "sample": f"routing+dispatch on all {w.T} tokens ({cb['t_route_s']:.2f}s), expert math on "
                      f"{args.cpu_tokens} evenly spaced tokens ({cb['t_expert_s']:.1f}s); rate extrapolated",
            "parity_on_sample": ok, "max_abs_err_on_sample": float(err.max()),
        }
        log(f"[bench] cpu oracle: {line['cpu_baseline']}")

    res["ctx"].close()
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
