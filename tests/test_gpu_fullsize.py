"""Parity at the full sizes of the workload list, in the launch configuration bench.py times.

Routing tables are compared in full (integers, cheap on the CPU); layer outputs on sampled tokens
that the oracle computes one by one.  Needs an MI355X.
"""
from dataclasses import replace

import numpy as np
import pytest

from paper_2509_07379_amd import synth as S

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

from test_gpu_parity import check_out, gpu  # noqa: E402,F401  (fixture + tolerance)


def sample_tokens(T, n, seed=0):
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(T, size=min(n, T), replace=False)).astype(np.int32)


def ids_against_fp64_logits(oracle, x_np, router_np, bias_np, k, gpu_ids, tag):
    """The Top-k is taken on fp32 logits summed in a fixed order, which the oracle replays.  Independently
    of that order: wherever the fp64 logits separate the k-th from the (k+1)-th expert by more than
    1e-4 of the largest logit, the selected SET must be the fp64 one.  Returns the tokens under the margin."""
    _, l64 = oracle.router_logits(x_np, router_np, bias_np, want_f64=True)
    E = l64.shape[1]
    order = np.lexsort((np.broadcast_to(np.arange(E), l64.shape), -l64), axis=1)   # logit descending, id ascending
    if k == E:
        return 0
    srt = np.take_along_axis(l64, order, 1)
    clear = (srt[:, k - 1] - srt[:, k]) > 1e-4 * np.abs(l64).max()
    want = np.sort(order[:, :k], 1)
    got = np.sort(gpu_ids, 1)
    bad = np.nonzero(clear & np.any(want != got, axis=1))[0]
    assert bad.size == 0, f"{tag}: tokens {bad[:8]} differ from the fp64 Top-k although the margin is clear"
    under = int((~clear).sum())
    print(f"{tag}: {under} of {l64.shape[0]} tokens have a k/(k+1) margin under 1e-4 of the largest logit")
    return under


def prefill_case(gpu, oracle, w, slots, n_sample, prefetch=None, with_attention=False, layer=0, fmt=0):
    """One prefill layer of workload w; `layer` picks the seeded weights, activations and (config 4) the
    rank permutation of the popularity bias; fmt: the experts' format in the CPU expert cache (the oracle
    then runs on its own expansion of the same blobs)."""
    H, B = gpu["harness"], gpu["binding"]
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, layer + 1, slots, w.I_shared, host_format=fmt)   # only `layer` is bound
    pool = H.HostPool(w, layer, fmt=fmt)
    initial = list(range(w.E)) if slots == w.E else None
    lay = H.DeviceLayer(ctx, w, layer, pool, initial, poison=initial is None)
    buf = H.Buffers(ctx, w.T)
    x_np = S.activations(w, layer, 0)
    x = H.np_to_dev(x_np)
    bias_np = S.zipf_route_bias(w, layer) if w.zipf_s > 0 else None
    bias = None if bias_np is None else H.np_to_dev(bias_np)
    torch.cuda.synchronize()
    if prefetch is not None:
        ctx.expert_cache_prefetch(layer, prefetch, gpu["copy"])
    if with_attention:  # stand-in non-MoE block the first fetches hide behind (Section V-B)
        wa = H.np_to_dev(S.normal_bf16((w.d, w.d), w.seed, S.stream_id(S.KIND_ATTN), 0.02))
        tmp = torch.empty((w.T, w.d), dtype=torch.int16, device="cuda")
        B.moe_dense_gemm_bf16(x, wa, tmp, w.T, w.d, w.d, gpu["compute"])
    ctx.moe_prefill_layer(layer, x, w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"], bias, 0)
    gpu["compute"].synchronize()
    out = H.dev_to_np_u16(buf.y)
    routing = buf.routing(ctx, gpu["compute"])
    stats, state = ctx.moe_get_stats(layer), ctx.moe_cache_state(layer)
    ctx.close()
    sel = sample_tokens(w.T, n_sample, seed=layer)
    expand = {1: oracle.dequant_blob, 2: oracle.dequant4_blob, 3: oracle.dequant_mx4_blob}.get(fmt)
    blobs = [expand(pool.blob_np(e), w.d, w.I) if fmt else pool.ptr(e) for e in range(w.E)]
    ref = oracle.moe_layer(x_np, lay.router_np, blobs, w.k, bias=bias_np, sel=sel,
                           shared_blob=lay.shared_np, I=w.I, I_shared=w.I_shared)
    for key in ("ids", "counts", "offsets", "perm", "inv_perm"):
        np.testing.assert_array_equal(routing[key], ref[key], err_msg=key)
    ids_against_fp64_logits(oracle, x_np, lay.router_np, bias_np, w.k, routing["ids"], f"{w.name} layer {layer}")
    np.testing.assert_allclose(routing["w"], ref["w"], rtol=2e-5, atol=1e-7)
    check_out(out[sel], ref["out_f64"], w.name)
    return dict(out=out, routing=routing, stats=stats, state=state, ref=ref)


def test_c2_mixtral_prefill_resident(gpu, oracle):
    """The configuration bench.py times: all 8 experts resident, one grouped launch."""
    w = S.WORKLOADS["c2_mixtral_prefill"]
    r = prefill_case(gpu, oracle, w, w.E, 320)
    assert r["stats"]["misses"] == 0 and r["stats"]["bytes_h2d"] == 0
    assert r["routing"]["counts"].sum() == w.T * w.k


def test_c2_mixtral_prefill_two_slots_matches_resident(gpu, oracle):
    """GPU expert cache of 2 (Section V-A): experts stream from pinned memory, same bits out."""
    from oracle.cache_sim import CacheSim
    w = S.WORKLOADS["c2_mixtral_prefill"]
    res = prefill_case(gpu, oracle, w, w.E, 8)
    off = prefill_case(gpu, oracle, w, w.S, 8, prefetch=list(range(w.S)), with_attention=True)
    np.testing.assert_array_equal(off["out"], res["out"])
    sim = CacheSim(w.E, w.S, w.blob_bytes)
    sim.prefetch(range(w.S))
    sim.serve(np.nonzero(res["routing"]["counts"])[0])
    assert off["stats"] == {**sim.counters(), "layer_calls": 1}
    assert off["state"] == sim.slot_expert
    assert off["stats"]["bytes_h2d"] == w.E * w.blob_bytes  # every expert fetched exactly once


def test_c2_shape_large_batch_rows_beyond_2gib(gpu, oracle):
    """A prefill batch of 20 sequences: the sorted intermediate rows H span more than 2 GiB, so the
    down projection's tiles sit past the reach of a 31-bit byte offset from the start of H."""
    w = replace(S.WORKLOADS["c2_mixtral_prefill"], name="c2_shape_T40960", T=40960)
    assert w.T * w.k * w.I * 2 > 2 ** 31
    r = prefill_case(gpu, oracle, w, w.E, 16)
    assert r["routing"]["offsets"][-1] == w.T * w.k
    # sampled tokens include rows of the last experts, which lie in the upper part of H
    last_rows = r["routing"]["inv_perm"].reshape(w.T, w.k)[sample_tokens(w.T, 16)].max()
    assert int(last_rows) * w.I * 2 > 2 ** 31


@pytest.mark.parametrize("layer", [0, 1, 2, 3, 27])
def test_c4_deepseek_prefill_layer(gpu, oracle, layer):
    """64 routed experts top-6 with Zipf-skewed popularity + shared experts, 16 slots; five of the 28
    layers, each with its own weights, activations and rank permutation of the popularity bias."""
    from oracle.cache_sim import CacheSim
    w = S.WORKLOADS["c4_deepseek_prefill"]
    r = prefill_case(gpu, oracle, w, w.S, 32, prefetch=list(range(w.S)), layer=layer)
    counts = r["routing"]["counts"]
    assert counts.max() > 8 * max(1, counts[counts > 0].min())  # the load really is imbalanced
    sim = CacheSim(w.E, w.S, w.blob_bytes)
    sim.prefetch(range(w.S))
    sim.serve(np.nonzero(counts)[0])
    assert r["stats"] == {**sim.counters(), "layer_calls": 1}
    assert r["state"] == sim.slot_expert


@pytest.mark.parametrize("fmt", [1, 3])
def test_c4_shape_quantised_experts_through_16_slots(gpu, oracle, fmt):
    """The same layer on e4m3 / MXFP4 experts, 64 of them streaming through 16 slots of quantised blobs
    (single-expert launches of the persistent kernel behind each copy, the last fetch split), and with
    every expert resident (one launch over all groups from the work plans)."""
    from oracle.cache_sim import CacheSim
    w = S.WORKLOADS["c4_deepseek_prefill"]
    r = prefill_case(gpu, oracle, w, w.S, 32, prefetch=list(range(w.S)), fmt=fmt)
    nbytes = S.q8_blob_bytes(w.d, w.I) if fmt == 1 else S.mx4_blob_bytes(w.d, w.I)
    sim = CacheSim(w.E, w.S, nbytes)
    sim.prefetch(range(w.S))
    sim.serve(np.nonzero(r["routing"]["counts"])[0])
    assert r["stats"] == {**sim.counters(), "layer_calls": 1}
    assert r["state"] == sim.slot_expert
    res = prefill_case(gpu, oracle, w, w.E, 32, fmt=fmt)
    assert res["stats"]["misses"] == 0 and res["stats"]["bytes_h2d"] == 0


def decode_case(gpu, oracle, w, n_layers, steps, check_every=1):
    """Decode steps with trace-driven routing, the linear predictor one layer ahead, prefetch and
    re-fetch; routing tables of every layer call and outputs of every check_every-th step are checked
    against the oracle, the counters and slot contents against the simulator (after every call)."""
    from oracle.cache_sim import CacheSim
    H, B = gpu["harness"], gpu["binding"]
    w = replace(w, L=n_layers, steps=steps)
    pred = torch.cuda.Stream()
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, n_layers, w.S, w.I_shared)
    pools = [H.HostPool(w, l) for l in range(n_layers)]
    init = list(range(w.S))
    lays = [H.DeviceLayer(ctx, w, l, pools[l], init) for l in range(n_layers)]
    wps_np = [S.predictor_weight(w, l) for l in range(n_layers)]
    wps = [H.np_to_dev(a) for a in wps_np]
    sims = [CacheSim(w.E, w.S, w.blob_bytes, init) for _ in range(n_layers)]
    trace = S.markov_trace(w)
    buf = H.Buffers(ctx, w.T)
    top = torch.zeros(w.top_m, dtype=torch.int32).pin_memory()
    for s in range(steps):
        for l in range(n_layers):
            x_np = S.activations(w, l, s)
            x = H.np_to_dev(x_np)
            bias_np = S.trace_route_bias(trace[s, l], w.E)
            bias = H.np_to_dev(bias_np)
            if l + 1 < n_layers:
                ctx.predictor_score(l + 1, x, w.T, wps[l + 1], w.top_m, top, pred)
            ctx.moe_decode_layer(l, x, w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"], bias, w.E)
            gpu["compute"].synchronize()
            out = H.dev_to_np_u16(buf.y)
            routing = buf.routing(ctx, gpu["compute"])
            full = s % check_every == 0 or s == steps - 1
            ref = oracle.moe_layer(x_np, lays[l].router_np, [pools[l].ptr(e) for e in range(w.E)], w.k,
                                   bias=bias_np, shared_blob=lays[l].shared_np, I=w.I, I_shared=w.I_shared,
                                   sel=None if full else np.zeros(0, dtype=np.int32))
            for key in ("ids", "counts", "offsets", "perm", "inv_perm"):
                np.testing.assert_array_equal(routing[key], ref[key], err_msg=f"{key} step {s} layer {l}")
            assert np.array_equal(np.sort(ref["ids"], 1), np.sort(trace[s, l], 1))  # the trace drives routing
            if full:
                check_out(out, ref["out_f64"], f"{w.name} step {s} layer {l}")
            sims[l].serve(np.nonzero(ref["counts"])[0])
            assert ctx.moe_cache_state(l) == sims[l].slot_expert, f"step {s} layer {l}"
            if l + 1 < n_layers:
                pred.synchronize()
                _, ref_top = oracle.predictor_score(x_np, wps_np[l + 1], w.top_m)
                np.testing.assert_array_equal(top.numpy(), ref_top)
                ctx.expert_cache_prefetch(l + 1, top.tolist(), gpu["copy"])
                sims[l + 1].prefetch(ref_top)
    torch.cuda.synchronize()
    for l in range(n_layers):
        st = ctx.moe_get_stats(l)
        assert st == {**sims[l].counters(), "layer_calls": steps}, f"layer {l}"
        assert ctx.moe_cache_state(l) == sims[l].slot_expert
        full = ctx.moe_get_stats(l, full=True)
        # every prefetched expert that was used either had landed or made the compute stream wait
        assert full["prefetch_ready"] + full["prefetch_stalled"] == full["prefetch_useful"]
    ctx.close()


def test_c3_mixtral_decode_steps(gpu, oracle):
    decode_case(gpu, oracle, S.WORKLOADS["c3_mixtral_decode"], n_layers=2, steps=32, check_every=4)


def test_c5_qwen_decode_steps(gpu, oracle):
    decode_case(gpu, oracle, S.WORKLOADS["c5_qwen_decode"], n_layers=3, steps=32, check_every=4)


@pytest.mark.parametrize("fmt", [1, 3])
def test_c2_shape_quantised_host_pool(gpu, oracle, fmt):
    """The Mixtral-shaped layer served from an 8-bit (e4m3 rows) or MXFP4 CPU expert cache at full size:
    prefill through two slots (every expert fetched and used once; the GEMMs read the codes as fetched
    and expand tiles on their way into LDS), then decode on resident experts, where the mat-vec kernels
    stream the same blobs.  Outputs on sampled tokens against the oracle run on its
    own expansion of the same blobs."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.WORKLOADS["c2_mixtral_prefill"]
    pool = H.HostPool(w, 0, fmt=fmt)
    expand = {1: oracle.dequant_blob, 3: oracle.dequant_mx4_blob}[fmt]
    blobs = [expand(pool.blob_np(e), w.d, w.I) for e in range(w.E)]
    x_np = S.activations(w)

    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, 2, 0, True, host_format=fmt)
    lay = H.DeviceLayer(ctx, w, 0, pool, None, poison=True)
    buf = H.Buffers(ctx, w.T)
    x = H.np_to_dev(x_np)
    ctx.expert_cache_prefetch(0, [0, 1], gpu["copy"])
    ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"])
    gpu["compute"].synchronize()
    sel = sample_tokens(w.T, 12)
    ref = oracle.moe_layer(x_np, lay.router_np, blobs, w.k, sel=sel, I=w.I)
    routing = buf.routing(ctx, gpu["compute"])
    for key in ("ids", "counts", "perm"):
        np.testing.assert_array_equal(routing[key], ref[key], err_msg=key)
    check_out(H.dev_to_np_u16(buf.y)[sel], ref["out_f64"], f"format {fmt} prefill through two slots")
    st = ctx.moe_get_stats(0)
    assert st["bytes_h2d"] == w.E * pool.bytes_per_expert and st["misses"] == w.E - 2
    ctx.close()

    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E, 0, True, host_format=fmt)
    lay = H.DeviceLayer(ctx, w, 0, pool, None, poison=True)
    ctx.expert_cache_prefetch(0, list(range(w.E)), gpu["copy"])
    torch.cuda.synchronize()
    for T in (1, 4, 8, 24):    # 8 and 24: groups of several tokens, the matrix-core mat-vec on the copies
        buf = H.Buffers(ctx, T)
        ctx.moe_decode_layer(0, H.np_to_dev(x_np[:T]), T, buf.y, buf.ws, gpu["compute"], gpu["copy"])
        gpu["compute"].synchronize()
        ref = oracle.moe_layer(x_np[:T], lay.router_np, blobs, w.k, I=w.I)
        np.testing.assert_array_equal(buf.routing(ctx, gpu["compute"])["ids"], ref["ids"])
        check_out(H.dev_to_np_u16(buf.y), ref["out_f64"], f"format {fmt} decode T={T}")
    ctx.close()


@pytest.mark.parametrize("fmt", [1, 3])
@pytest.mark.parametrize("workload", ["c2_mixtral_prefill", "c4_deepseek_prefill"])
def test_full_size_quantised_gemm_kernels_agree(gpu, fmt, workload):
    """Quantised experts, every expert resident, at full size (Mixtral shape: 64 and 224 K steps, blocks that
    walk over several tiles in a fixed order; DeepSeek shape: 64 experts of very different size, work plans
    with queues, short row tiles, shared experts beside them): the persistent kernel, which builds its B fragments from the codes in LDS, against the
    single-phase kernel, which expands code tiles into LDS.  Gate/up sums are formed in the same order, so
    with the down GEMM on the same kernel in both runs the outputs are equal bit for bit; with both GEMMs
    on the persistent kernel (other K slices of the down projection) they agree within the bf16 tolerance."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.WORKLOADS[workload]
    pool = H.HostPool(w, 0, fmt=fmt)
    x = H.np_to_dev(S.activations(w))
    bias = H.np_to_dev(S.zipf_route_bias(w, 0)) if w.zipf_s else None
    outs = {}
    for name, tunes in (("single-phase", [(0, 6), (1, 6)]), ("gate/up persistent", [(1, 6)]), ("persistent", [])):
        ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E, w.I_shared, True, host_format=fmt)
        lay = H.DeviceLayer(ctx, w, 0, pool, list(range(w.E)))
        buf = H.Buffers(ctx, w.T)
        for mode, variant in tunes:
            ctx.moe_tune(mode, variant)
        for _ in range(3):       # the launches' timing differs from call to call; the bits must not
            ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"], bias, 0)
            gpu["compute"].synchronize()
            out = H.dev_to_np_u16(buf.y)
            assert name not in outs or np.array_equal(outs[name], out), f"format {fmt}, {name}: not repeatable"
            outs[name] = out
        ctx.close()
    np.testing.assert_array_equal(outs["gate/up persistent"], outs["single-phase"])
    ref = S.bf16_to_f32(outs["single-phase"]).astype(np.float64)
    check_out(outs["persistent"], ref, f"format {fmt}: persistent against single-phase kernel")


@pytest.mark.parametrize("T", [8, 12])
def test_c3_shape_decode_batches_resident(gpu, oracle, T):
    """The Mixtral-shaped decode layer at the batch sizes bench.py also times (and the paper's largest,
    12), experts resident in bf16 slots: per-token mat-vecs for the gate/up rows, 16x16x32 MFMAs for the
    long down rows.  Every token against the oracle; routing tables bit for bit."""
    from dataclasses import replace
    H, B = gpu["harness"], gpu["binding"]
    w = replace(S.WORKLOADS["c3_mixtral_decode"], T=T, L=1)
    pool = H.HostPool(w, 0)
    x_np = S.activations(w)
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E, w.I_shared, True)
    lay = H.DeviceLayer(ctx, w, 0, pool, list(range(w.E)))
    buf = H.Buffers(ctx, T)
    ctx.moe_decode_layer(0, H.np_to_dev(x_np), T, buf.y, buf.ws, gpu["compute"], gpu["copy"])
    gpu["compute"].synchronize()
    blobs = [pool.blob_np(e) for e in range(w.E)]
    ref = oracle.moe_layer(x_np, lay.router_np, blobs, w.k, I=w.I)
    routing = buf.routing(ctx, gpu["compute"])
    for key in ("ids", "counts", "perm"):
        np.testing.assert_array_equal(routing[key], ref[key], err_msg=key)
    assert ref["counts"].max() >= 3
    check_out(H.dev_to_np_u16(buf.y), ref["out_f64"], f"decode batch {T}")
    st = ctx.moe_get_stats(0)
    assert st["misses"] == 0
    ctx.close()

