"""Parity of the HIP path (through the C ABI) with the CPU oracle.  Needs an MI355X."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2509_07379_amd import synth as S

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

# tolerance stated for bf16-in / fp32-accumulate outputs: 2e-2 relative + 1e-2 absolute
RTOL, ATOL = 2e-2, 1e-2


def check_out(got_bits, ref_f64, tag=""):
    """Element-wise |gpu - ref| <= ATOL + RTOL*|ref|, plus a scale-aware bound (the stated absolute
    term alone would hide errors on outputs much smaller than 1e-2)."""
    got = S.bf16_to_f32(got_bits).astype(np.float64)
    err = np.abs(got - ref_f64)
    assert np.all(np.isfinite(got)), tag
    assert np.all(err <= ATOL + RTOL * np.abs(ref_f64)), f"{tag}: max err {err.max()}"
    rms = float(np.sqrt(np.mean(ref_f64 ** 2)))
    assert np.all(err <= RTOL * np.abs(ref_f64) + RTOL * rms), f"{tag}: max err {err.max()} rms {rms}"


# Tuning hooks (csrc/moe_tuning.h) belong to a context: a test names the ones it wants with set_tune
# and every context made by new_ctx gets them; the fixture clears the list after each test.
TUNE = {}


def set_tune(mode, variant):
    TUNE[mode] = variant


def new_ctx(B, *args, **kw):
    ctx = B.MoeContext(*args, **kw)
    for mode, variant in TUNE.items():
        ctx.moe_tune(mode, variant)
    return ctx


@pytest.fixture(autouse=True)
def _default_hooks():
    yield
    TUNE.clear()


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests selected but no GPU is visible")
    from paper_2509_07379_amd import binding, harness
    binding.load()
    torch.cuda.set_device(0)
    return dict(binding=binding, harness=harness, compute=torch.cuda.Stream(), copy=torch.cuda.Stream())


def oracle_layer(oracle, w, x, router, pool, bias=None, sel=None, shared=None):
    blobs = [pool.blob_np(e) for e in range(w.E)]
    if pool.q8:   # quantised CPU expert cache: the layer computes with the oracle's expansion of it
        expand = {1: oracle.dequant_blob, 2: oracle.dequant4_blob, 3: oracle.dequant_mx4_blob}[pool.fmt]
        blobs = [expand(b, w.d, w.I) for b in blobs]
    return oracle.moe_layer(x, router, blobs, w.k, bias=bias, sel=sel, shared_blob=shared, I=w.I,
                            I_shared=w.I_shared)


def run_layer(gpu, w, T, x_np, S_slots, initial, decode=False, bias=None, prefetch=None, poison=False,
              pool=None, q8=False, fmt=None):
    H, B = gpu["harness"], gpu["binding"]
    fmt = (1 if q8 else 0) if fmt is None else fmt
    ctx = new_ctx(B, w.d, w.I, w.E, w.k, 1, S_slots, w.I_shared, True, host_format=fmt)
    pool = pool or H.HostPool(w, 0, fmt=fmt)
    lay = H.DeviceLayer(ctx, w, 0, pool, initial, poison=poison)
    buf = H.Buffers(ctx, T)
    x = H.np_to_dev(x_np)
    bias_t = None if bias is None else H.np_to_dev(bias)
    stride = 0 if bias is None or bias.ndim == 1 else w.E
    torch.cuda.synchronize()
    if prefetch is not None:
        ctx.expert_cache_prefetch(0, prefetch, gpu["copy"])
    fn = ctx.moe_decode_layer if decode else ctx.moe_prefill_layer
    fn(0, x, T, buf.y, buf.ws, gpu["compute"], gpu["copy"], bias_t, stride)
    gpu["compute"].synchronize()
    out = H.dev_to_np_u16(buf.y)
    routing = buf.routing(ctx, gpu["compute"])
    stats = ctx.moe_get_stats(0)
    state = ctx.moe_cache_state(0)
    ctx.close()
    return dict(out=out, routing=routing, stats=stats, state=state, pool=pool, lay=lay)


# ---------------------------------------------------------------- the MFMA tile itself
# The last five shapes take the persistent 256 x 256 kernel: a single K step, two K steps, a last
# column tile that overlaps its neighbour, row tiles with 1..4 fragments per wave, and more tiles
# than blocks (so blocks walk over several tiles).
@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (200, 136, 192), (8, 8, 8), (513, 264, 1096),
                                   (300, 256, 64), (257, 511, 128), (1000, 300, 512), (97, 2048, 192),
                                   (4136, 4360, 128)])
def test_dense_gemm_matches_matmul(gpu, M, N, K):
    a = S.normal_bf16((M, K), 1, 100 + M, 1.0)
    b = S.normal_bf16((N, K), 1, 200 + N, 1.0)
    H, B = gpu["harness"], gpu["binding"]
    c = torch.empty((M, N), dtype=torch.int16, device="cuda")
    B.moe_dense_gemm_bf16(H.np_to_dev(a), H.np_to_dev(b), c, M, N, K, gpu["compute"])
    gpu["compute"].synchronize()
    want = S.bf16_to_f32(a).astype(np.float64) @ S.bf16_to_f32(b).astype(np.float64).T
    got = S.bf16_to_f32(H.dev_to_np_u16(c)).astype(np.float64)
    assert np.all(np.abs(got - want) <= 2.0 ** -7 * np.abs(want) + 1e-3 * np.sqrt(K))


@pytest.mark.parametrize("variant", [1, 6, 12])
def test_every_gemm_kernel_on_one_layer(gpu, oracle, variant):
    """The shape heuristic picks one GEMM kernel per launch; here each of them is forced onto the same
    layer (groups of unequal height, shared experts, K a multiple of 64) and checked against the oracle."""
    B = gpu["binding"]
    w = S.Workload("variants", d=256, I=384, E=6, k=2, T=1100, I_shared=256, seed=33, zipf_s=1.1)
    x = S.activations(w)
    bias = S.zipf_route_bias(w, 0)
    try:
        for mode in (0, 1):
            set_tune(mode, variant)
        r = run_layer(gpu, w, w.T, x, w.E, list(range(w.E)), bias=bias)
    finally:
        for mode in (0, 1):
            set_tune(mode, 0)
    ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"], bias=bias, shared=r["lay"].shared_np)
    np.testing.assert_array_equal(r["routing"]["perm"], ref["perm"])
    check_out(r["out"], ref["out_f64"], f"gemm variant {variant}")


# ---------------------------------------------------------------- gate logits, bit for bit
@pytest.mark.parametrize("d,E,k,T", [(4096, 8, 2, 70), (2048, 64, 6, 131), (1024, 60, 4, 97), (264, 6, 2, 80),
                                     (4096, 8, 2, 5), (2048, 64, 6, 1)])
def test_gate_logits_bit_exact(gpu, oracle, d, E, k, T):
    """Both gate launches (four tokens per block for 64 tokens or more, one block per token for small
    batches) sum in the documented order: the logits equal the oracle's scalar replay bit for bit,
    with a per-token bias added last."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("logits", d=d, I=64, E=E, k=k, T=T, seed=61)
    x = S.activations(w)
    bias = S.normal_f32((T, E), 61, 900, 0.5)
    ctx = new_ctx(B, w.d, w.I, w.E, w.k, 1, w.E)
    pool = H.HostPool(w, 0)
    lay = H.DeviceLayer(ctx, w, 0, pool, list(range(E)))
    buf = H.Buffers(ctx, T)
    got = torch.empty((T, E), dtype=torch.float32, device="cuda")
    ctx.moe_prefill_layer(0, H.np_to_dev(x), T, buf.y, buf.ws, gpu["compute"], gpu["copy"],
                          H.np_to_dev(bias), E)
    ctx.moe_debug_logits(buf.ws, T, got, gpu["compute"])
    gpu["compute"].synchronize()
    want = oracle.router_logits(x, lay.router_np, bias)
    np.testing.assert_array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))
    ids, _ = oracle.topk_weights(want, k)
    np.testing.assert_array_equal(buf.routing(ctx, gpu["compute"])["ids"], ids)
    ctx.close()


# ---------------------------------------------------------------- config 1, all resident
def test_c1_routing_bit_exact_and_output(gpu, oracle):
    w = S.WORKLOADS["c1_tiny"]
    x = S.activations(w)
    r = run_layer(gpu, w, w.T, x, w.E, list(range(w.E)))
    ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"])
    for key in ("ids", "counts", "offsets", "perm", "inv_perm"):
        np.testing.assert_array_equal(r["routing"][key], ref[key], err_msg=key)
    np.testing.assert_allclose(r["routing"]["w"], ref["w"], rtol=1e-5, atol=1e-7)
    check_out(r["out"], ref["out_f64"], "c1 prefill")
    assert r["stats"]["hits"] == int((ref["counts"] > 0).sum()) and r["stats"]["misses"] == 0
    assert r["stats"]["bytes_h2d"] == 0


def test_c1_decode_kernels_same_layer(gpu, oracle):
    # the mat-vec path on the same 64 tokens (several passes of 8 tokens per expert)
    w = S.WORKLOADS["c1_tiny"]
    x = S.activations(w)
    r = run_layer(gpu, w, w.T, x, w.E, list(range(w.E)), decode=True)
    ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"])
    np.testing.assert_array_equal(r["routing"]["perm"], ref["perm"])
    check_out(r["out"], ref["out_f64"], "c1 decode kernels")


# ---------------------------------------------------------------- ragged shapes, biases, shared experts
@pytest.mark.parametrize("d,I,E,k,T,Ish", [(256, 384, 60, 4, 333, 0), (512, 128, 64, 6, 777, 256),
                                           (128, 64, 8, 2, 1, 0), (256, 192, 5, 5, 37, 64),
                                           # large groups of unequal height: the persistent GEMM's ragged tiles
                                           (512, 640, 4, 2, 1500, 384), (256, 320, 8, 2, 2900, 0),
                                           # one token: many experts (only the active ones are launched) and few
                                           # (one launch for all, the wider shared expert in further grid rows)
                                           (256, 384, 60, 4, 1, 256), (256, 192, 8, 2, 1, 320)])
@pytest.mark.parametrize("decode", [False, True])
def test_ragged_shapes(gpu, oracle, d, I, E, k, T, Ish, decode):
    if decode and T > 64:
        T = 9
    w = S.Workload("rag", d=d, I=I, E=E, k=k, T=T, I_shared=Ish, seed=21, zipf_s=1.1)
    x = S.activations(w)
    bias = S.zipf_route_bias(w, 0)  # skewed popularity: some experts get few or no rows
    r = run_layer(gpu, w, T, x, E, list(range(E)), decode=decode, bias=bias)
    ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"], bias=bias, shared=r["lay"].shared_np)
    for key in ("ids", "counts", "offsets", "perm", "inv_perm"):
        np.testing.assert_array_equal(r["routing"][key], ref[key], err_msg=key)
    check_out(r["out"], ref["out_f64"], f"ragged decode={decode}")


@pytest.mark.parametrize("E,k,Ish", [(60, 4, 128), (8, 2, 0), (64, 6, 0)])
def test_one_token_decode_enqueued_from_the_gates_id_list(gpu, oracle, E, k, Ish):
    """One token, every expert resident: the call does not wait for the gate; the mat-vec launches
    take the k experts from the id list the gate wrote on the device.  Same output, routing tables and
    counters as the path in which the host looks at the counts first."""
    B = gpu["binding"]
    w = S.Workload("one_token", d=512, I=256, E=E, k=k, T=1, I_shared=Ish, seed=71)
    got = []
    for host_path in (0, 1):
        set_tune(5, 0 if host_path else 1)
        for step in range(3):                       # different tokens choose different experts
            x = S.activations(w, 0, step)
            r = run_layer(gpu, w, 1, x, E, list(range(E)), decode=True)
            ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"], shared=r["lay"].shared_np)
            for key in ("ids", "counts", "offsets", "perm", "inv_perm"):
                np.testing.assert_array_equal(r["routing"][key], ref[key], err_msg=key)
            check_out(r["out"], ref["out_f64"], f"one token, host_path={host_path}")
            assert r["stats"]["hits"] == k and r["stats"]["misses"] == 0
            got.append(r["out"])
    for a, b in zip(got[:3], got[3:]):
        np.testing.assert_array_equal(a, b)          # the same kernels on the same experts: the same bits


@pytest.mark.parametrize("fmt,d,I,E,k,Ish", [(f, d, I, E, k, Ish) for f in (0, 1, 3)
                                             for d, I, E, k, Ish in ((512, 256, 8, 2, 0), (4096, 64, 64, 6, 0),
                                                                     (264, 136, 5, 5, 0), (512, 256, 60, 4, 384),
                                                                     (256, 64, 8, 2, 2048))
                                             if f == 0 or (d % 64 == 0 and I % 64 == 0)])
def test_one_token_down_projection_and_weighted_sum_in_one_launch(gpu, oracle, fmt, d, I, E, k, Ish):
    """One token: the down mat-vec walks over the token's k experts, applies the gate values itself and
    adds the shared experts' rows.  The same bits as the two-launch path (same row sums, same order of
    the weighted sum), for bf16 slots and for the quantised copies; and the oracle's output."""
    B = gpu["binding"]
    w = S.Workload("fused_down", d=d, I=I, E=E, k=k, T=1, I_shared=Ish, seed=91)
    outs = []
    for two_launches in (0, 1):
        set_tune(7, two_launches)
        for step in range(2):
            x = S.activations(w, 0, step)
            r = run_layer(gpu, w, 1, x, E, None if fmt else list(range(E)), decode=True,
                          prefetch=list(range(E)) if fmt else None, fmt=fmt)
            ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"], shared=r["lay"].shared_np)
            check_out(r["out"], ref["out_f64"], f"fused down, format {fmt}, two_launches={two_launches}")
            outs.append(r["out"])
    np.testing.assert_array_equal(outs[0], outs[2])
    np.testing.assert_array_equal(outs[1], outs[3])


def test_per_token_bias_forces_trace(gpu, oracle):
    w = S.Workload("trace", d=256, I=128, E=60, k=4, T=8, seed=5, L=3, steps=2, p_stay=0.5)
    trace = S.markov_trace(w)
    x = S.activations(w)
    bias = S.trace_route_bias(trace[1, 2], w.E)
    r = run_layer(gpu, w, w.T, x, w.E, list(range(w.E)), decode=True, bias=bias)
    assert np.array_equal(np.sort(r["routing"]["ids"], 1), np.sort(trace[1, 2], 1))
    ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"], bias=bias)
    np.testing.assert_array_equal(r["routing"]["ids"], ref["ids"])
    check_out(r["out"], ref["out_f64"], "trace bias")


# ---------------------------------------------------------------- offloaded: results never depend on the cache
@pytest.mark.parametrize("up,down", [(0, 0), (2, 2), (1, 3), (2, 1)])
def test_work_plans_of_the_persistent_gemm(gpu, oracle, up, down):
    """The grouping kernel writes, per GEMM launch, the prefix of work items per group, eight item ranges
    and eight queue counters.  Recomputed here from the groups' sizes: items per group for both ways of
    cutting a group into row tiles, ranges that cover the list in order, and counters that show every range
    was emptied; the layer's output against the oracle under each schedule (0 = by shape: 32 experts take
    full tiles plus a remainder from queues)."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("plan", d=512, I=384, E=32, k=4, T=900, seed=77, zipf_s=1.1)
    x_np, bias = S.activations(w), S.zipf_route_bias(w, 0)
    ctx = new_ctx(B, w.d, w.I, w.E, w.k, 1, w.E, 0, True)
    ctx.moe_tune(12, up)
    ctx.moe_tune(11, down)
    pool = H.HostPool(w, 0)
    lay = H.DeviceLayer(ctx, w, 0, pool, list(range(w.E)))
    buf = H.Buffers(ctx, w.T)
    ctx.moe_prefill_layer(0, H.np_to_dev(x_np), w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"], H.np_to_dev(bias), 0)
    gpu["compute"].synchronize()
    routing = buf.routing(ctx, gpu["compute"])
    plans = ctx.moe_debug_plans(buf.ws, w.T, gpu["compute"])
    ref = oracle_layer(oracle, w, x_np, lay.router_np, pool, bias=bias)
    np.testing.assert_array_equal(routing["counts"], ref["counts"])
    check_out(H.dev_to_np_u16(buf.y), ref["out_f64"], f"schedules {up}/{down}")
    ctx.close()
    counts = ref["counts"].astype(np.int64)
    assert counts.max() > 256 and (counts % 256 != 0).any() and (counts < 64).any()   # the case is ragged
    # (launch, columns per column tile, schedule): a fixed order (1) uses no plan
    for plan, ntn, sched in ((plans[0], -(-w.I // 128), up or 2), (plans[1], -(-w.d // 256), down or 2)):
        if sched == 1:
            continue
        equal = sched == 3
        tiles = -(-counts // 256) if equal else counts // 256 + (counts % 256 > 0)
        s = plan["s_full"]
        assert s >= 1 and plan["s_rem"] == s
        begin = np.concatenate([[0], np.cumsum(tiles * ntn * s)])
        assert plan["item_begin"][:w.E + 1] == begin.tolist()
        assert plan["n_items"] == begin[-1] and all(v == begin[-1] for v in plan["item_begin"][w.E + 1:])
        xb = plan["xcd_begin"]
        assert xb[0] == 0 and xb[8] == plan["n_items"] and all(a <= b for a, b in zip(xb, xb[1:]))
        sizes = [b - a for a, b in zip(xb, xb[1:])]
        assert max(sizes) <= 2 * (plan["n_items"] / 8) + ntn * s * 2      # ranges of comparable cost
        assert all(q >= n for q, n in zip(plan["queue"], sizes)), (plan["queue"], sizes)


@pytest.mark.parametrize("decode", [False, True])
def test_streaming_through_two_slots_is_bit_identical(gpu, oracle, decode):
    from oracle.cache_sim import CacheSim
    w = S.WORKLOADS["c1_tiny"]
    T = 16 if decode else w.T
    x = S.activations(w, T=T)
    res = run_layer(gpu, w, T, x, w.E, list(range(w.E)), decode=decode)
    off = run_layer(gpu, w, T, x, 2, None, decode=decode, prefetch=[0, 1], poison=True)
    np.testing.assert_array_equal(off["out"], res["out"])  # same kernels, same numbers
    sim = CacheSim(w.E, 2, w.blob_bytes)
    sim.prefetch([0, 1])
    active = np.nonzero(res["routing"]["counts"])[0]
    sim.serve(active)
    assert off["stats"] == {**sim.counters(), "layer_calls": 1}
    assert off["state"] == sim.slot_expert
    # each active expert fetched exactly once (Section V-B)
    assert off["stats"]["bytes_h2d"] == len(set(active) | {0, 1}) * w.blob_bytes


def test_wrong_prediction_is_refetched_not_used(gpu, oracle):
    from oracle.cache_sim import CacheSim
    w = S.Workload("mis", d=256, I=128, E=8, k=2, T=1, seed=9)
    x = S.activations(w)
    res = run_layer(gpu, w, 1, x, 8, list(range(8)), decode=True)
    act = sorted(res["routing"]["ids"][0].tolist())
    wrong = [e for e in range(8) if e not in act][:3]
    off = run_layer(gpu, w, 1, x, 3, None, decode=True, prefetch=wrong, poison=True)
    np.testing.assert_array_equal(off["out"], res["out"])
    sim = CacheSim(8, 3, w.blob_bytes)
    sim.prefetch(wrong)
    sim.serve(act)
    assert off["stats"] == {**sim.counters(), "layer_calls": 1}
    assert off["stats"]["misses"] == 2 and off["stats"]["prefetch_useful"] == 0


# ---------------------------------------------------------------- one GPU expert cache for all layers
@pytest.mark.parametrize("slots,q8", [(2, False), (3, False), (2, True)])
def test_shared_cache_decode_steps(gpu, oracle, slots, q8):
    """Section V-A / V-C with the paper's cache size: ONE cache of k (or k + 1) experts serves every
    layer of a decode step in turn; the predictor of layer l + 1 runs on a third stream, its choice is
    prefetched into the slots that layer l frees, wrong guesses are fetched again.  Every layer call
    is checked against the oracle, counters and slot contents against the shared-cache simulator."""
    from oracle.cache_sim import SharedCacheSim
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("shared_cache", d=256, I=128, E=8, k=2, T=1, seed=17, L=4, steps=5, p_stay=0.6, top_m=2)
    ctx = new_ctx(B, w.d, w.I, w.E, w.k, w.L, slots, 0, True, shared_slots=True, host_format=1 if q8 else 0)
    pools = [H.HostPool(w, l, q8=q8) for l in range(w.L)]
    cache = torch.full((ctx.moe_cache_bytes() // 2,), 0x7FC0, dtype=torch.int16, device="cuda")  # NaN until filled
    lays = [H.DeviceLayer(ctx, w, l, pools[l], None, slots=cache) for l in range(w.L)]
    wps_np = [S.predictor_weight(w, l) for l in range(w.L)]
    wps = [H.np_to_dev(a) for a in wps_np]
    sim = SharedCacheSim(w.L, w.E, slots, pools[0].bytes_per_expert)
    trace = S.markov_trace(w)
    buf = H.Buffers(ctx, w.T)
    pred = torch.cuda.Stream()
    top = torch.zeros(w.top_m, dtype=torch.int32).pin_memory()
    for s in range(w.steps):
        for l in range(w.L):
            x_np = S.activations(w, l, s)
            x = H.np_to_dev(x_np)
            bias_np = S.trace_route_bias(trace[s, l], w.E)
            bias = H.np_to_dev(bias_np)
            nxt = l + 1                              # the first layer of a step has no prediction:
            if nxt < w.L:                            # its experts are fetched after the gate has chosen
                ctx.predictor_score(nxt, x, w.T, wps[nxt], w.top_m, top, pred)
            ctx.moe_decode_layer(l, x, w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"], bias, w.E)
            gpu["compute"].synchronize()
            ref = oracle_layer(oracle, w, x_np, lays[l].router_np, pools[l], bias=bias_np)
            np.testing.assert_array_equal(buf.routing(ctx, gpu["compute"])["ids"], ref["ids"])
            check_out(H.dev_to_np_u16(buf.y), ref["out_f64"], f"shared cache step {s} layer {l}")
            sim.serve(l, np.nonzero(ref["counts"])[0])
            assert ctx.moe_cache_state(l) == sim.state(l), f"step {s} layer {l}"
            if nxt == w.L:
                continue
            pred.synchronize()
            _, ref_top = oracle.predictor_score(x_np, wps_np[nxt], w.top_m)
            np.testing.assert_array_equal(top.numpy(), ref_top)
            ctx.expert_cache_prefetch(nxt, top.tolist(), gpu["copy"])
            sim.prefetch(nxt, ref_top)
            assert ctx.moe_cache_state(nxt) == sim.state(nxt)
    torch.cuda.synchronize()
    for l in range(w.L):
        assert ctx.moe_get_stats(l) == {**sim.counters(l), "layer_calls": w.steps}, f"layer {l}"
    ctx.close()


def test_shared_cache_prefill_streams_every_layer_through_two_slots(gpu, oracle):
    """Section V-B: the two slots of the one cache are in turn computed on and fetched into, layer after
    layer; each expert with tokens is fetched exactly once per layer and the output is the all-resident one."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("shared_prefill", d=256, I=128, E=8, k=2, T=96, seed=23, L=3)
    ctx = new_ctx(B, w.d, w.I, w.E, w.k, w.L, 2, 0, True, shared_slots=True)
    pools = [H.HostPool(w, l) for l in range(w.L)]
    cache = torch.full((2, w.blob_elems), 0x7FC0, dtype=torch.int16, device="cuda")
    lays = [H.DeviceLayer(ctx, w, l, pools[l], None, slots=cache) for l in range(w.L)]
    buf = H.Buffers(ctx, w.T)
    for l in range(w.L):
        x_np = S.activations(w, l, 0)
        ctx.expert_cache_prefetch(l, [0, 1], gpu["copy"])
        ctx.moe_prefill_layer(l, H.np_to_dev(x_np), w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"])
        gpu["compute"].synchronize()
        ref = oracle.moe_layer(x_np, lays[l].router_np, [pools[l].ptr(e) for e in range(w.E)], w.k, I=w.I)
        check_out(H.dev_to_np_u16(buf.y), ref["out_f64"], f"shared cache prefill layer {l}")
        active = int((ref["counts"] > 0).sum())
        extra = sum(1 for e in (0, 1) if ref["counts"][e] == 0)   # speculative fetches without tokens
        assert ctx.moe_get_stats(l)["bytes_h2d"] == (active + extra) * w.blob_bytes
    ctx.close()


# ---------------------------------------------------------------- 8-bit experts on the host link
@pytest.mark.parametrize("fmt", [1, 3])
def test_q8_cache_holds_the_8bit_blobs_and_prefill_reads_them(gpu, oracle, fmt):
    """Experts stored as e4m3 codes with per-row scales, or as MXFP4: the GPU expert cache is those blobs and
    nothing else (half / about a quarter of the bytes of bf16 slots), every fetched expert's slot holds
    exactly the bytes of the CPU expert cache, and the prefill GEMMs, which expand the codes on their way
    into LDS, give the oracle's output on the oracle's expansion.  The rest of the cache is a NaN pattern
    throughout."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("q8_slots", d=256, I=192, E=6, k=2, T=300, I_shared=64, seed=51)
    x = S.activations(w)
    r = run_layer(gpu, w, w.T, x, w.E, None, poison=True, fmt=fmt)
    ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"], shared=r["lay"].shared_np)
    np.testing.assert_array_equal(r["routing"]["perm"], ref["perm"])
    check_out(r["out"], ref["out_f64"], "q8 prefill")
    nbytes = S.q8_blob_bytes(w.d, w.I) if fmt == 1 else S.mx4_blob_bytes(w.d, w.I)
    assert r["lay"].cache.numel() * 2 == w.E * ((nbytes + 255) // 256 * 256) < w.E * w.blob_bytes * (0.51 if fmt == 1 else 0.27)
    slots = r["lay"].slots.cpu().numpy().view(np.uint8)
    active = [e for e in range(w.E) if ref["counts"][e] > 0]
    assert len(active) >= 4
    for e in active:
        s = r["state"].index(e)
        np.testing.assert_array_equal(slots[s][:nbytes], r["pool"].blob_np(e), err_msg=f"expert {e}")
    for s, e in enumerate(r["state"]):
        if e < 0:
            assert np.all(slots[s].view(np.uint16) == 0x7FC0)      # never written
    assert r["stats"]["bytes_h2d"] == len(active) * nbytes
    assert r["stats"]["misses"] == len(active)


@pytest.mark.parametrize("d,I,E,k,T,Ish,variant", [(256, 128, 8, 2, 1200, 0, 0), (512, 192, 5, 3, 700, 128, 0),
                                                   (256, 320, 16, 4, 2500, 0, 0), (256, 128, 8, 2, 1200, 0, 1),
                                                   (1024, 64, 64, 6, 900, 64, 0), (128, 4096, 3, 1, 150, 0, 0),
                                                   (256, 256, 16, 4, 2500, 128, 0), (256, 128, 8, 2, 6200, 0, 0),
                                                   (384, 640, 6, 2, 1500, 0, 0)])
@pytest.mark.parametrize("fmt", [1, 3])
def test_q8_prefill_gemm_on_codes(gpu, oracle, fmt, d, I, E, k, T, Ish, variant):
    """The GEMM kernels that read e4m3 or MXFP4 experts: 256 x 256 and 128 x 128 tiles (by the groups' height, or
    forced), for MXFP4 also the persistent kernel (K a multiple of 128: fixed order, and work plans with
    queues for 16 experts or 1550 rows per expert), several K slices of the down projection, ragged groups,
    resident experts placed by the caller (initial_resident names quantised blobs) and experts streaming
    through three slots: the same bits either way, and the oracle's output on its own expansion of the
    codes."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("q8_gemm", d=d, I=I, E=E, k=k, T=T, I_shared=Ish, seed=77, zipf_s=0.9)
    x = S.activations(w)
    bias = S.zipf_route_bias(w, 0)
    pool = H.HostPool(w, 0, fmt=fmt)
    if variant:
        set_tune(0, 1)
        set_tune(1, 1)
    res = run_layer(gpu, w, T, x, E, list(range(E)), bias=bias, pool=pool, fmt=fmt)
    ref = oracle_layer(oracle, w, x, res["lay"].router_np, pool, bias=bias, shared=res["lay"].shared_np)
    np.testing.assert_array_equal(res["routing"]["perm"], ref["perm"])
    check_out(res["out"], ref["out_f64"], "resident quantised experts")
    assert res["stats"]["misses"] == 0 and res["stats"]["bytes_h2d"] == 0
    streamed = run_layer(gpu, w, T, x, 3, None, bias=bias, pool=pool, fmt=fmt, prefetch=[1, 0], poison=True)
    np.testing.assert_array_equal(streamed["out"], res["out"])


def test_q4_fetch_expands_into_slots_bit_exact(gpu, oracle):
    """4-bit experts (groups of 128, scale and zero point): slots hold the oracle's expansion bit for
    bit, the output is the oracle's on those weights, the link carried the 4-bit blobs; prefill through
    all slots, then streaming through two with a wrong prefetch (prefill and decode)."""
    from oracle.cache_sim import CacheSim
    w = S.Workload("q4_slots", d=256, I=384, E=6, k=2, T=300, I_shared=64, seed=57)
    x = S.activations(w)
    r = run_layer(gpu, w, w.T, x, w.E, None, poison=True, fmt=2)
    ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"], shared=r["lay"].shared_np)
    np.testing.assert_array_equal(r["routing"]["perm"], ref["perm"])
    check_out(r["out"], ref["out_f64"], "q4 prefill")
    slots = r["lay"].slots.cpu().numpy().view(np.uint16)
    active = [e for e in range(w.E) if ref["counts"][e] > 0]
    assert len(active) >= 4
    for e in active:
        np.testing.assert_array_equal(slots[r["state"].index(e)], oracle.dequant4_blob(r["pool"].blob_np(e), w.d, w.I),
                                      err_msg=f"expert {e}")
    assert r["stats"]["bytes_h2d"] == len(active) * S.q4_blob_bytes(w.d, w.I)
    for T, decode in ((300, False), (3, True)):
        r2 = run_layer(gpu, w, T, x[:T], 2, None, decode=decode, prefetch=[5, 4], poison=True, fmt=2, pool=r["pool"])
        ref2 = oracle_layer(oracle, w, x[:T], r2["lay"].router_np, r2["pool"], shared=r2["lay"].shared_np)
        check_out(r2["out"], ref2["out_f64"], f"q4 streaming T={T}")
        sim = CacheSim(w.E, 2, S.q4_blob_bytes(w.d, w.I))
        sim.prefetch([5, 4])
        sim.serve(np.nonzero(ref2["counts"])[0])
        assert r2["stats"] == {**sim.counters(), "layer_calls": 1}


@pytest.mark.parametrize("fmt", [1, 3])
@pytest.mark.parametrize("T,decode", [(700, False), (3, True)])
def test_q8_streaming_through_two_slots(gpu, oracle, T, decode, fmt):
    """Two slots of quantised blobs (e4m3 rows, MXFP4) are reused expert after expert, the last fetch split in
    two pieces; prefill streams all active experts, decode is served after a wrong prefetch."""
    from oracle.cache_sim import CacheSim
    w = S.Workload("q8_stream", d=256, I=192, E=8, k=2, T=T, seed=52, zipf_s=0.8)
    x = S.activations(w)
    bias = S.zipf_route_bias(w, 0)
    r = run_layer(gpu, w, T, x, 2, None, decode=decode, bias=bias, prefetch=[7, 6], poison=True, fmt=fmt)
    ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"], bias=bias)
    np.testing.assert_array_equal(r["routing"]["ids"], ref["ids"])
    check_out(r["out"], ref["out_f64"], f"q8 streaming T={T}")
    sim = CacheSim(w.E, 2, S.q8_blob_bytes(w.d, w.I) if fmt == 1 else S.mx4_blob_bytes(w.d, w.I))
    sim.prefetch([7, 6])
    sim.serve(np.nonzero(ref["counts"])[0])
    assert r["stats"] == {**sim.counters(), "layer_calls": 1}
    assert r["state"] == sim.slot_expert


@pytest.mark.parametrize("d,I,I_shared,T", [(256, 192, 64, 1), (256, 192, 64, 2), (256, 192, 0, 5), (256, 192, 64, 8),
                                            (256, 192, 64, 11), (2048, 128, 0, 1), (2048, 128, 32, 3), (4096, 64, 0, 8)])
@pytest.mark.parametrize("fmt", [1, 3])
def test_q8_decode_streams_the_8bit_blobs(gpu, oracle, fmt, d, I, I_shared, T):
    """Decode on experts held in quantised form (there is no other form in the cache): the mat-vec kernels
    read the codes and scales and expand them in registers to the bf16 weights the format defines (e4m3:
    hardware conversion, one fp32 multiply, nearest-even bf16; MXFP4: the hardware's scaled conversion of
    the two codes of a byte, exact, which also pins nibble and byte order), so the output is the oracle's
    on its own expansion.  Shared experts (bf16) ride in the same launches.  Then the same call through
    two slots with a wrong prefetch: misses fetched and read in the same call."""
    from oracle.cache_sim import CacheSim
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("q8_decode", d=d, I=I, E=6, k=2, T=T, I_shared=I_shared, seed=54 + T)
    x = S.activations(w)
    ctx = new_ctx(B, w.d, w.I, w.E, w.k, 1, w.E, w.I_shared, True, host_format=fmt)
    pool = H.HostPool(w, 0, fmt=fmt)
    lay = H.DeviceLayer(ctx, w, 0, pool, None, poison=True)
    buf = H.Buffers(ctx, T)
    ctx.expert_cache_prefetch(0, list(range(w.E)), gpu["copy"])
    ctx.moe_decode_layer(0, H.np_to_dev(x), T, buf.y, buf.ws, gpu["compute"], gpu["copy"])
    gpu["compute"].synchronize()
    ref = oracle_layer(oracle, w, x, lay.router_np, pool, shared=lay.shared_np)
    np.testing.assert_array_equal(buf.routing(ctx, gpu["compute"])["ids"], ref["ids"])
    check_out(H.dev_to_np_u16(buf.y), ref["out_f64"], f"format {fmt} decode T={T}")
    st = ctx.moe_get_stats(0)
    assert st["misses"] == 0 and st["prefetch_issued"] == w.E
    ctx.close()
    r2 = run_layer(gpu, w, T, x, 2, None, decode=True, prefetch=[5, 4], poison=True, fmt=fmt, pool=pool)
    check_out(r2["out"], ref["out_f64"], f"format {fmt} decode through two slots T={T}")
    sim = CacheSim(w.E, 2, pool.bytes_per_expert)
    sim.prefetch([5, 4])
    sim.serve(np.nonzero(ref["counts"])[0])
    assert r2["stats"] == {**sim.counters(), "layer_calls": 1}


@pytest.mark.parametrize("fmt", [0, 1, 3])
@pytest.mark.parametrize("d,I,I_shared,T", [(512, 256, 256, 1), (256, 512, 0, 2), (256, 512, 0, 6), (512, 256, 256, 9),
                                            (256, 768, 64, 20), (2304, 256, 0, 40)])
def test_decode_batches_through_the_matrix_core_matvec(gpu, oracle, fmt, d, I, I_shared, T):
    """Decode groups of three tokens and more take the mat-vec kernel that forms the sums with 16x16x32
    MFMAs (16 weight rows by up to 16 tokens per instruction): bf16 slots, e4m3 and MXFP4 blobs (the
    only form of those experts in the cache, fetched into a cache of NaN patterns), shared experts in the same launch, K cut into several LDS segments (d = 2304 at 16 tokens per
    pass), groups of more than 16 tokens in several passes (the mat-vec limit is raised so that the
    GEMM kernels do not take them), and the same layer through the per-token kernels for comparison.  One
    token (the launch takes its experts from the gate's id list on the device) and two are forced
    onto the kernel as well."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("skinny", d=d, I=I, E=5, k=2, T=T, I_shared=I_shared, seed=70 + T + fmt, zipf_s=0.8)
    x = S.activations(w)
    bias = S.zipf_route_bias(w, 0)
    ctx = new_ctx(B, w.d, w.I, w.E, w.k, 1, w.E, w.I_shared, True, host_format=fmt)
    pool = H.HostPool(w, 0, fmt=fmt)
    lay = H.DeviceLayer(ctx, w, 0, pool, None if fmt else list(range(w.E)), poison=bool(fmt))
    buf = H.Buffers(ctx, T)
    if fmt:
        ctx.expert_cache_prefetch(0, list(range(w.E)), gpu["copy"])
        torch.cuda.synchronize()
    ref = oracle_layer(oracle, w, x, lay.router_np, pool, bias=bias, shared=lay.shared_np)
    assert T < 6 or (ref["counts"].max() >= 3 and (T < 20 or ref["counts"].max() > 16))
    outs = {}
    for name, min_tok in (("mfma", 1), ("per-token", 1 << 20)):    # 1: wherever the shapes allow it
        ctx.moe_tune(8, min_tok)
        ctx.moe_tune(9, 64)
        ctx.moe_decode_layer(0, H.np_to_dev(x), T, buf.y, buf.ws, gpu["compute"], gpu["copy"], H.np_to_dev(bias), 0)
        gpu["compute"].synchronize()
        np.testing.assert_array_equal(buf.routing(ctx, gpu["compute"])["perm"], ref["perm"])
        outs[name] = H.dev_to_np_u16(buf.y)
        check_out(outs[name], ref["out_f64"], f"{name} fmt={fmt} T={T}")
    ctx.close()


def test_prefill_seeded_random_shapes(gpu, oracle):
    """Thirty seeded random prefill layers: host format, widths (multiples of the format's unit, not of
    the tiles), shared experts, 3 to 64 experts, top-1 to top-8, up to 1500 tokens, Zipf or even
    routing, every expert resident or streamed through fewer slots than experts with a partly wrong
    prefetch.  Routing tables bit for bit, outputs within the bf16 tolerance of the oracle, cache
    counters equal to the simulator's."""
    from oracle.cache_sim import CacheSim
    rng = np.random.default_rng(5151)
    for it in range(30):
        fmt = int(rng.choice([0, 0, 1, 2, 3]))
        unit = {0: 8, 1: 64, 2: 128, 3: 64}[fmt]
        d = int(rng.integers(1, 5)) * unit * int(rng.choice([1, 3, 8]))
        I = int(rng.integers(1, 5)) * unit * int(rng.choice([1, 2]))
        I_shared = int(rng.choice([0, 0, 64, 136]))
        E = int(rng.choice([3, 6, 8, 17, 64]))
        k = int(rng.integers(1, min(E, 8) + 1))
        T = int(rng.choice([1, 5, 63, 64, 200, 777, 1500]))
        slots = E if rng.random() < 0.5 else int(rng.integers(1, E))   # one slot: fetch and compute take turns
        prefetch = [int(e) for e in rng.permutation(E)[:min(slots, 2)]]
        case = f"case {it}: fmt={fmt} d={d} I={I} I_shared={I_shared} E={E} k={k} T={T} slots={slots} prefetch={prefetch}"
        w = S.Workload("random", d=d, I=I, E=E, k=k, T=T, I_shared=I_shared, seed=2000 + it,
                       zipf_s=float(rng.choice([0.0, 1.1])))
        x = S.activations(w)
        bias = S.zipf_route_bias(w, 0)
        r = run_layer(gpu, w, T, x, slots, None, bias=bias, prefetch=prefetch, poison=True, fmt=fmt)
        ref = oracle_layer(oracle, w, x, r["lay"].router_np, r["pool"], bias=bias, shared=r["lay"].shared_np)
        for key in ("ids", "counts", "perm"):
            np.testing.assert_array_equal(r["routing"][key], ref[key], err_msg=f"{case} {key}")
        check_out(r["out"], ref["out_f64"], case)
        sim = CacheSim(E, slots, r["pool"].bytes_per_expert)
        sim.prefetch(prefetch)
        sim.serve(np.nonzero(ref["counts"])[0])
        assert r["stats"] == {**sim.counters(), "layer_calls": 1}, case


def test_decode_seeded_random_shapes(gpu, oracle):
    """Forty seeded random decode layers (format, widths that are whole steps of the matrix-core kernel
    or not, shared experts of several widths, 3 to 64 experts, top-1 to top-8, 1 to 63 tokens, Zipf or
    even routing, the matrix-core mat-vec by rule or forced, 1 to 8 K slices per block): routing tables
    bit for bit, outputs within the bf16 tolerance of the oracle on the same (expanded) weights."""
    H, B = gpu["harness"], gpu["binding"]
    rng = np.random.default_rng(4242)
    for it in range(40):
        fmt = int(rng.choice([0, 1, 3]))
        kmul = {0: 64, 1: 128, 3: 256}[fmt]
        d = int(rng.integers(1, 6)) * kmul * int(rng.choice([1, 2]))
        I = int(rng.integers(1, 5)) * kmul
        I_shared = int(rng.choice([0, 40, 64, 192, 320]))
        E = int(rng.choice([3, 5, 8, 17, 60, 64]))
        k = int(rng.integers(1, min(E, 8) + 1))
        T = int(rng.choice([1, 2, 3, 4, 7, 9, 16, 21, 40, 63]))
        forced, slices = int(rng.choice([0, 1])), int(rng.choice([0, 1, 3, 8]))
        case = f"case {it}: fmt={fmt} d={d} I={I} I_shared={I_shared} E={E} k={k} T={T} forced={forced} slices={slices}"
        w = S.Workload("random", d=d, I=I, E=E, k=k, T=T, I_shared=I_shared, seed=1000 + it,
                       zipf_s=float(rng.choice([0.0, 1.0])))
        x = S.activations(w)
        bias = S.zipf_route_bias(w, 0)
        ctx = new_ctx(B, w.d, w.I, w.E, w.k, 1, w.E, w.I_shared, True, host_format=fmt)
        pool = H.HostPool(w, 0, fmt=fmt)
        lay = H.DeviceLayer(ctx, w, 0, pool, None if fmt else list(range(E)), poison=bool(fmt))
        buf = H.Buffers(ctx, T)
        if fmt:
            ctx.expert_cache_prefetch(0, list(range(E)), gpu["copy"])
            torch.cuda.synchronize()
        ctx.moe_tune(8, 1 if forced else 0)
        ctx.moe_tune(9, 64)
        ctx.moe_tune(10, slices)
        ctx.moe_decode_layer(0, H.np_to_dev(x), T, buf.y, buf.ws, gpu["compute"], gpu["copy"], H.np_to_dev(bias), 0)
        gpu["compute"].synchronize()
        ref = oracle_layer(oracle, w, x, lay.router_np, pool, bias=bias, shared=lay.shared_np)
        np.testing.assert_array_equal(buf.routing(ctx, gpu["compute"])["perm"], ref["perm"], err_msg=case)
        check_out(H.dev_to_np_u16(buf.y), ref["out_f64"], case)
        ctx.close()


@pytest.mark.parametrize("fmt", [1, 3])
def test_quantised_decode_then_prefill_without_a_pause(gpu, oracle, fmt):
    """A decode call and a prefill call enqueued right behind it, on quantised experts whose copies are
    still in flight when the first is made: each waits for the bytes it reads to land (mat-vec kernels,
    then the GEMMs that expand code tiles).  Both against the oracle."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("q_then_prefill", d=512, I=256, E=6, k=2, T=96, seed=59)
    ctx = new_ctx(B, w.d, w.I, w.E, w.k, 1, w.E, 0, True, host_format=fmt)
    pool = H.HostPool(w, 0, fmt=fmt)
    lay = H.DeviceLayer(ctx, w, 0, pool, None, poison=True)
    xd_np, xp_np = S.activations(w, 0, 1)[:2], S.activations(w, 0, 2)
    xd, xp = H.np_to_dev(xd_np), H.np_to_dev(xp_np)
    bd, bp = H.Buffers(ctx, 2), H.Buffers(ctx, w.T)
    ctx.expert_cache_prefetch(0, list(range(w.E)), gpu["copy"])           # copies still in flight
    ctx.moe_decode_layer(0, xd, 2, bd.y, bd.ws, gpu["compute"], gpu["copy"])
    ctx.moe_prefill_layer(0, xp, w.T, bp.y, bp.ws, gpu["compute"], gpu["copy"])
    gpu["compute"].synchronize()
    for x_np, buf, tag in ((xd_np, bd, "decode"), (xp_np, bp, "prefill")):
        ref = oracle_layer(oracle, w, x_np, lay.router_np, pool)
        check_out(H.dev_to_np_u16(buf.y), ref["out_f64"], f"format {fmt}: {tag}")
    assert ctx.moe_get_stats(0)["misses"] == 0
    ctx.close()


def test_q8_and_bf16_pools_of_the_same_weights_agree_within_the_format_error(gpu, oracle):
    """The 8-bit path is the bf16 path run on rounded weights: on the same seeded experts the two
    outputs differ by what 3 mantissa bits cost (a few per cent of the output's rms), not more."""
    w = S.Workload("q8_vs_bf16", d=512, I=256, E=8, k=2, T=64, seed=53)
    x = S.activations(w)
    a = run_layer(gpu, w, w.T, x, w.E, None, q8=True)
    b = run_layer(gpu, w, w.T, x, w.E, None)
    np.testing.assert_array_equal(a["routing"]["ids"], b["routing"]["ids"])
    ya, yb = S.bf16_to_f32(a["out"]).astype(np.float64), S.bf16_to_f32(b["out"]).astype(np.float64)
    rms = np.sqrt(np.mean(yb ** 2))
    rel = np.sqrt(np.mean((ya - yb) ** 2)) / rms
    assert 1e-3 < rel < 0.1, rel


# ---------------------------------------------------------------- ExpertMLP predictor (Section IV-B)
def mlp_on_device(H, dims, params):
    ws, bs, sc, sh = params
    dev = lambda arrs: [H.np_to_dev(a) for a in arrs]
    act = torch.empty(2 * max(dims), dtype=torch.float32, device="cuda")
    return dev(ws), dev(bs), dev(sc), dev(sh), act


@pytest.mark.parametrize("L,E,k,m", [(32, 8, 2, 2), (24, 60, 4, 8), (3, 64, 6, 64)])
def test_mlp_predictor_scores_bit_exact(gpu, oracle, L, E, k, m):
    """Seven hidden layers 2048 .. 64 and E logits: the fp32 sums follow the documented order, so the
    logits equal the oracle's replay bit for bit and the top-m is the same list."""
    H, B = gpu["harness"], gpu["binding"]
    dims = S.mlp_dims(L, E, k)
    params = S.mlp_params(dims, 41 + E)
    ws, bs, sc, sh, act = mlp_on_device(H, dims, params)
    ctx = new_ctx(B, 256, 128, E, k, 1, E)
    scores = torch.empty(E, dtype=torch.float32, device="cuda")
    top = torch.zeros(m, dtype=torch.int32).pin_memory()
    pred = torch.cuda.Stream()
    for trial in range(3):
        state_np = np.abs(S.normal_f32((dims[0],), 7, 500 + trial, 0.3))
        state = torch.from_numpy(state_np).pin_memory()          # the state vector is built on the host
        ctx.predictor_mlp_score(state, dims, ws, bs, sc, sh, act, m, top, pred, scores)
        pred.synchronize()
        l32, l64 = oracle.mlp_forward(state_np, *params)
        np.testing.assert_array_equal(scores.cpu().numpy(), l32)
        np.testing.assert_array_equal(top.numpy(), oracle.top_m(l32, m))
        assert np.abs(l32 - l64).max() <= 1e-4 * max(1.0, np.abs(l64).max())
    ctx.close()


def test_paper_decode_flow_state_constructor_mlp_and_one_cache(gpu, oracle):
    """Section V-C end to end on a small model: the first layer of a step is served on demand; every
    layer's selection goes to the State Constructor; its vector for the next layer feeds ExpertMLP on a
    third stream; the predicted experts are prefetched into the one cache of k slots; wrong guesses are
    fetched again; the state is cleared after the round.  Checked against oracle and simulator."""
    from oracle import predictor as P
    from oracle.cache_sim import SharedCacheSim
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("paper_flow", d=256, I=128, E=8, k=2, T=1, seed=29, L=4, steps=4, p_stay=0.6)
    history_trace = S.markov_trace(replace(w, seed=30, steps=500))     # the "preprocessing" traces
    history_trace = history_trace[:, :, 0, :] if history_trace.ndim == 4 else history_trace
    pop = P.popularity(history_trace, w.E).astype(np.float32)
    aff = P.affinity(history_trace, w.E).astype(np.float32)
    st = B.MoeState(w.L, w.E, w.k, pop, aff)
    dims = S.mlp_dims(w.L, w.E, w.k)
    params = [S.mlp_params(dims, 77, l) for l in range(w.L)]           # one predictor per target layer
    dev_params = [mlp_on_device(H, dims, p) for p in params]
    ctx = new_ctx(B, w.d, w.I, w.E, w.k, w.L, w.k, 0, True, shared_slots=True)
    pools = [H.HostPool(w, l) for l in range(w.L)]
    cache = torch.full((w.k, w.blob_elems), 0x7FC0, dtype=torch.int16, device="cuda")
    lays = [H.DeviceLayer(ctx, w, l, pools[l], None, slots=cache) for l in range(w.L)]
    sim = SharedCacheSim(w.L, w.E, w.k, w.blob_bytes)
    trace = S.markov_trace(w)
    buf = H.Buffers(ctx, w.T)
    pred = torch.cuda.Stream()
    top = torch.zeros(w.k, dtype=torch.int32).pin_memory()
    state = torch.zeros(st.moe_state_dim(), dtype=torch.float32).pin_memory()
    for s in range(w.steps):
        history = []
        for l in range(w.L):
            x_np = S.activations(w, l, s)
            bias_np = S.trace_route_bias(trace[s, l], w.E)
            ctx.moe_decode_layer(l, H.np_to_dev(x_np), w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"],
                                 H.np_to_dev(bias_np), w.E)
            gpu["compute"].synchronize()
            ref = oracle.moe_layer(x_np, lays[l].router_np, [pools[l].ptr(e) for e in range(w.E)], w.k,
                                   bias=bias_np, I=w.I)
            ids = buf.routing(ctx, gpu["compute"])["ids"][0]
            np.testing.assert_array_equal(ids, ref["ids"][0])
            check_out(H.dev_to_np_u16(buf.y), ref["out_f64"], f"paper flow step {s} layer {l}")
            sim.serve(l, ref["ids"][0])
            assert ctx.moe_cache_state(l) == sim.state(l)
            st.moe_state_record(l, ids)
            history.append([int(i) for i in ref["ids"][0]])
            if l + 1 == w.L:
                continue
            st.moe_state_vector(l + 1, state)
            want_state = P.state_vector(history, l + 1, pop.astype(np.float64), aff.astype(np.float64), w.k)
            np.testing.assert_array_equal(state.numpy(), want_state)
            dws, dbs, dsc, dsh, act = dev_params[l + 1]
            ctx.predictor_mlp_score(state, dims, dws, dbs, dsc, dsh, act, w.k, top, pred)
            pred.synchronize()
            l32, _ = oracle.mlp_forward(want_state, *params[l + 1])
            np.testing.assert_array_equal(top.numpy(), oracle.top_m(l32, w.k))
            ctx.expert_cache_prefetch(l + 1, top.tolist(), gpu["copy"])
            sim.prefetch(l + 1, oracle.top_m(l32, w.k))
        st.moe_state_clear()
    torch.cuda.synchronize()
    for l in range(w.L):
        assert ctx.moe_get_stats(l) == {**sim.counters(l), "layer_calls": w.steps}
    assert ctx.moe_get_stats(0)["hits"] == 0          # no prediction for the first layer: always on demand
    st.close()
    ctx.close()


# ---------------------------------------------------------------- predictor stand-in
@pytest.mark.parametrize("B,d,E,m", [(1, 4096, 8, 3), (8, 2048, 60, 8), (3, 256, 64, 64)])
def test_predictor_scores_and_topm(gpu, oracle, B, d, E, m):
    Bn, H = gpu["binding"], gpu["harness"]
    x = S.normal_bf16((B, d), 3, 1, 1.0)
    wp = S.normal_bf16((E, d), 3, 2, 0.02)
    ctx = Bn.MoeContext(d, 64, E, 1, 1, 1)
    top = torch.zeros(m, dtype=torch.int32).pin_memory()
    scores = torch.empty(E, dtype=torch.float32, device="cuda")
    ctx.predictor_score(0, H.np_to_dev(x), B, H.np_to_dev(wp), m, top, gpu["compute"], scores)
    gpu["compute"].synchronize()
    ref_s, ref_top = oracle.predictor_score(x, wp, m)
    np.testing.assert_array_equal(scores.cpu().numpy(), ref_s)  # same fp32 summation order
    np.testing.assert_array_equal(top.numpy(), ref_top)
    ctx.close()


# ---------------------------------------------------------------- error paths (host checks only)
def test_error_codes(gpu):
    B = gpu["binding"]
    with pytest.raises(B.MoeError) as e:
        new_ctx(B, 256, 128, 8, 9)
    assert e.value.code == -1
    with pytest.raises(B.MoeError) as e:
        new_ctx(B, 256, 128, 8, 2, 1, 0)
    assert e.value.code == -1
    with pytest.raises(B.MoeError) as e:
        new_ctx(B, 256, 128, 65, 2)
    assert e.value.code == -2
    with pytest.raises(B.MoeError) as e:
        new_ctx(B, 250, 128, 8, 2)
    assert e.value.code == -2
    ctx = new_ctx(B, 256, 128, 8, 2)
    x = torch.zeros((4, 256), dtype=torch.int16, device="cuda")
    y = torch.zeros_like(x)
    ws = torch.empty(ctx.moe_workspace_bytes(4), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.MoeError) as e:
        ctx.moe_prefill_layer(0, x, 4, y, ws, gpu["compute"], gpu["copy"])
    assert e.value.code == -4
    with pytest.raises(B.MoeError) as e:
        ctx.moe_prefill_layer(3, x, 4, y, ws, gpu["compute"], gpu["copy"])
    assert e.value.code == -1
    w = S.Workload("err", d=256, I=128, E=8, k=2, T=4)
    H = gpu["harness"]
    pool = H.HostPool(w, 0)
    H.DeviceLayer(ctx, w, 0, pool, list(range(8)))
    with pytest.raises(B.MoeError) as e:
        ctx.moe_prefill_layer(0, x, 0, y, ws, gpu["compute"], gpu["copy"])
    assert e.value.code == -1
    with pytest.raises(B.MoeError) as e:
        ctx.moe_prefill_layer(0, x, 4, y, ws[:1024], gpu["compute"], gpu["copy"])
    assert e.value.code == -5
    with pytest.raises(B.MoeError) as e:
        ctx.expert_cache_prefetch(0, [8], gpu["copy"])
    assert e.value.code == -1
    ctx.close()
