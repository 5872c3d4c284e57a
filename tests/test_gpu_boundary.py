"""Boundary behaviour of the C ABI on the GPU: the full-softmax gate, large caches, calls that only
enqueue, per-call counters and the state a call leaves behind when a HIP call fails midway.
Needs an MI355X."""
import time

import numpy as np
import pytest

from paper_2509_07379_amd import synth as S

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

from test_gpu_parity import check_out, gpu  # noqa: E402,F401  (fixture + tolerance)


# ---------------------------------------------------------------- gate values over all experts
@pytest.mark.parametrize("E,k", [(8, 3), (8, 8), (60, 4), (5, 5)])
@pytest.mark.parametrize("T,decode", [(150, False), (5, True), (1, True)])
def test_gate_values_as_softmax_over_all_experts(gpu, oracle, E, k, T, decode):
    """renormalize = 0 (Section II-A: the gate's values are a softmax over the whole pool; the Top-k
    keeps k of them, so they no longer sum to one unless k = E).  ids bit for bit, values against the
    oracle's fp64 softmax, the layer output within the stated tolerance."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("full_softmax", d=512, I=256, E=E, k=k, T=T, I_shared=128, seed=5)
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E, w.I_shared, renormalize=False)
    pool = H.HostPool(w, 0)
    lay = H.DeviceLayer(ctx, w, 0, pool, list(range(E)))
    buf = H.Buffers(ctx, T)
    x_np = S.activations(w)
    # spread logits so that the values differ visibly from the renormalised ones
    bias_np = (np.arange(E, dtype=np.float32) % 7) * 0.37
    fn = ctx.moe_decode_layer if decode else ctx.moe_prefill_layer
    fn(0, H.np_to_dev(x_np), T, buf.y, buf.ws, gpu["compute"], gpu["copy"], H.np_to_dev(bias_np), 0)
    gpu["compute"].synchronize()
    ref = oracle.moe_layer(x_np, lay.router_np, [pool.blob_np(e) for e in range(E)], k, bias=bias_np,
                           renormalize=False, shared_blob=lay.shared_np, I=w.I, I_shared=w.I_shared)
    got = buf.routing(ctx, gpu["compute"])
    for key in ("ids", "counts", "offsets", "perm", "inv_perm"):
        np.testing.assert_array_equal(got[key], ref[key], err_msg=key)
    np.testing.assert_allclose(got["w"], ref["w"], rtol=2e-5, atol=1e-8)
    sums = got["w"].sum(1)
    if k == E:
        np.testing.assert_allclose(sums, 1.0, rtol=1e-5)
    else:
        assert np.all(sums < 1.0 - 1e-3)     # really the values of the whole pool's softmax
    check_out(H.dev_to_np_u16(buf.y), ref["out_f64"], f"full softmax E={E} k={k} T={T}")
    ctx.close()


# ---------------------------------------------------------------- slot indices beyond one byte
def test_one_cache_of_200_slots_for_all_layers(gpu, oracle):
    """One GPU expert cache of 200 slots shared by 28 layers: slots fill in index order, so from layer
    16 on the experts sit in slots 128 and above, which the kernels must address as they are."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("wide_cache", d=128, I=64, E=8, k=2, T=64, seed=29, L=28)
    slots = 200
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, w.L, slots, 0, True, shared_slots=True)
    cache = torch.full((slots, w.blob_elems), 0x7FC0, dtype=torch.int16, device="cuda")
    pools, lays = [], []
    for l in range(w.L):
        pools.append(H.HostPool(w, l))
        lays.append(H.DeviceLayer(ctx, w, l, pools[l], None, slots=cache))
    buf = H.Buffers(ctx, w.T)
    seen_high = False
    for l in range(w.L):
        x_np = S.activations(w, l, 0)
        for decode, T in ((False, w.T), (True, 3)):
            fn = ctx.moe_decode_layer if decode else ctx.moe_prefill_layer
            b = buf if T == w.T else H.Buffers(ctx, T)
            fn(l, H.np_to_dev(x_np[:T]), T, b.y, b.ws, gpu["compute"], gpu["copy"])
            gpu["compute"].synchronize()
            if l >= 15:
                ref = oracle.moe_layer(x_np[:T], lays[l].router_np, [pools[l].blob_np(e) for e in range(w.E)],
                                       w.k, I=w.I)
                np.testing.assert_array_equal(b.routing(ctx, gpu["compute"])["ids"], ref["ids"])
                check_out(H.dev_to_np_u16(b.y), ref["out_f64"], f"layer {l} decode={decode}")
        state = ctx.moe_cache_state(l)
        held = [s for s, e in enumerate(state) if e >= 0]
        assert len(held) == w.E
        if (l + 1) * w.E <= slots:      # empty slots are taken in index order; after that the least recently used
            assert held == list(range(l * w.E, (l + 1) * w.E))
        seen_high |= l >= 15 and max(held) >= 128
    assert seen_high
    ctx.close()


# ---------------------------------------------------------------- calls that only enqueue
def test_resident_calls_return_before_the_first_one_has_run(gpu, oracle):
    """With every expert resident a layer call only enqueues: eight prefill calls come back while the
    stream is still busy, and their cache counters are there once they are asked for."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("enqueue_only", d=2048, I=4096, E=8, k=2, T=4096, seed=3)
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E)
    pool = H.HostPool(w, 0)
    lay = H.DeviceLayer(ctx, w, 0, pool, list(range(w.E)))
    buf = H.Buffers(ctx, w.T)
    x = H.np_to_dev(S.activations(w))
    for _ in range(3):
        ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"])
    torch.cuda.synchronize()
    ctx.moe_reset_stats()
    calls = 8
    done = torch.cuda.Event()
    t0 = time.perf_counter()
    for _ in range(calls):
        ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"])
    t_host = time.perf_counter() - t0
    done.record(gpu["compute"])
    busy_after_loop = not done.query()
    done.synchronize()
    t_all = time.perf_counter() - t0
    assert busy_after_loop, f"host needed {t_host * 1e3:.2f} ms for {calls} calls that run {t_all * 1e3:.2f} ms"
    assert t_host < 0.6 * t_all
    st = ctx.moe_get_stats(0)
    assert st["hits"] == calls * w.E and st["misses"] == 0 and st["layer_calls"] == calls
    ctx.close()


def test_counters_of_enqueued_calls_keep_the_order_of_the_calls(gpu, oracle):
    """Forty one-token decode calls on two fully resident layers of one shared cache (more calls than
    the library has mailboxes), none of which waits for the gate; then a third layer's prefetch needs
    victims.  Recency stamps, hits and victims are those of the simulator, which takes every call in
    order."""
    from oracle.cache_sim import SharedCacheSim
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("lazy_counters", d=256, I=128, E=6, k=2, T=1, seed=41, L=3, steps=20, p_stay=0.5)
    slots = 2 * w.E
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, w.L, slots, 0, True, shared_slots=True)
    cache = torch.full((slots, w.blob_elems), 0x7FC0, dtype=torch.int16, device="cuda")
    pools = [H.HostPool(w, l) for l in range(w.L)]
    lays = [H.DeviceLayer(ctx, w, l, pools[l], None, slots=cache) for l in range(w.L)]
    sim = SharedCacheSim(w.L, w.E, slots, w.blob_bytes)
    for l in range(2):
        ctx.expert_cache_prefetch(l, list(range(w.E)), gpu["copy"])
        sim.prefetch(l, range(w.E))
    trace = S.markov_trace(w)
    buf = H.Buffers(ctx, 1)
    xs, biases, refs = {}, {}, {}
    for s in range(w.steps):
        for l in range(2):
            x_np = S.activations(w, l, s)
            bias_np = S.trace_route_bias(trace[s, l], w.E)
            xs[s, l], biases[s, l] = H.np_to_dev(x_np), H.np_to_dev(bias_np)
            refs[s, l] = oracle.topk_weights(oracle.router_logits(x_np, lays[l].router_np, bias_np), w.k)[0]
    for s in range(w.steps):
        for l in range(2):
            ctx.moe_decode_layer(l, xs[s, l], 1, buf.y, buf.ws, gpu["compute"], gpu["copy"], biases[s, l], w.E)
            sim.serve(l, refs[s, l].ravel())
    # a layer that owns nothing yet: each of its experts evicts the least recently used slot
    ctx.expert_cache_prefetch(2, [0, 1, 2, 3], gpu["copy"])
    sim.prefetch(2, [0, 1, 2, 3])
    torch.cuda.synchronize()
    for l in range(w.L):
        assert ctx.moe_cache_state(l) == sim.state(l), f"layer {l}"
        calls = w.steps if l < 2 else 0
        assert ctx.moe_get_stats(l) == {**sim.counters(l), "layer_calls": calls}, f"layer {l}"
    ctx.close()


def test_counters_of_one_call(gpu, oracle):
    """The optional moe_stats of a layer call holds that call's own counters: they add up to the layer's."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("per_call", d=256, I=128, E=8, k=2, T=40, seed=13)
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, 3)
    pool = H.HostPool(w, 0)
    H.DeviceLayer(ctx, w, 0, pool, None, poison=True)
    buf = H.Buffers(ctx, w.T)
    total = dict(hits=0, misses=0, bytes_h2d=0, layer_calls=0, prefetch_useful=0)
    for step in range(4):
        x = H.np_to_dev(S.activations(w, 0, step))
        if step == 2:
            ctx.expert_cache_prefetch(0, [0, 1], gpu["copy"])
        T = w.T if step % 2 == 0 else 2
        fn = ctx.moe_prefill_layer if step % 2 == 0 else ctx.moe_decode_layer
        one = fn(0, x, T, buf.y, buf.ws, gpu["compute"], gpu["copy"], want_stats=True)
        assert one["layer_calls"] == 1 and one["wait_ms"] >= 0.0 and one["compute_ms"] == 0.0
        assert one["bytes_h2d"] == one["misses"] * w.blob_bytes
        for key in total:
            total[key] += one[key]
    torch.cuda.synchronize()
    st = ctx.moe_get_stats(0, full=True)
    for key in ("hits", "misses", "layer_calls", "prefetch_useful"):
        assert st[key] == total[key], key
    assert st["bytes_h2d"] == total["bytes_h2d"] + st["prefetch_issued"] * w.blob_bytes
    assert st["prefetch_ready"] + st["prefetch_stalled"] == st["prefetch_useful"]
    assert st["wait_ms"] > 0.0
    ctx.close()


# ---------------------------------------------------------------- a HIP call that fails midway
def test_cache_stays_consistent_when_a_hip_call_fails(gpu, oracle):
    """Every HIP call of a layer call that has to fetch (and of a prefetch) is made to fail once, on the
    host, without anything wrong reaching the GPU.  After each failure every slot the tables name still
    holds exactly that expert's bytes, no expert is named twice, and the same call repeated gives the
    bits of an undisturbed run."""
    H, B = gpu["harness"], gpu["binding"]
    lib = B.load()
    w = S.Workload("fail_midway", d=256, I=128, E=8, k=2, T=48, I_shared=64, seed=19)
    x_np = S.activations(w)
    pool = H.HostPool(w, 0)
    blobs = [pool.blob_np(e) for e in range(w.E)]

    def fresh():
        ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, 3, w.I_shared)
        lay = H.DeviceLayer(ctx, w, 0, pool, None, poison=True)
        return ctx, lay, H.Buffers(ctx, w.T)

    ctx, lay, buf = fresh()
    x = H.np_to_dev(x_np)
    ctx.expert_cache_prefetch(0, [5, 6], gpu["copy"])
    ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"])
    torch.cuda.synchronize()
    want = H.dev_to_np_u16(buf.y).copy()
    ref = oracle.moe_layer(x_np, lay.router_np, blobs, w.k, shared_blob=lay.shared_np, I=w.I, I_shared=w.I_shared)
    check_out(want, ref["out_f64"], "undisturbed run")
    ctx.close()

    def check_state(ctx, lay, tag):
        torch.cuda.synchronize()
        state = ctx.moe_cache_state(0)
        named = [e for e in state if e >= 0]
        assert len(named) == len(set(named)), f"{tag}: {state}"
        slots = H.dev_to_np_u16(lay.slots)
        for s, e in enumerate(state):
            if e >= 0:
                assert np.array_equal(slots[s], blobs[e]), f"{tag}: slot {s} does not hold expert {e}"

    failures = 0
    for what in ("prefetch", "layer"):
        n = 0
        while True:
            n += 1
            assert n < 400, "the call never got through"
            ctx, lay, buf = fresh()
            x = H.np_to_dev(x_np)
            failed = False
            try:
                if what == "prefetch":
                    lib.moe_inject_failure(n)
                ctx.expert_cache_prefetch(0, [5, 6], gpu["copy"])
                if what == "layer":
                    lib.moe_inject_failure(n)
                ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"])
            except B.MoeError as err:
                assert err.code == -3 and "injected" in str(err)
                failed = True
            finally:
                lib.moe_inject_failure(0)
            if failed:
                failures += 1
                check_state(ctx, lay, f"{what} call {n}")
                ctx.moe_prefill_layer(0, x, w.T, buf.y, buf.ws, gpu["compute"], gpu["copy"])
                check_state(ctx, lay, f"{what} call {n}, repeated")
                np.testing.assert_array_equal(H.dev_to_np_u16(buf.y), want, err_msg=f"{what} call {n}")
            ctx.close()
            if not failed:
                break
    assert failures > 20
