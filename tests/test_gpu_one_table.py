"""The library and the oracle driven through ONE table of calls: the same seeded program of prefetches,
prefill calls, decode calls and predictions goes to `MoeContext` (C ABI, MI355X) and to `RefMoe`
(oracle/entry_points.py, host arrays), and after every call the two are compared: routing tables bit
for bit, outputs within the stated tolerance, the call's own counters, the cache's slot contents, and at
the end every layer's counters.  Needs an MI355X."""
import numpy as np
import pytest

from paper_2509_07379_amd import synth as S

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

RTOL, ATOL = 2e-2, 1e-2   # the tolerance stated for bf16-in / fp32-accumulate outputs
COUNTERS = ("hits", "misses", "prefetch_issued", "prefetch_useful", "prefetch_dropped", "layer_calls", "bytes_h2d")


def check_out(got_bits, ref_f64, tag):
    got = S.bf16_to_f32(got_bits).astype(np.float64)
    err = np.abs(got - ref_f64)
    assert np.all(np.isfinite(got)), tag
    assert np.all(err <= ATOL + RTOL * np.abs(ref_f64)), f"{tag}: max err {err.max()}"
    rms = float(np.sqrt(np.mean(ref_f64 ** 2)))
    assert np.all(err <= RTOL * np.abs(ref_f64) + RTOL * rms), f"{tag}: max err {err.max()} rms {rms}"


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests selected but no GPU is visible")
    from paper_2509_07379_amd import binding, harness
    binding.load()
    torch.cuda.set_device(0)
    return dict(binding=binding, harness=harness, compute=torch.cuda.Stream(), copy=torch.cuda.Stream(),
                pred=torch.cuda.Stream())


# name, E, k, I_shared, slots, one cache for all layers, host format, calls
CASES = [("slots_per_layer", 16, 2, 0, 5, False, 0, 48),
         ("one_cache", 16, 2, 0, 6, True, 0, 48),
         ("all_resident_many_experts", 60, 4, 128, 60, False, 0, 36),   # calls are only enqueued
         ("eight_bit_experts", 16, 4, 64, 7, False, 1, 36),
         ("mxfp4_experts_one_cache", 16, 2, 64, 4, True, 3, 36)]


@pytest.mark.parametrize("name,E,k,Ish,slots,shared,fmt,n_calls", CASES)
def test_same_program_through_both_tables(gpu, name, E, k, Ish, slots, shared, fmt, n_calls):
    from oracle.entry_points import RefMoe
    H, B = gpu["harness"], gpu["binding"]
    L = 3
    w = S.Workload(name, d=256, I=128, E=E, k=k, T=1, I_shared=Ish, seed=101 + E + k, L=L)
    rng = np.random.default_rng(E * 1000 + k * 10 + fmt)
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, L, slots, w.I_shared, True, shared_slots=shared, host_format=fmt)
    pools = [H.HostPool(w, l, fmt=fmt) for l in range(L)]
    ref = RefMoe(w.d, w.I, w.E, w.k, L, slots, w.I_shared, True, shared_slots=shared, host_format=fmt,
                 blob_bytes=pools[0].bytes_per_expert)
    all_in = slots == E and not shared
    initial = list(range(E)) if all_in else None
    cache = torch.full((ctx.moe_cache_bytes() // 2,), 0x7FC0, dtype=torch.int16, device="cuda") if shared else None
    lays = [H.DeviceLayer(ctx, w, l, pools[l], initial, slots=cache, poison=True) for l in range(L)]
    for l in range(L):
        ref.moe_bind_layer(l, [pools[l].blob_np(e) for e in range(E)], lays[l].router_np, lays[l].shared_np, initial)
    wps_np = [S.predictor_weight(w, l) for l in range(L)]
    wps = [H.np_to_dev(a) for a in wps_np]
    top = torch.zeros(3, dtype=torch.int32).pin_memory()
    bufs = {}
    for call in range(n_calls):
        l = int(rng.integers(L))
        op = rng.choice(["prefetch", "prefill", "decode", "decode", "predict"])
        tag = f"{name} call {call} {op} layer {l}"
        if op == "prefetch":
            ids = rng.choice(E, size=int(rng.integers(1, 5)), replace=True).tolist()   # repeats are allowed
            ctx.expert_cache_prefetch(l, ids, gpu["copy"])
            ref.expert_cache_prefetch(l, ids)
        elif op == "predict":
            T = int(rng.integers(1, 9))
            x_np = S.activations(S.Workload(name, d=w.d, I=w.I, E=E, k=k, T=T, seed=7000 + call), l, call)
            ctx.predictor_score(l, H.np_to_dev(x_np), T, wps[l], 3, top, gpu["pred"])
            gpu["pred"].synchronize()
            _, want = ref.predictor_score(l, x_np, T, wps_np[l], 3)
            np.testing.assert_array_equal(top.numpy(), want, err_msg=tag)
            continue
        else:
            T = int(rng.choice([65, 130, 300, 700]) if op == "prefill" else rng.choice([1, 1, 2, 3, 8, 12, 24, 32]))
            wl = S.Workload(name, d=w.d, I=w.I, E=E, k=k, T=T, seed=9000 + call, zipf_s=1.1)
            x_np = S.activations(wl, l, call)
            bias_np = S.zipf_route_bias(wl, l) if rng.integers(2) else None   # skewed popularity, or the plain gate
            buf = bufs.setdefault(T, H.Buffers(ctx, T))
            want_stats = bool(rng.integers(2))       # every other call asks for its own counters
            fn = ctx.moe_prefill_layer if op == "prefill" else ctx.moe_decode_layer
            got_stats = fn(l, H.np_to_dev(x_np), T, buf.y, buf.ws, gpu["compute"], gpu["copy"],
                           None if bias_np is None else H.np_to_dev(bias_np), 0, want_stats=want_stats)
            r = (ref.moe_prefill_layer if op == "prefill" else ref.moe_decode_layer)(l, x_np, T, bias_np, 0)
            gpu["compute"].synchronize()
            routing = buf.routing(ctx, gpu["compute"])
            for key in ("ids", "counts", "offsets", "perm", "inv_perm"):
                np.testing.assert_array_equal(routing[key], r[key], err_msg=f"{tag} {key}")
            check_out(H.dev_to_np_u16(buf.y), r["out_f64"], tag)
            if want_stats:
                assert {c: got_stats[c] for c in COUNTERS} == r["call_stats"], tag
        for ll in range(L):
            assert ctx.moe_cache_state(ll) == ref.moe_cache_state(ll), f"{tag}: slots of layer {ll}"
    torch.cuda.synchronize()
    for l in range(L):
        assert ctx.moe_get_stats(l) == ref.moe_get_stats(l), f"{name}: counters of layer {l}"
    ctx.close()
