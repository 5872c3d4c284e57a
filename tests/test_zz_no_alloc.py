"""moe_decode_layer_static, the decode entry point that allocates nothing (its workspace is a static
device array of the library), against moe_decode_layer on the same inputs: same kernels, so the same
bits, routing tables and cache counters.  Collected last on purpose.  Needs an MI355X."""
import numpy as np
import pytest

from paper_2509_07379_amd import synth as S

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

from test_gpu_parity import check_out, gpu  # noqa: E402,F401  (fixture + tolerance)


@pytest.mark.parametrize("slots,shared", [(16, 256), (5, 256), (16, 0)])
def test_static_workspace_decode_matches_the_workspace_argument(gpu, oracle, slots, shared):
    """Two contexts over the same expert pool run the same two decode calls, the second on fewer
    tokens than the first: one through moe_decode_layer with a caller's workspace, one through
    moe_decode_layer_static.  With 5 slots of 16 experts the calls also fetch."""
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("no_alloc", d=512, I=256, E=16, k=4, T=8, I_shared=shared, seed=61)
    pool = H.HostPool(w, 0)
    blobs = [pool.blob_np(e) for e in range(w.E)]
    init = list(range(slots)) if slots == w.E else None
    ctxs, lays = [], []
    for _ in range(2):
        ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, slots, w.I_shared)
        lays.append(H.DeviceLayer(ctx, w, 0, pool, init, poison=init is None))
        ctxs.append(ctx)
    for step, T in enumerate((8, 3, 1)):
        x_np = S.activations(w, 0, step, T=T)
        x = H.np_to_dev(x_np)
        buf = H.Buffers(ctxs[0], T)
        y_static = torch.full((T, w.d), 0x7FC0, dtype=torch.int16, device="cuda")
        st_arg = ctxs[0].moe_decode_layer(0, x, T, buf.y, buf.ws, gpu["compute"], gpu["copy"], want_stats=True)
        gpu["compute"].synchronize()
        before = torch.cuda.memory_allocated()
        st_static = ctxs[1].moe_decode_layer_static(0, x, T, y_static, gpu["compute"], gpu["copy"], want_stats=True)
        gpu["compute"].synchronize()
        assert torch.cuda.memory_allocated() == before
        ref = oracle.moe_layer(x_np, lays[0].router_np, blobs, w.k, shared_blob=lays[0].shared_np, I=w.I,
                               I_shared=w.I_shared)
        got = H.dev_to_np_u16(y_static)
        np.testing.assert_array_equal(got, H.dev_to_np_u16(buf.y), err_msg=f"call {step} (T={T})")
        check_out(got, ref["out_f64"], f"static workspace, call {step}")
        for key in ("hits", "misses", "bytes_h2d", "prefetch_useful"):
            assert st_static[key] == st_arg[key], key
        assert ctxs[1].moe_cache_state(0) == ctxs[0].moe_cache_state(0)
    for ctx in ctxs:
        ctx.close()


def test_static_workspace_refuses_what_does_not_fit(gpu):
    H, B = gpu["harness"], gpu["binding"]
    w = S.Workload("no_alloc_big", d=512, I=256, E=16, k=4, T=8, seed=61)
    ctx = B.MoeContext(w.d, w.I, w.E, w.k, 1, w.E)
    pool = H.HostPool(w, 0)
    H.DeviceLayer(ctx, w, 0, pool, list(range(w.E)))
    T = 1
    while ctx.moe_workspace_bytes(T) <= 8 << 20:
        T *= 2
    x = torch.zeros((T, w.d), dtype=torch.int16, device="cuda")
    y = torch.zeros_like(x)
    with pytest.raises(B.MoeError) as e:
        ctx.moe_decode_layer_static(0, x, T, y, gpu["compute"], gpu["copy"])
    assert e.value.code == -5 and "static" in str(e.value)
    ctx.close()
