"""ctypes binding of libmoe_offload.so: argument marshalling only.

Function names and arguments mirror include/moe_offload.h.  Device buffers are torch CUDA
tensors (plumbing: memory and streams); every step of the layer runs in the library's HIP
kernels.  There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_offload.so")

K_ROUTER, K_DISPATCH, K_GEMM1, K_GEMM2, K_GEMV1, K_GEMV2, K_COMBINE, K_PREDICTOR, K_COUNT = range(9)
KERNEL_NAMES = ["router", "dispatch", "gemm1", "gemm2", "gemv1", "gemv2", "combine", "predictor"]

EXPORTS = [
    "moe_last_error", "moe_create", "moe_destroy", "moe_workspace_bytes", "moe_bind_layer",
    "expert_cache_prefetch", "predictor_score", "moe_prefill_layer", "moe_decode_layer",
    "moe_debug_routing", "moe_get_stats", "moe_reset_stats", "moe_cache_invalidate", "moe_cache_state", "moe_set_profiling",
    "moe_get_kernel_times", "moe_dense_gemm_bf16",
    "predictor_mlp_score", "moe_state_create", "moe_state_destroy", "moe_state_dim", "moe_state_record",
    "moe_state_clear", "moe_state_vector", "moe_host_blob_bytes", "moe_cache_bytes", "moe_debug_logits",
    "moe_decode_layer_static",
]
# exported for the parity tests only, declared in csrc/moe_tuning.h (not part of the public header)
INTERNAL_EXPORTS = ["moe_tune", "moe_inject_failure", "moe_debug_gemm_choice", "moe_debug_plans"]


class MoeConfig(Structure):
    _fields_ = [(n, c_int32) for n in
                ("d", "I", "E", "k", "n_layers", "cache_slots", "I_shared", "renormalize", "shared_slots", "host_format")]


class MoeStats(Structure):
    _fields_ = ([(n, c_int32) for n in ("hits", "misses", "prefetch_issued", "prefetch_useful",
                                        "prefetch_dropped", "layer_calls")] + [("bytes_h2d", c_int64)] +
                [("prefetch_ready", c_int32), ("prefetch_stalled", c_int32), ("wait_ms", c_float),
                 ("compute_ms", c_float)])
    CACHE_COUNTERS = ("hits", "misses", "prefetch_issued", "prefetch_useful", "prefetch_dropped", "layer_calls",
                      "bytes_h2d")

    def as_dict(self, full=False):
        """The cache counters (what the cache simulator also keeps); full: every field."""
        d = {n: int(getattr(self, n)) for n in self.CACHE_COUNTERS}
        if full:
            d.update(prefetch_ready=int(self.prefetch_ready), prefetch_stalled=int(self.prefetch_stalled),
                     wait_ms=float(self.wait_ms), compute_ms=float(self.compute_ms))
        return d


class MoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"moe_offload error {code}: {msg}")
        self.code = code


_lib = None


def load():
    """Loads the C-ABI library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2509_07379_amd.build` "
            "(hipcc, gfx950); the MoE path has no fallback")
    lib = ctypes.CDLL(LIB_PATH)
    vp = c_void_p
    lib.moe_last_error.restype = c_char_p
    lib.moe_last_error.argtypes = []
    lib.moe_create.argtypes = [POINTER(MoeConfig), POINTER(vp)]
    lib.moe_destroy.argtypes = [vp]
    lib.moe_workspace_bytes.argtypes = [POINTER(MoeConfig), c_int]
    lib.moe_workspace_bytes.restype = c_size_t
    lib.moe_bind_layer.argtypes = [vp, c_int, POINTER(vp), vp, vp, vp, POINTER(c_int32)]
    lib.expert_cache_prefetch.argtypes = [vp, c_int, POINTER(c_int32), c_int, vp]
    lib.predictor_score.argtypes = [vp, c_int, vp, c_int, vp, c_int, vp, vp, vp]
    layer_args = [vp, c_int, vp, c_int, vp, c_int, vp, vp, c_size_t, vp, vp, POINTER(MoeStats)]
    lib.moe_prefill_layer.argtypes = layer_args
    lib.moe_decode_layer.argtypes = layer_args
    lib.moe_decode_layer_static.argtypes = [vp, c_int, vp, c_int, vp, c_int, vp, vp, vp, POINTER(MoeStats)]
    lib.moe_debug_routing.argtypes = [vp, vp, c_int, vp, vp, vp, vp, vp, vp, vp]
    lib.moe_debug_logits.argtypes = [vp, vp, c_int, vp, vp]
    lib.moe_get_stats.argtypes = [vp, c_int, POINTER(MoeStats)]
    lib.moe_reset_stats.argtypes = [vp]
    lib.moe_cache_state.argtypes = [vp, c_int, POINTER(c_int32)]
    lib.moe_cache_invalidate.argtypes = [vp, c_int]
    lib.moe_set_profiling.argtypes = [vp, c_int]
    lib.moe_get_kernel_times.argtypes = [vp, POINTER(c_float), POINTER(c_int32)]
    lib.moe_dense_gemm_bf16.argtypes = [vp, vp, vp, c_int, c_int, c_int, vp]
    lib.moe_tune.argtypes = [vp, c_int, c_int]
    lib.moe_tune.restype = c_int
    lib.moe_inject_failure.argtypes = [c_int]
    lib.moe_debug_plans.argtypes = [vp, vp, c_int, POINTER(c_int32), vp]
    lib.moe_debug_plans.restype = c_int
    lib.moe_inject_failure.restype = c_int
    lib.moe_debug_gemm_choice.argtypes = [c_int, c_int, c_int64, c_int, c_int, c_int, c_int, c_int64, c_int, c_int]
    lib.moe_debug_gemm_choice.restype = c_int
    lib.predictor_mlp_score.argtypes = [vp, vp, POINTER(c_int32), c_int, POINTER(vp), POINTER(vp), POINTER(vp),
                                        POINTER(vp), vp, c_int, vp, vp, vp]
    lib.moe_state_create.argtypes = [c_int, c_int, c_int, POINTER(c_float), POINTER(c_float), POINTER(vp)]
    lib.moe_state_destroy.argtypes = [vp]
    lib.moe_state_dim.argtypes = [vp]
    lib.moe_state_record.argtypes = [vp, c_int, POINTER(c_int32)]
    lib.moe_state_clear.argtypes = [vp]
    lib.moe_state_vector.argtypes = [vp, c_int, vp]
    for name in ("moe_host_blob_bytes", "moe_cache_bytes"):
        getattr(lib, name).argtypes = [POINTER(MoeConfig)]
        getattr(lib, name).restype = c_size_t
    for name in EXPORTS:
        if name not in ("moe_last_error", "moe_workspace_bytes", "moe_host_blob_bytes", "moe_cache_bytes"):
            getattr(lib, name).restype = c_int
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise MoeError(rc, load().moe_last_error().decode())


def _ptr(t):
    """Raw address of a torch tensor (or None / int passthrough)."""
    if t is None:
        return None
    if isinstance(t, int):
        return c_void_p(t)
    return c_void_p(t.data_ptr())


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return c_void_p(s)
    return c_void_p(s.cuda_stream)


class MoeContext:
    """Owner of a moe_ctx handle; methods carry the C function names."""

    def __init__(self, d, I, E, k, n_layers=1, cache_slots=None, I_shared=0, renormalize=True,
                 shared_slots=False, host_format=0):
        self.lib = load()
        self.cfg = MoeConfig(d, I, E, k, n_layers, E if cache_slots is None else cache_slots, I_shared,
                             1 if renormalize else 0, 1 if shared_slots else 0, int(host_format))
        self._h = c_void_p()
        _check(self.lib.moe_create(byref(self.cfg), byref(self._h)))
        self._keep = {}

    def close(self):
        if self._h:
            self.lib.moe_destroy(self._h)
            self._h = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def moe_workspace_bytes(self, T: int) -> int:
        return int(self.lib.moe_workspace_bytes(byref(self.cfg), T))

    def moe_host_blob_bytes(self) -> int:
        return int(self.lib.moe_host_blob_bytes(byref(self.cfg)))

    def moe_cache_bytes(self) -> int:
        return int(self.lib.moe_cache_bytes(byref(self.cfg)))

    def moe_bind_layer(self, layer, host_blob_ptrs, router_w, shared_blob, slots, initial_resident=None):
        E, S = self.cfg.E, self.cfg.cache_slots
        arr = (c_void_p * E)(*[int(p) for p in host_blob_ptrs])
        init = None
        if initial_resident is not None:
            assert len(initial_resident) == S
            init = (c_int32 * S)(*[int(e) for e in initial_resident])
        self._keep[layer] = (arr, router_w, shared_blob, slots)
        _check(self.lib.moe_bind_layer(self._h, layer, arr, _ptr(router_w), _ptr(shared_blob), _ptr(slots), init))

    def expert_cache_prefetch(self, layer, ids, copy_stream):
        ids = [int(i) for i in ids]
        arr = (c_int32 * max(1, len(ids)))(*ids)
        _check(self.lib.expert_cache_prefetch(self._h, layer, arr, len(ids), _stream(copy_stream)))

    def predictor_score(self, layer, x, T, wp, m, pinned_topm, stream, scores=None):
        _check(self.lib.predictor_score(self._h, layer, _ptr(x), T, _ptr(wp), m, _ptr(scores), _ptr(pinned_topm),
                                        _stream(stream)))

    def predictor_mlp_score(self, state, dims, weights, biases, scales, shifts, act, m, pinned_topm, stream,
                            scores=None):
        """state / act / scores / pinned_topm: tensors; weights / biases / scales / shifts: lists of
        device tensors, one per layer (scales, shifts: one per hidden layer)."""
        n_fc = len(weights)
        dims_a = (c_int32 * (n_fc + 1))(*[int(v) for v in dims])

        def parr(ts):
            a = (c_void_p * n_fc)()
            for i, t in enumerate(ts):
                a[i] = t.data_ptr()
            return a

        _check(self.lib.predictor_mlp_score(self._h, _ptr(state), dims_a, n_fc, parr(weights), parr(biases),
                                            parr(scales), parr(shifts), _ptr(act), m, _ptr(scores),
                                            _ptr(pinned_topm), _stream(stream)))

    def _layer(self, fn, layer, x, T, y, ws, compute_stream, copy_stream, route_bias, bias_stride, want_stats):
        st = MoeStats() if want_stats else None
        _check(fn(self._h, layer, _ptr(x), T, _ptr(route_bias), bias_stride, _ptr(y), _ptr(ws),
                  ws.numel() * ws.element_size(), _stream(compute_stream), _stream(copy_stream),
                  byref(st) if want_stats else None))
        return st.as_dict(full=True) if want_stats else None

    def moe_prefill_layer(self, layer, x, T, y, ws, compute_stream, copy_stream, route_bias=None,
                          bias_stride=0, want_stats=False):
        """want_stats: pass a moe_stats for this call's own counters and return it as a dict."""
        return self._layer(self.lib.moe_prefill_layer, layer, x, T, y, ws, compute_stream, copy_stream,
                           route_bias, bias_stride, want_stats)

    def moe_decode_layer(self, layer, x, T, y, ws, compute_stream, copy_stream, route_bias=None,
                         bias_stride=0, want_stats=False):
        return self._layer(self.lib.moe_decode_layer, layer, x, T, y, ws, compute_stream, copy_stream,
                           route_bias, bias_stride, want_stats)

    def moe_decode_layer_static(self, layer, x, T, y, compute_stream, copy_stream, route_bias=None,
                                bias_stride=0, want_stats=False):
        """moe_decode_layer on the library's static workspace (no workspace argument, nothing allocated)."""
        st = MoeStats() if want_stats else None
        _check(self.lib.moe_decode_layer_static(self._h, layer, _ptr(x), T, _ptr(route_bias), bias_stride, _ptr(y),
                                                _stream(compute_stream), _stream(copy_stream),
                                                byref(st) if want_stats else None))
        return st.as_dict(full=True) if want_stats else None

    def moe_debug_routing(self, ws, T, ids=None, w=None, counts=None, offsets=None, perm=None,
                          inv_perm=None, stream=None):
        _check(self.lib.moe_debug_routing(self._h, _ptr(ws), T, _ptr(ids), _ptr(w), _ptr(counts),
                                          _ptr(offsets), _ptr(perm), _ptr(inv_perm), _stream(stream)))

    def moe_debug_logits(self, ws, T, logits, stream=None):
        _check(self.lib.moe_debug_logits(self._h, _ptr(ws), T, _ptr(logits), _stream(stream)))

    def moe_get_stats(self, layer=-1, full=False) -> dict:
        st = MoeStats()
        _check(self.lib.moe_get_stats(self._h, layer, byref(st)))
        return st.as_dict(full)

    def moe_debug_plans(self, ws, T, stream):
        """Internal parity hook: the gate/up and down GEMM work plans of the last prefill call, as dicts."""
        n = 3 + 9 + 65 + 128
        arr = (c_int32 * (2 * n))()
        _check(self.lib.moe_debug_plans(self._h, _ptr(ws), T, arr, _stream(stream)))
        out = []
        for i in range(2):
            v = list(arr[i * n:(i + 1) * n])
            out.append(dict(n_items=v[0], s_full=v[1], s_rem=v[2], xcd_begin=v[3:12], item_begin=v[12:77],
                            queue=v[77::16][:8]))
        return out

    def moe_tune(self, mode: int, variant: int):
        """Internal test / tuning hook (csrc/moe_tuning.h): forces a kernel variant for this context."""
        _check(self.lib.moe_tune(self._h, mode, variant))

    def moe_reset_stats(self):
        _check(self.lib.moe_reset_stats(self._h))

    def moe_cache_invalidate(self, layer):
        _check(self.lib.moe_cache_invalidate(self._h, layer))

    def moe_cache_state(self, layer):
        S = self.cfg.cache_slots
        arr = (c_int32 * S)()
        _check(self.lib.moe_cache_state(self._h, layer, arr))
        return list(arr)

    def moe_set_profiling(self, on: bool):
        _check(self.lib.moe_set_profiling(self._h, 1 if on else 0))

    def moe_get_kernel_times(self):
        ms = (c_float * K_COUNT)()
        n = (c_int32 * K_COUNT)()
        _check(self.lib.moe_get_kernel_times(self._h, ms, n))
        return {KERNEL_NAMES[i]: (float(ms[i]), int(n[i])) for i in range(K_COUNT)}


def moe_dense_gemm_bf16(a, b, c, M, N, K, stream=None):
    _check(load().moe_dense_gemm_bf16(_ptr(a), _ptr(b), _ptr(c), M, N, K, _stream(stream)))


class MoeState:
    """State Constructor handle (host bookkeeping of the selections of one decode round)."""

    def __init__(self, n_layers, n_experts, k, popularity, affinity):
        import numpy as np
        self.lib = load()
        P = np.ascontiguousarray(popularity, dtype=np.float32)
        A = np.ascontiguousarray(affinity, dtype=np.float32)
        assert P.shape == (n_layers, n_experts) and A.shape == (max(n_layers - 1, 0), n_experts, n_experts)
        self._h = c_void_p()
        _check(self.lib.moe_state_create(n_layers, n_experts, k, P.ctypes.data_as(POINTER(c_float)),
                                         A.ctypes.data_as(POINTER(c_float)), byref(self._h)))
        self.k = k

    def close(self):
        if self._h:
            self.lib.moe_state_destroy(self._h)
            self._h = c_void_p()

    def moe_state_dim(self) -> int:
        return int(self.lib.moe_state_dim(self._h))

    def moe_state_record(self, layer, ids):
        arr = (c_int32 * self.k)(*[int(i) for i in ids])
        _check(self.lib.moe_state_record(self._h, layer, arr))

    def moe_state_clear(self):
        _check(self.lib.moe_state_clear(self._h))

    def moe_state_vector(self, layer, out):
        """out: a host tensor (plain or pinned) of moe_state_dim() fp32 values."""
        _check(self.lib.moe_state_vector(self._h, layer, _ptr(out)))
