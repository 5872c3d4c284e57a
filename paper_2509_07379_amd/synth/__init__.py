"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

Nothing here is part of the MoE method: the module only names the workload
shapes and fills tensors (Gaussian bf16 weights and activations, routing
traces, popularity biases).  The shapes imitate the model table of the paper
(Table I: Mixtral-8x7B 2-of-8, DeepSeekMoE 8-of-66 = 6 routed of 64 + 2 shared)
and its observations that prefill activates every expert (Section II-B) while
consecutive layers' choices are correlated (Section II-A, Fig. 2).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynth.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the generator with gcc (host only)."""
    src = os.path.join(_HERE, "synth.c")
    if force or not os.path.exists(_LIB_PATH):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", src, "-o", _LIB_PATH, "-lm"]
        )
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        for name, ptr in (("synth_normal_bf16", ctypes.c_void_p), ("synth_normal_f32", ctypes.c_void_p)):
            fn = getattr(lib, name)
            fn.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64,
                           ctypes.c_float, ptr]
            fn.restype = None
        lib.synth_quantize_e4m3_rows.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                                 ctypes.c_void_p]
        lib.synth_quantize_e4m3_rows.restype = None
        lib.synth_quantize_int4_g128.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                                 ctypes.c_void_p, ctypes.c_void_p]
        lib.synth_quantize_int4_g128.restype = None
        lib.synth_quantize_mxfp4.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                             ctypes.c_void_p]
        lib.synth_quantize_mxfp4.restype = None
        _lib = lib
    return _lib


# ---------------------------------------------------------------------------
# stream ids: one Gaussian stream per (tensor kind, layer, expert)
# ---------------------------------------------------------------------------
KIND_X, KIND_ROUTER, KIND_EXPERT, KIND_SHARED, KIND_PREDICTOR, KIND_ATTN, KIND_MLP = range(7)


def stream_id(kind: int, layer: int = 0, index: int = 0, step: int = 0) -> int:
    return ((kind * 4096 + layer) * 4096 + index) * 65536 + step


def normal_bf16_into(ptr: int, n: int, seed: int, stream: int, sigma: float, first: int = 0) -> None:
    """Fill n bf16 values at raw host address ptr (e.g. pinned memory)."""
    _load().synth_normal_bf16(seed, stream, first, n, sigma, ctypes.c_void_p(ptr))


def normal_bf16(shape, seed: int, stream: int, sigma: float) -> np.ndarray:
    """bf16 bit patterns (uint16) of sigma*N(0,1), C-contiguous."""
    out = np.empty(shape, dtype=np.uint16)
    normal_bf16_into(out.ctypes.data, out.size, seed, stream, sigma)
    return out


def normal_f32(shape, seed: int, stream: int, sigma: float) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().synth_normal_f32(seed, stream, 0, out.size, sigma, ctypes.c_void_p(out.ctypes.data))
    return out


def bf16_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32)


# ---------------------------------------------------------------------------
# workload shapes
# ---------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    d: int
    I: int
    E: int
    k: int
    T: int            # prompt tokens (prefill) or batch (decode)
    L: int = 1
    S: int = 0        # HBM cache slots per layer (0 = all experts resident)
    I_shared: int = 0
    steps: int = 0    # decode steps (0 = prefill workload)
    p_stay: float = 0.0
    top_m: int = 0    # predictor prefetch width
    zipf_s: float = 0.0
    seed: int = 0
    sigma_w: float = 0.02

    @property
    def blob_elems(self) -> int:
        return 3 * self.d * self.I

    @property
    def blob_bytes(self) -> int:
        return 6 * self.d * self.I

    @property
    def shared_blob_bytes(self) -> int:
        return 6 * self.d * self.I_shared


WORKLOADS = {
    "c1_tiny": Workload("c1_tiny", d=256, I=512, E=8, k=2, T=64, S=8),
    "c2_mixtral_prefill": Workload("c2_mixtral_prefill", d=4096, I=14336, E=8, k=2, T=2048, S=2),
    "c3_mixtral_decode": Workload("c3_mixtral_decode", d=4096, I=14336, E=8, k=2, T=1, L=32, S=3,
                                  steps=256, p_stay=0.6, top_m=3),
    "c4_deepseek_prefill": Workload("c4_deepseek_prefill", d=2048, I=1408, E=64, k=6, T=4096, L=28,
                                    S=16, I_shared=2816, zipf_s=1.1),
    "c5_qwen_decode": Workload("c5_qwen_decode", d=2048, I=1408, E=60, k=4, T=8, L=24, S=15,
                                I_shared=5632, steps=128, p_stay=0.5, top_m=8),
}


# ---------------------------------------------------------------------------
# tensors
# ---------------------------------------------------------------------------
def activations(w: Workload, layer: int = 0, step: int = 0, T: int | None = None) -> np.ndarray:
    """x [T, d] bf16 ~ N(0,1); independent per (layer, step): no residual chaining."""
    T = w.T if T is None else T
    return normal_bf16((T, w.d), w.seed, stream_id(KIND_X, layer, 0, step), 1.0)


def router_weight(w: Workload, layer: int = 0) -> np.ndarray:
    """Wr [E, d] bf16 ~ N(0, 0.02^2)."""
    return normal_bf16((w.E, w.d), w.seed, stream_id(KIND_ROUTER, layer), w.sigma_w)


def predictor_weight(w: Workload, layer: int = 0) -> np.ndarray:
    """Wp [E, d] bf16 ~ N(0, 0.02^2): the seeded linear stand-in for the paper's ExpertMLP."""
    return normal_bf16((w.E, w.d), w.seed, stream_id(KIND_PREDICTOR, layer), w.sigma_w)


def expert_blob(w: Workload, layer: int, e: int) -> np.ndarray:
    """One expert, flat bf16: [W_gate (I x d); W_up (I x d); W_down (d x I)], row-major."""
    return normal_bf16((w.blob_elems,), w.seed, stream_id(KIND_EXPERT, layer, e), w.sigma_w)


def expert_blob_into(ptr: int, w: Workload, layer: int, e: int) -> None:
    normal_bf16_into(ptr, w.blob_elems, w.seed, stream_id(KIND_EXPERT, layer, e), w.sigma_w)


def shared_blob(w: Workload, layer: int) -> np.ndarray | None:
    """Shared experts fused into one SwiGLU expert of width I_shared (same blob layout)."""
    if w.I_shared == 0:
        return None
    return normal_bf16((3 * w.d * w.I_shared,), w.seed, stream_id(KIND_SHARED, layer), w.sigma_w)


def split_blob(blob: np.ndarray, d: int, I: int):
    """Views (W_gate [I,d], W_up [I,d], W_down [d,I]) of a flat blob."""
    g = blob[: I * d].reshape(I, d)
    u = blob[I * d: 2 * I * d].reshape(I, d)
    dn = blob[2 * I * d: 3 * I * d].reshape(d, I)
    return g, u, dn


# ---------------------------------------------------------------------------
# routing structure
# ---------------------------------------------------------------------------
def zipf_route_bias(w: Workload, layer: int) -> np.ndarray:
    """bias[e] = ln p_e with p_e ~ rank(e)^-s, rank a seeded permutation per layer."""
    rng = np.random.default_rng([w.seed, 7001, layer])
    rank = rng.permutation(w.E) + 1
    p = rank.astype(np.float64) ** (-w.zipf_s)
    p /= p.sum()
    return np.log(p).astype(np.float32)


def markov_trace(w: Workload, steps: int | None = None) -> np.ndarray:
    """ids [steps, L, B, k] int32.

    Layer 0: uniform random k-subset.  Layer l: slot j keeps the previous layer's
    slot-j expert with probability p_stay, else draws uniformly over E; a
    duplicate within the token is redrawn uniformly from the unused ids.
    Tokens and steps are independent.
    """
    steps = w.steps if steps is None else steps
    B = w.T
    rng = np.random.default_rng([w.seed, 7002])
    out = np.empty((steps, w.L, B, w.k), dtype=np.int32)
    for s in range(steps):
        for b in range(B):
            prev = rng.choice(w.E, size=w.k, replace=False)
            out[s, 0, b] = prev
            for l in range(1, w.L):
                cur = []
                for j in range(w.k):
                    e = int(prev[j]) if rng.random() < w.p_stay else int(rng.integers(w.E))
                    if e in cur:
                        unused = [q for q in range(w.E) if q not in cur]
                        e = int(unused[int(rng.integers(len(unused)))])
                    cur.append(e)
                prev = np.asarray(cur)
                out[s, l, b] = prev
    return out


def trace_route_bias(ids_tk: np.ndarray, E: int, boost: float = 64.0) -> np.ndarray:
    """[T, E] fp32 additive router bias that forces the traced experts to win.

    Every traced expert gets the same shift, so the renormalised weights among
    them still come from the natural logits.
    """
    T = ids_tk.shape[0]
    b = np.zeros((T, E), dtype=np.float32)
    b[np.arange(T)[:, None], ids_tk] = boost
    return b


# ---------------------------------------------------------------------------
# ExpertMLP predictor (Section IV-B): shapes and seeded, untrained parameters
# ---------------------------------------------------------------------------
MLP_HIDDEN = (2048, 1024, 512, 256, 128, 64, 64)   # seven hidden layers, 2048 down to 64


def mlp_dims(L: int, E: int, k: int):
    """Layer sizes: state vector (L*k + E + k*E) -> seven hidden layers -> E logits."""
    return [L * k + E + k * E, *MLP_HIDDEN, E]


def mlp_params(dims, seed: int, layer: int = 0):
    """He-scaled bf16 weights [out, in], small fp32 biases, batch-norm affine (scale near 1, small
    shift) for every layer but the last.  Returns (weights, biases, scales, shifts)."""
    ws, bs, sc, sh = [], [], [], []
    n_fc = len(dims) - 1
    for l in range(n_fc):
        fan_in, out = dims[l], dims[l + 1]
        ws.append(normal_bf16((out, fan_in), seed, stream_id(KIND_MLP, layer, 4 * l), float(np.sqrt(2.0 / fan_in))))
        bs.append(normal_f32((out,), seed, stream_id(KIND_MLP, layer, 4 * l + 1), 0.05))
        if l + 1 < n_fc:
            sc.append((1.0 + normal_f32((out,), seed, stream_id(KIND_MLP, layer, 4 * l + 2), 0.1)).astype(np.float32))
            sh.append(normal_f32((out,), seed, stream_id(KIND_MLP, layer, 4 * l + 3), 0.1))
    return ws, bs, sc, sh


# ---------------------------------------------------------------------------
# expert blobs quantised for the host link: e4m3 codes + one fp32 scale per output row
# ---------------------------------------------------------------------------
def q8_blob_bytes(d: int, I: int) -> int:
    """[scales fp32: 2I gate/up rows, d down rows][W_gate codes I x d][W_up codes I x d][W_down codes d x I]"""
    return 4 * (2 * I + d) + 3 * d * I


def quantize_blob_into(ptr: int, blob_bf16: np.ndarray, d: int, I: int) -> None:
    """Quantise a bf16 expert blob ([W_gate; W_up] (2I x d), W_down (d x I)) into the byte layout
    above at raw host address ptr (offline preparation of the CPU expert cache)."""
    blob_bf16 = np.ascontiguousarray(blob_bf16, dtype=np.uint16)
    assert blob_bf16.size == 3 * d * I
    lib = _load()
    scales_bytes = 4 * (2 * I + d)
    lib.synth_quantize_e4m3_rows(ctypes.c_void_p(blob_bf16.ctypes.data), 2 * I, d, ctypes.c_void_p(ptr),
                                 ctypes.c_void_p(ptr + scales_bytes))
    lib.synth_quantize_e4m3_rows(ctypes.c_void_p(blob_bf16.ctypes.data + 2 * (2 * I * d)), d, I,
                                 ctypes.c_void_p(ptr + 4 * 2 * I), ctypes.c_void_p(ptr + scales_bytes + 2 * I * d))


# ---------------------------------------------------------------------------
# expert blobs in 4 bits: unsigned codes in groups of 128 along a row, fp32 scale + zero point per group
# ---------------------------------------------------------------------------
def q4_layout(d: int, I: int) -> dict:
    """Byte offsets inside a 4-bit blob:
    [scales of [W_gate; W_up] (2I x d/128 fp32)][scales of W_down (d x I/128 fp32)]
    [zero points of [W_gate; W_up] (bytes)][zero points of W_down (bytes)][pad to 16]
    [codes of [W_gate; W_up] (2I x d/2 bytes)][codes of W_down (d x I/2 bytes)]"""
    assert d % 128 == 0 and I % 128 == 0
    n_up, n_dn = 2 * I * (d // 128), d * (I // 128)
    lay = dict(scales_up=0, scales_down=4 * n_up, zeros_up=4 * (n_up + n_dn), zeros_down=4 * (n_up + n_dn) + n_up)
    meta = (5 * (n_up + n_dn) + 15) // 16 * 16
    lay.update(meta=meta, codes_up=meta, codes_down=meta + I * d, total=meta + 3 * d * I // 2)
    return lay


def q4_blob_bytes(d: int, I: int) -> int:
    return q4_layout(d, I)["total"]


def quantize4_blob_into(ptr: int, blob_bf16: np.ndarray, d: int, I: int) -> None:
    """Quantise a bf16 expert blob into the 4-bit layout at raw host address ptr (offline preparation)."""
    blob_bf16 = np.ascontiguousarray(blob_bf16, dtype=np.uint16)
    assert blob_bf16.size == 3 * d * I
    lib, lay = _load(), q4_layout(d, I)
    vp = ctypes.c_void_p
    lib.synth_quantize_int4_g128(vp(blob_bf16.ctypes.data), 2 * I, d, vp(ptr + lay["scales_up"]),
                                 vp(ptr + lay["zeros_up"]), vp(ptr + lay["codes_up"]))
    lib.synth_quantize_int4_g128(vp(blob_bf16.ctypes.data + 2 * (2 * I * d)), d, I, vp(ptr + lay["scales_down"]),
                                 vp(ptr + lay["zeros_down"]), vp(ptr + lay["codes_down"]))


# ---------------------------------------------------------------------------
# expert blobs in MXFP4: e2m1 codes, blocks of 32 along a row share a power-of-two scale (one byte)
# ---------------------------------------------------------------------------
def mx4_layout(d: int, I: int) -> dict:
    """Byte offsets inside an MXFP4 blob:
    [scales of [W_gate; W_up] (2I x d/32 bytes)][scales of W_down (d x I/32 bytes)][pad to 16]
    [codes of [W_gate; W_up] (2I x d/2 bytes)][codes of W_down (d x I/2 bytes)]"""
    assert d % 32 == 0 and I % 32 == 0
    n_up, n_dn = 2 * I * (d // 32), d * (I // 32)
    meta = (n_up + n_dn + 15) // 16 * 16
    return dict(scales_up=0, scales_down=n_up, meta=meta, codes_up=meta, codes_down=meta + I * d,
                total=meta + 3 * d * I // 2)


def mx4_blob_bytes(d: int, I: int) -> int:
    return mx4_layout(d, I)["total"]


def quantize_mx4_blob_into(ptr: int, blob_bf16: np.ndarray, d: int, I: int) -> None:
    """Quantise a bf16 expert blob into the MXFP4 layout at raw host address ptr (offline preparation)."""
    blob_bf16 = np.ascontiguousarray(blob_bf16, dtype=np.uint16)
    assert blob_bf16.size == 3 * d * I
    lib, lay = _load(), mx4_layout(d, I)
    vp = ctypes.c_void_p
    lib.synth_quantize_mxfp4(vp(blob_bf16.ctypes.data), 2 * I, d, vp(ptr + lay["scales_up"]), vp(ptr + lay["codes_up"]))
    lib.synth_quantize_mxfp4(vp(blob_bf16.ctypes.data + 2 * (2 * I * d)), d, I, vp(ptr + lay["scales_down"]),
                             vp(ptr + lay["codes_down"]))
