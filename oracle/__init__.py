"""CPU oracle of the MoE layer and of the expert-cache bookkeeping.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this; only
tests, the smoke check and the benchmark's cpu_baseline leg do.  The numerical
part is plain C (moe_oracle.c, loaded through ctypes); the cache simulator is
plain Python (cache_sim.py).  Neither shares code with the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    src = os.path.join(_HERE, "moe_oracle.c")
    if force or not os.path.exists(_LIB_PATH):
        subprocess.check_call([
            "gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
            src, "-o", _LIB_PATH, "-lm",
        ])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        lib.ref_router_logits.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp]
        lib.ref_topk_weights.argtypes = [vp, ci, ci, ci, ci, vp, vp]
        lib.ref_dispatch.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp]
        lib.ref_expert_ffn.argtypes = [vp, vp, ci, ci, vp]
        lib.ref_moe_tokens.argtypes = [vp, ci, ci, ci, vp, vp, ci, vp, vp, vp, ci, vp, vp]
        lib.ref_predictor_score.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp]
        lib.ref_mlp_forward.argtypes = [vp, vp, ci, vp, vp, vp, vp, vp, vp]
        lib.ref_mlp_forward.restype = None
        lib.ref_e4m3_value.argtypes = [ci]
        lib.ref_e4m3_value.restype = ctypes.c_float
        lib.ref_dequant_e4m3_rows.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int64, vp]
        lib.ref_dequant_e4m3_rows.restype = None
        lib.ref_dequant_int4_g128_rows.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int64, vp]
        lib.ref_dequant_int4_g128_rows.restype = None
        lib.ref_e2m1_value.argtypes = [ci]
        lib.ref_e2m1_value.restype = ctypes.c_double
        lib.ref_dequant_mxfp4_rows.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int64, vp]
        lib.ref_dequant_mxfp4_rows.restype = None
        lib.ref_bf16_from_f64.argtypes = [ctypes.c_double]
        lib.ref_bf16_from_f64.restype = ctypes.c_uint16
        for f in ("ref_router_logits", "ref_topk_weights", "ref_dispatch", "ref_expert_ffn",
                  "ref_moe_tokens", "ref_predictor_score"):
            getattr(lib, f).restype = None
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bf16 tensors travel as uint16 bit patterns"
    return a


def bf16_from_f64(v: float) -> int:
    return int(_load().ref_bf16_from_f64(float(v)))


def router_logits(x, wr, bias=None, want_f64=False):
    """logits [T,E] fp32 in the fixed summation order (+ fp64 values on request)."""
    x, wr = _u16(x), _u16(wr)
    T, d = x.shape
    E = wr.shape[0]
    assert wr.shape[1] == d
    stride = 0
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        if bias.ndim == 2:
            assert bias.shape == (T, E)
            stride = E
        else:
            assert bias.shape == (E,)
    l32 = np.empty((T, E), dtype=np.float32)
    l64 = np.empty((T, E), dtype=np.float64) if want_f64 else None
    _load().ref_router_logits(_p(x), _p(wr), _p(bias), stride, T, d, E, _p(l32), _p(l64))
    return (l32, l64) if want_f64 else l32


def topk_weights(logits, k, renormalize=True):
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    assert 1 <= k <= E
    ids = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float32)
    _load().ref_topk_weights(_p(logits), T, E, k, 1 if renormalize else 0, _p(ids), _p(w))
    return ids, w


def dispatch(ids, E):
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, k = ids.shape
    counts = np.empty(E, dtype=np.int32)
    offsets = np.empty(E + 1, dtype=np.int32)
    perm = np.empty(T * k, dtype=np.int32)
    inv = np.empty(T * k, dtype=np.int32)
    _load().ref_dispatch(_p(ids), T, k, E, _p(counts), _p(offsets), _p(perm), _p(inv))
    return counts, offsets, perm, inv


def expert_ffn(x_row, blob, d, I):
    x_row, blob = _u16(x_row), _u16(blob)
    assert x_row.size == d and blob.size == 3 * d * I
    y = np.empty(d, dtype=np.float64)
    _load().ref_expert_ffn(_p(x_row), _p(blob), d, I, _p(y))
    return y


def moe_tokens(x, blobs, ids, w, sel=None, shared_blob=None, I=None, I_shared=0):
    """Layer output for tokens `sel` (default: all).  blobs: list of E flat uint16 arrays or
    raw host addresses (ints).  Returns (out_bf16 [n_sel,d] uint16, out_f64 [n_sel,d])."""
    x = _u16(x)
    T, d = x.shape
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    k = ids.shape[1]
    keep = []
    ptrs = (ctypes.c_void_p * len(blobs))()
    for e, b in enumerate(blobs):
        if isinstance(b, (int, np.integer)):
            ptrs[e] = int(b)
        else:
            b = _u16(b)
            if I is None:
                I = b.size // (3 * d)
            assert b.size == 3 * d * I
            keep.append(b)
            ptrs[e] = b.ctypes.data
    assert I is not None
    if sel is None:
        sel = np.arange(T, dtype=np.int32)
    sel = np.ascontiguousarray(sel, dtype=np.int32)
    if shared_blob is not None:
        shared_blob = _u16(shared_blob)
        assert I_shared > 0 and shared_blob.size == 3 * d * I_shared
    out16 = np.empty((sel.size, d), dtype=np.uint16)
    out64 = np.empty((sel.size, d), dtype=np.float64)
    _load().ref_moe_tokens(_p(x), d, I, k, ctypes.cast(ptrs, ctypes.c_void_p), _p(shared_blob),
                           I_shared if shared_blob is not None else 0, _p(ids), _p(w), _p(sel),
                           int(sel.size), _p(out16), _p(out64))
    return out16, out64


def moe_layer(x, wr, blobs, k, bias=None, renormalize=True, sel=None, shared_blob=None,
              I=None, I_shared=0):
    """Whole layer: gate -> top-k -> grouping -> experts -> weighted sum.  Returns a dict."""
    E = wr.shape[0]
    logits = router_logits(x, wr, bias)
    ids, w = topk_weights(logits, k, renormalize)
    counts, offsets, perm, inv = dispatch(ids, E)
    out16, out64 = moe_tokens(x, blobs, ids, w, sel, shared_blob, I, I_shared)
    return dict(logits=logits, ids=ids, w=w, counts=counts, offsets=offsets, perm=perm,
                inv_perm=inv, out=out16, out_f64=out64)


def predictor_score(x, wp, m):
    x, wp = _u16(x), _u16(wp)
    B, d = x.shape
    E = wp.shape[0]
    scores = np.empty(E, dtype=np.float32)
    top = np.empty(m, dtype=np.int32)
    _load().ref_predictor_score(_p(x), _p(wp), B, d, E, m, _p(scores), _p(top))
    return scores, top


def mlp_forward(s, weights, biases, scales, shifts):
    """ExpertMLP forward (Section IV-B).  weights[l]: uint16 (bf16 bits) [out, in]; biases[l] fp32
    [out]; scales[l], shifts[l] fp32 [out] for every layer but the last.  Returns the experts'
    logits in the fixed fp32 order and in fp64."""
    n_fc = len(weights)
    ws = [_u16(w) for w in weights]
    dims = np.array([ws[0].shape[1]] + [w.shape[0] for w in ws], dtype=np.int32)
    s = np.ascontiguousarray(s, dtype=np.float32)
    assert s.shape == (dims[0],)
    bs = [np.ascontiguousarray(b, dtype=np.float32) for b in biases]
    sc = [np.ascontiguousarray(a, dtype=np.float32) for a in scales]
    sh = [np.ascontiguousarray(a, dtype=np.float32) for a in shifts]
    assert len(bs) == n_fc and len(sc) == n_fc - 1 and len(sh) == n_fc - 1

    def parr(arrs, n):
        out = (ctypes.c_void_p * n)()
        for i, a in enumerate(arrs):
            out[i] = a.ctypes.data
        return out

    pw, pb, psc, psh = parr(ws, n_fc), parr(bs, n_fc), parr(sc, n_fc), parr(sh, n_fc)
    l32 = np.empty(dims[-1], dtype=np.float32)
    l64 = np.empty(dims[-1], dtype=np.float64)
    _load().ref_mlp_forward(_p(s), _p(dims), n_fc, ctypes.cast(pw, ctypes.c_void_p), ctypes.cast(pb, ctypes.c_void_p),
                            ctypes.cast(psc, ctypes.c_void_p), ctypes.cast(psh, ctypes.c_void_p), _p(l32), _p(l64))
    return l32, l64


def top_m(scores, m):
    """The m best (score descending, lower index on ties)."""
    order = sorted(range(len(scores)), key=lambda e: (-float(scores[e]), e))
    return np.array(order[:m], dtype=np.int32)


def e4m3_value(code: int) -> float:
    return float(_load().ref_e4m3_value(int(code)))


def dequant_blob(qblob, d: int, I: int) -> np.ndarray:
    """8-bit expert blob ([scales fp32: 2I, d][W_gate codes][W_up codes][W_down codes]) -> the bf16 blob
    ([W_gate; W_up] (2I x d), W_down (d x I)) the layer computes with."""
    q = np.ascontiguousarray(qblob).view(np.uint8).ravel()
    sb = 4 * (2 * I + d)
    assert q.size == sb + 3 * d * I
    scales = q[:sb].view(np.float32)
    out = np.empty(3 * d * I, dtype=np.uint16)
    codes = q[sb:]
    lib = _load()
    lib.ref_dequant_e4m3_rows(_p(codes[:2 * I * d]), _p(scales[:2 * I]), 2 * I, d, _p(out[:2 * I * d]))
    lib.ref_dequant_e4m3_rows(_p(codes[2 * I * d:]), _p(scales[2 * I:]), d, I, _p(out[2 * I * d:]))
    return out


def dequant4_blob(qblob, d: int, I: int) -> np.ndarray:
    """4-bit expert blob -> the bf16 blob the layer computes with.  Layout: fp32 scales of [W_gate; W_up]
    (2I x d/128) and of W_down (d x I/128), their zero points (bytes, same shapes), padding to 16 bytes,
    then the codes of [W_gate; W_up] (2I x d/2 bytes) and of W_down (d x I/2 bytes)."""
    q = np.ascontiguousarray(qblob).view(np.uint8).ravel()
    n_up, n_dn = 2 * I * (d // 128), d * (I // 128)
    meta = (5 * (n_up + n_dn) + 15) // 16 * 16
    assert d % 128 == 0 and I % 128 == 0 and q.size == meta + 3 * d * I // 2
    scales = q[:4 * (n_up + n_dn)].view(np.float32)
    zeros = q[4 * (n_up + n_dn):5 * (n_up + n_dn)]
    codes = q[meta:]
    out = np.empty(3 * d * I, dtype=np.uint16)
    lib = _load()
    lib.ref_dequant_int4_g128_rows(_p(codes[:I * d]), _p(scales[:n_up]), _p(zeros[:n_up]), 2 * I, d, _p(out[:2 * I * d]))
    lib.ref_dequant_int4_g128_rows(_p(codes[I * d:]), _p(scales[n_up:]), _p(zeros[n_up:]), d, I, _p(out[2 * I * d:]))
    return out


def e2m1_value(code: int) -> float:
    return float(_load().ref_e2m1_value(int(code)))


def dequant_mx4_blob(qblob, d: int, I: int) -> np.ndarray:
    """MXFP4 expert blob -> the bf16 blob the layer computes with (exact: no rounding).  Layout: scale
    bytes of [W_gate; W_up] (2I x d/32) and of W_down (d x I/32), padding to 16 bytes, then the codes of
    [W_gate; W_up] (2I x d/2 bytes) and of W_down (d x I/2 bytes)."""
    q = np.ascontiguousarray(qblob).view(np.uint8).ravel()
    n_up, n_dn = 2 * I * (d // 32), d * (I // 32)
    meta = (n_up + n_dn + 15) // 16 * 16
    assert d % 32 == 0 and I % 32 == 0 and q.size == meta + 3 * d * I // 2
    scales, codes = q[:n_up + n_dn], q[meta:]
    out = np.empty(3 * d * I, dtype=np.uint16)
    lib = _load()
    lib.ref_dequant_mxfp4_rows(_p(codes[:I * d]), _p(scales[:n_up]), 2 * I, d, _p(out[:2 * I * d]))
    lib.ref_dequant_mxfp4_rows(_p(codes[I * d:]), _p(scales[n_up:]), d, I, _p(out[2 * I * d:]))
    return out
