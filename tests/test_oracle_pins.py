"""Pins of the CPU oracle against things other than itself (no GPU needed).

Every check compares the oracle with a closed form, an invariant the paper states, a
library routine used as an independent definition, or brute force on tiny inputs.
"""
import itertools

import numpy as np
import pytest
import torch
from scipy.special import softmax as sp_softmax

from paper_2509_07379_amd import synth as S


def f32_to_bf16_bits(a):
    """Independent bf16 rounding of fp32 values: PyTorch's CPU conversion (RNE)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bits(vals):
    return f32_to_bf16_bits(np.asarray(vals, dtype=np.float32))


def tiny(E=4, d=32, I=16, T=5, seed=3):
    x = S.normal_bf16((T, d), seed, 1, 1.0)
    wr = S.normal_bf16((E, d), seed, 2, 0.5)
    blobs = [S.normal_bf16((3 * d * I,), seed, 10 + e, 0.3) for e in range(E)]
    return x, wr, blobs


def dense_ffn_f64(x_bits, blob_bits, d, I):
    """Textbook SwiGLU MLP with numpy matmuls in fp64 (h NOT rounded to bf16)."""
    x = S.bf16_to_f32(x_bits).astype(np.float64)
    g, u, dn = (S.bf16_to_f32(m).astype(np.float64) for m in S.split_blob(blob_bits, d, I))
    a = x @ g.T
    h = a / (1.0 + np.exp(-a)) * (x @ u.T)
    return h @ dn.T, h, np.abs(h) @ np.abs(dn).T


# ---------------------------------------------------------------- bf16 rounding
def test_bf16_rounding_matches_library_on_fp32_inputs(oracle):
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * 3,
        (rng.standard_normal(500) * 1e-30).astype(np.float32),
        (rng.standard_normal(500) * 1e30).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 65504.0, 3.3895314e38, 1e-40, -1e-40, 9.18e-41], np.float32),
    ])
    want = f32_to_bf16_bits(vals)
    got = np.array([oracle.bf16_from_f64(float(v)) for v in vals], dtype=np.uint16)
    np.testing.assert_array_equal(got, want)


def test_bf16_rounding_ties_and_no_double_rounding(oracle):
    # spacing of bf16 at 1.0 is 2^-7; halfway cases go to the even significand
    assert oracle.bf16_from_f64(1.0 + 2.0 ** -8) == 0x3F80
    assert oracle.bf16_from_f64(1.0 + 3 * 2.0 ** -8) == 0x3F82
    assert oracle.bf16_from_f64(-(1.0 + 3 * 2.0 ** -8)) == 0xBF82
    # just above a tie: rounding through fp32 first would lose the 2^-40 and tie down
    assert oracle.bf16_from_f64(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81
    assert oracle.bf16_from_f64(1.0 + 2.0 ** -8 - 2.0 ** -40) == 0x3F80
    assert oracle.bf16_from_f64(float("inf")) == 0x7F80
    assert oracle.bf16_from_f64(1e39) == 0x7F80


# ---------------------------------------------------------------- router logits
def test_logits_exact_on_integer_inputs(oracle):
    # small integers: every partial sum is exact in fp32, so any order must give the integer
    rng = np.random.default_rng(1)
    T, E, d = 7, 5, 200  # d not a multiple of 8 or 64: ragged bins
    xi = rng.integers(-4, 5, size=(T, d))
    wi = rng.integers(-4, 5, size=(E, d))
    l32, l64 = oracle.router_logits(bits(xi), bits(wi), want_f64=True)
    want = xi @ wi.T  # token rows x expert rows: pins the operand orientation
    np.testing.assert_array_equal(l32, want.astype(np.float32))
    np.testing.assert_array_equal(l64, want.astype(np.float64))


def test_logits_bias_forms(oracle):
    rng = np.random.default_rng(2)
    T, E, d = 4, 6, 64
    xi, wi = rng.integers(-3, 4, (T, d)), rng.integers(-3, 4, (E, d))
    b1 = rng.integers(-5, 6, E).astype(np.float32)
    b2 = rng.integers(-5, 6, (T, E)).astype(np.float32)
    base = (xi @ wi.T).astype(np.float32)
    np.testing.assert_array_equal(oracle.router_logits(bits(xi), bits(wi), b1), base + b1[None, :])
    np.testing.assert_array_equal(oracle.router_logits(bits(xi), bits(wi), b2), base + b2)


def test_logits_fixed_order_bins(oracle):
    # elements 0 and 512 share bin 0; element 8 is bin 1.  2^24 and -2^24 cancel inside
    # bin 0 before the 1.0 of bin 1 is added; a running sum over i would lose the 1.0.
    d = 1024
    x = np.ones((1, d), np.float32)
    w = np.zeros((1, d), np.float32)
    w[0, 0], w[0, 8], w[0, 512] = 2.0 ** 24, 1.0, -(2.0 ** 24)
    assert oracle.router_logits(bits(x), bits(w))[0, 0] == 1.0
    assert np.float32(np.float32(2.0 ** 24 + 1.0) - 2.0 ** 24) == 0.0  # what a running sum gives


def test_logits_fixed_order_tree(oracle):
    # bins 0 and 32 (elements 0 and 256) are paired at the first tree level, before bin 1
    d = 512
    x = np.ones((1, d), np.float32)
    w = np.zeros((1, d), np.float32)
    w[0, 0], w[0, 8], w[0, 256] = 2.0 ** 24, 1.0, -(2.0 ** 24)
    assert oracle.router_logits(bits(x), bits(w))[0, 0] == 1.0
    # pairing neighbours first (bit 0 first) would give (2^24 + 1) - 2^24 = 0
    w2 = np.zeros((1, d), np.float32)
    w2[0, 0], w2[0, 8], w2[0, 16] = 2.0 ** 24, 1.0, -(2.0 ** 24)  # bins 0,1,2: level bit1 pairs 0&2
    assert oracle.router_logits(bits(x), bits(w2))[0, 0] == 1.0


def test_logits_fp32_close_to_fp64(oracle):
    w = S.WORKLOADS["c1_tiny"]
    x, wr = S.activations(w), S.router_weight(w)
    l32, l64 = oracle.router_logits(x, wr, want_f64=True)
    mag = np.abs(S.bf16_to_f32(x)).astype(np.float64) @ np.abs(S.bf16_to_f32(wr)).astype(np.float64).T
    assert np.all(np.abs(l32 - l64) <= mag * 16 * 2.0 ** -24)
    np.testing.assert_allclose(
        l64, S.bf16_to_f32(x).astype(np.float64) @ S.bf16_to_f32(wr).astype(np.float64).T, rtol=1e-12,
        atol=1e-12)


# ---------------------------------------------------------------- top-k and gate values
@pytest.mark.parametrize("E,k", [(8, 2), (60, 4), (64, 6), (5, 5), (3, 1)])
def test_topk_matches_full_sort(oracle, E, k):
    rng = np.random.default_rng(E * 10 + k)
    logits = rng.standard_normal((200, E)).astype(np.float32)
    logits[:50] = np.round(logits[:50])  # many exact ties
    ids, w = oracle.topk_weights(logits, k)
    for t in range(logits.shape[0]):
        order = np.lexsort((np.arange(E), -logits[t].astype(np.float64)))  # desc logit, asc index
        np.testing.assert_array_equal(ids[t], order[:k])
    assert np.all(w >= 0)
    np.testing.assert_allclose(w.sum(1), 1.0, atol=1e-6)  # gate values sum to 1 (Section II-A)
    sel = np.take_along_axis(logits.astype(np.float64), ids.astype(np.int64), 1)
    np.testing.assert_allclose(w, sp_softmax(sel, axis=1), rtol=2e-7, atol=1e-9)


def test_topk_tie_break_lower_index(oracle):
    logits = np.array([[1.0, 3.0, 3.0, 0.0, 3.0]], np.float32)
    ids, w = oracle.topk_weights(logits, 2)
    np.testing.assert_array_equal(ids, [[1, 2]])
    np.testing.assert_allclose(w, [[0.5, 0.5]])


def test_full_softmax_weights_when_not_renormalised(oracle):
    rng = np.random.default_rng(5)
    logits = rng.standard_normal((30, 8)).astype(np.float32)
    ids, w = oracle.topk_weights(logits, 2, renormalize=False)
    p = sp_softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(w, np.take_along_axis(p, ids.astype(np.int64), 1), rtol=2e-7)
    # renormalising the selected full-softmax values gives the restricted softmax
    _, wr = oracle.topk_weights(logits, 2, renormalize=True)
    np.testing.assert_allclose(w / w.sum(1, keepdims=True), wr, rtol=1e-6)


# ---------------------------------------------------------------- dispatch
@pytest.mark.parametrize("T,k,E", [(64, 2, 8), (333, 6, 64), (8, 4, 60), (1, 2, 8), (50, 3, 3)])
def test_dispatch_invariants(oracle, T, k, E):
    rng = np.random.default_rng(T + k + E)
    ids = np.stack([rng.choice(E, k, replace=False) for _ in range(T)]).astype(np.int32)
    counts, offsets, perm, inv = oracle.dispatch(ids, E)
    flat = ids.reshape(-1)
    np.testing.assert_array_equal(counts, np.bincount(flat, minlength=E))
    assert counts.sum() == T * k
    np.testing.assert_array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    np.testing.assert_array_equal(perm, np.argsort(flat, kind="stable"))  # library stable sort
    np.testing.assert_array_equal(inv[perm], np.arange(T * k))
    np.testing.assert_array_equal(perm[inv], np.arange(T * k))
    tok = np.sort(perm // k)
    np.testing.assert_array_equal(tok, np.repeat(np.arange(T), k))  # every token exactly k times
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e)
        assert np.all(np.diff(seg) > 0)  # stability


def test_dispatch_with_empty_experts(oracle):
    ids = np.array([[5, 2], [2, 5], [5, 7]], np.int32)
    counts, offsets, perm, inv = oracle.dispatch(ids, 9)
    np.testing.assert_array_equal(counts, [0, 0, 2, 0, 0, 3, 0, 1, 0])
    np.testing.assert_array_equal(perm, [1, 2, 0, 3, 4, 5])


# ---------------------------------------------------------------- expert FFN and combine
def test_single_expert_is_plain_swiglu_mlp(oracle):
    d, I = 48, 40
    x, _, blobs = tiny(E=1, d=d, I=I, T=6)
    want, h, mag = dense_ffn_f64(x, blobs[0], d, I)
    for t in range(x.shape[0]):
        y = oracle.expert_ffn(x[t], blobs[0], d, I)
        # only difference allowed: h rounded to bf16 (relative error at most 2^-8 per element)
        assert np.all(np.abs(y - want[t]) <= mag[t] * 2.0 ** -8 + 1e-12)
        assert np.abs(y - want[t]).max() > 0  # the rounding of h is really there
    # E = 1, k = 1: the layer is that MLP with weight exactly 1
    r = oracle.moe_layer(x, S.normal_bf16((1, d), 0, 99, 1.0), blobs, 1)
    assert np.all(r["w"] == 1.0) and np.all(r["ids"] == 0)
    assert np.all(np.abs(r["out_f64"] - want) <= mag * 2.0 ** -8 + 1e-12)


def test_expert_exact_when_h_is_representable(oracle):
    # gate pre-activation 0 => silu(0) = 0 => h = 0 => y = 0 exactly; and with integer h the
    # down projection is an exact integer matmul: pins W_down's [d, I] orientation.
    d, I = 16, 8
    rng = np.random.default_rng(7)
    x = bits(rng.integers(-2, 3, (1, d)))
    wg = np.zeros((I, d), np.float32)
    blob = np.concatenate([bits(wg).ravel(), bits(rng.integers(-2, 3, (I, d))).ravel(),
                           bits(rng.integers(-2, 3, (d, I))).ravel()])
    np.testing.assert_array_equal(oracle.expert_ffn(x[0], blob, d, I), np.zeros(d))


def test_topk_equal_E_is_dense_mixture(oracle):
    # k = E: every expert contributes with its full-softmax gate value (textbook MoE)
    E, d, I, T = 4, 32, 16, 5
    x, wr, blobs = tiny(E, d, I, T)
    r = oracle.moe_layer(x, wr, blobs, E)
    logits = S.bf16_to_f32(x).astype(np.float64) @ S.bf16_to_f32(wr).astype(np.float64).T
    p = sp_softmax(logits, axis=1)
    want = np.zeros((T, d))
    bound = np.zeros((T, d))
    for e in range(E):
        y, _, mag = dense_ffn_f64(x, blobs[e], d, I)
        want += p[:, e:e + 1] * y
        bound += p[:, e:e + 1] * mag
    assert np.all(np.abs(r["out_f64"] - want) <= bound * 2.0 ** -8 + 1e-5 * np.abs(want) + 1e-9)
    # and the bf16 output is the rounding of the fp64 one
    np.testing.assert_array_equal(r["out"], f32_to_bf16_bits(r["out_f64"].astype(np.float32)))


def test_brute_force_topk_layer(oracle):
    # brute force over all k-subsets: the chosen subset maximises the summed logits, and the
    # output is the restricted-softmax mixture of exactly those experts
    E, d, I, T, k = 5, 32, 16, 6, 2
    x, wr, blobs = tiny(E, d, I, T, seed=11)
    r = oracle.moe_layer(x, wr, blobs, k)
    logits = S.bf16_to_f32(x).astype(np.float64) @ S.bf16_to_f32(wr).astype(np.float64).T
    ys = [dense_ffn_f64(x, blobs[e], d, I) for e in range(E)]
    for t in range(T):
        best = max(itertools.combinations(range(E), k), key=lambda c: sum(logits[t, list(c)]))
        assert set(r["ids"][t]) == set(best)
        assert logits[t, r["ids"][t, 0]] >= logits[t, r["ids"][t, 1]]
        sel = list(r["ids"][t])
        p = sp_softmax(logits[t, sel])
        want = sum(p[j] * ys[sel[j]][0][t] for j in range(k))
        bound = sum(p[j] * ys[sel[j]][2][t] for j in range(k))
        assert np.all(np.abs(r["out_f64"][t] - want) <= bound * 2.0 ** -8 + 1e-5 * np.abs(want) + 1e-9)


def test_shared_two_experts_equal_one_fused(oracle):
    # two always-on shared experts of width I_s == one expert of width 2*I_s whose W_gate/W_up
    # rows and W_down columns are concatenated
    E, d, I, T, k, Is = 4, 32, 16, 4, 2, 24
    x, wr, blobs = tiny(E, d, I, T, seed=5)
    s1 = S.normal_bf16((3 * d * Is,), 5, 50, 0.3)
    s2 = S.normal_bf16((3 * d * Is,), 5, 51, 0.3)
    g1, u1, d1 = S.split_blob(s1, d, Is)
    g2, u2, d2 = S.split_blob(s2, d, Is)
    fused = np.concatenate([np.concatenate([g1, g2]).ravel(), np.concatenate([u1, u2]).ravel(),
                            np.concatenate([d1, d2], axis=1).ravel()])
    r0 = oracle.moe_layer(x, wr, blobs, k)
    rf = oracle.moe_layer(x, wr, blobs, k, shared_blob=fused, I_shared=2 * Is)
    want = r0["out_f64"].copy()
    for t in range(T):
        want[t] += oracle.expert_ffn(x[t], s1, d, Is) + oracle.expert_ffn(x[t], s2, d, Is)
    np.testing.assert_allclose(rf["out_f64"], want, rtol=1e-12, atol=1e-12)
    assert np.abs(rf["out_f64"] - r0["out_f64"]).max() > 1e-3  # shared part is really added


def test_linearity_in_gate_values_and_relabelling(oracle):
    E, d, I, T, k = 6, 32, 16, 7, 3
    x, wr, blobs = tiny(E, d, I, T, seed=9)
    r = oracle.moe_layer(x, wr, blobs, k)
    _, o2 = oracle.moe_tokens(x, blobs, r["ids"], 2.0 * r["w"])
    np.testing.assert_allclose(o2, 2.0 * r["out_f64"], rtol=1e-12)
    # store the experts in another order and relabel the router rows: same output
    p = np.array([3, 0, 5, 1, 4, 2])
    r2 = oracle.moe_layer(x, wr[p], [blobs[i] for i in p], k)
    np.testing.assert_array_equal(p[r2["ids"]], r["ids"])
    np.testing.assert_allclose(r2["out_f64"], r["out_f64"], rtol=1e-12, atol=1e-15)


def test_selected_tokens_subset(oracle):
    E, d, I, T, k = 4, 32, 16, 9, 2
    x, wr, blobs = tiny(E, d, I, T, seed=13)
    full = oracle.moe_layer(x, wr, blobs, k)
    sel = np.array([7, 0, 3], np.int32)
    part = oracle.moe_layer(x, wr, blobs, k, sel=sel)
    np.testing.assert_array_equal(part["out"], full["out"][sel])


# ---------------------------------------------------------------- predictor stand-in
def test_predictor_topm(oracle):
    rng = np.random.default_rng(3)
    B, d, E, m = 3, 96, 10, 4
    xi, wi = rng.integers(-3, 4, (B, d)), rng.integers(-3, 4, (E, d))
    scores, top = oracle.predictor_score(bits(xi), bits(wi), m)
    want = (xi @ wi.T).sum(0)
    np.testing.assert_array_equal(scores, want.astype(np.float32))
    np.testing.assert_array_equal(top, np.lexsort((np.arange(E), -want))[:m])


# ---------------------------------------------------------------- stored digest of config 1
def test_c1_golden_digest(oracle):
    import json
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "c1_tiny_oracle.json")
    g = json.load(open(path))
    w = S.WORKLOADS["c1_tiny"]
    r = oracle.moe_layer(S.activations(w), S.router_weight(w),
                         [S.expert_blob(w, 0, e) for e in range(w.E)], w.k)
    assert r["counts"].tolist() == g["counts"]
    assert r["ids"][:8].tolist() == g["ids_first8"]
    assert r["out"][:2, :8].tolist() == g["out_bits_first"]
    assert int(r["out"].astype(np.uint64).sum()) == g["out_bits_sum"]
