"""Pins for the oracle of the preprocessing statistics, the predictor's input and ExpertMLP
(Sections IV-A, IV-B).  CPU only."""
import numpy as np
import pytest

import oracle
from oracle import predictor as P
from paper_2509_07379_amd import synth as S


def bf16_bits(a):
    """float array with bf16-representable values -> bit patterns."""
    u = np.asarray(a, dtype=np.float32).view(np.uint32)
    assert np.all((u & 0xFFFF) == 0)
    return (u >> 16).astype(np.uint16)


# ---------------------------------------------------------------- Eq. 2, Eq. 3 on a hand-worked example
TRACE = np.array([[[0, 1], [1, 2]], [[0, 2], [2, 1]], [[1, 0], [0, 1]]])   # 3 episodes, 2 layers, top-2, 3 experts


def test_popularity_hand_example():
    # layer 0 selections {0,1} {0,2} {1,0}: expert 0 three times, 1 twice, 2 once, of 6 selections
    want = np.array([[3, 2, 1], [1, 3, 2]]) / 6.0
    np.testing.assert_allclose(P.popularity(TRACE, 3), want, rtol=0, atol=1e-15)


def test_affinity_hand_example():
    # expert 0 at layer 0 in all three episodes, followed by {1,2} {2,1} {0,1}: j = 0 once, 1 three times, 2 twice
    want = np.array([[[1, 3, 2], [1, 2, 1], [0, 1, 1]]], dtype=np.float64)
    want /= want.sum(axis=2, keepdims=True)
    np.testing.assert_allclose(P.affinity(TRACE, 3), want, rtol=0, atol=1e-15)


def test_statistics_are_distributions_and_follow_the_trace_generator():
    w = S.Workload("stats", d=64, I=64, E=8, k=2, T=1, seed=3, L=6, steps=4000, p_stay=0.6)
    trace = S.markov_trace(w)[:, :, 0, :] if S.markov_trace(w).ndim == 4 else S.markov_trace(w)
    pop, aff = P.popularity(trace, w.E), P.affinity(trace, w.E)
    np.testing.assert_allclose(pop.sum(axis=1), 1.0, atol=1e-12)
    np.testing.assert_allclose(aff.sum(axis=2), 1.0, atol=1e-12)   # every expert occurs in 4000 episodes
    assert np.all(pop >= 0) and np.all(aff >= 0)
    # uniform first layer; a slot keeps its expert with probability 0.6: staying dominates each row
    np.testing.assert_allclose(pop[0], 1.0 / w.E, atol=0.02)
    diag = np.array([[aff[l, i, i] for i in range(w.E)] for l in range(w.L - 1)])
    off = (aff.sum(axis=2) - diag) / (w.E - 1)
    assert diag.min() > 0.3 and diag.min() > 3 * off.max()


def test_never_selected_expert_has_zero_affinity_row():
    tr = np.array([[[0], [1]], [[0], [0]]])
    aff = P.affinity(tr, 3)
    np.testing.assert_array_equal(aff[0, 1], 0.0)
    np.testing.assert_array_equal(aff[0, 2], 0.0)
    np.testing.assert_allclose(aff[0, 0], [0.5, 0.5, 0.0])


# ---------------------------------------------------------------- Eq. 4-5: the state vector
def test_state_vector_layout():
    pop, aff = P.popularity(TRACE, 3), P.affinity(TRACE, 3)
    L, M, k = 2, 3, 2
    assert P.state_dim(L, M, k) == 4 + 3 + 6
    s0 = P.state_vector([], 0, pop, aff, k)
    np.testing.assert_array_equal(s0[:4], 0.0)                      # no history yet
    np.testing.assert_allclose(s0[4:7], pop[0], rtol=1e-7)
    np.testing.assert_array_equal(s0[7:], 0.0)                      # no previous layer
    s1 = P.state_vector([[2, 0]], 1, pop, aff, k)
    np.testing.assert_allclose(s1[:4], [1.0, 1.0 / 3.0, 0, 0], rtol=1e-7)   # ids 2, 0 as (i + 1) / M, then padding
    np.testing.assert_allclose(s1[4:7], pop[1], rtol=1e-7)
    np.testing.assert_allclose(s1[7:10], aff[0, 2], rtol=1e-7)      # rows in the order the ids were recorded
    np.testing.assert_allclose(s1[10:13], aff[0, 0], rtol=1e-7)
    assert s1.dtype == np.float32


# ---------------------------------------------------------------- ExpertMLP forward
def test_mlp_fp64_is_the_matmul_chain():
    dims = [40, 96, 33, 7]
    ws, bs, sc, sh = S.mlp_params(dims, 11)
    s = S.normal_f32((dims[0],), 11, 999, 1.0)
    _, l64 = oracle.mlp_forward(s, ws, bs, sc, sh)
    a = s.astype(np.float64)
    for l in range(3):
        a = S.bf16_to_f32(ws[l]).astype(np.float64) @ a + bs[l]
        if l < 2:
            a = np.maximum(a * sc[l] + sh[l], 0.0)
    np.testing.assert_allclose(l64, a, rtol=1e-13, atol=1e-13)


def test_mlp_structure_on_exact_integers():
    """Small integers: every sum is exact in fp32, so the fixed-order result equals the definition, and
    the layer structure (bias, affine, ReLU, no affine on the last layer) can be checked by hand."""
    w0 = bf16_bits([[1, 2, 0], [-1, 0, 1]])          # 3 -> 2
    w1 = bf16_bits([[1, 1], [2, -3]])                # 2 -> 2 (last)
    s = np.array([1, 2, 3], dtype=np.float32)
    b0, sc0, sh0 = np.array([1, -10], np.float32), np.array([2, 1], np.float32), np.array([-1, 3], np.float32)
    b1 = np.array([0.5, 0.25], np.float32)
    l32, l64 = oracle.mlp_forward(s, [w0, w1], [b0, b1], [sc0], [sh0])
    # layer 0: z = [1+4+1, -1+3-10] = [6, -8]; affine [11, -5]; ReLU [11, 0]; layer 1: [11.5, 22.25]
    np.testing.assert_array_equal(l64, [11.5, 22.25])
    np.testing.assert_array_equal(l32, np.array([11.5, 22.25], np.float32))


def test_mlp_fp32_order_is_the_documented_one():
    """Elements 0 and 64 share a bin: 2^25 + 1 loses the 1 there, and the bin with -2^25 cancels the rest,
    so the fixed order gives 0 where adding the elements in sequence would give 1."""
    n_in = 128
    x = np.zeros(n_in, np.float32)
    x[0], x[1], x[64] = 2.0 ** 25, -(2.0 ** 25), 1.0
    w = bf16_bits(np.ones((1, n_in), np.float32))
    w_last = bf16_bits(np.ones((1, 1), np.float32))
    zero, one = np.zeros(1, np.float32), np.ones(1, np.float32)
    l32, l64 = oracle.mlp_forward(x, [w, w_last], [zero, zero], [one], [zero])
    assert l64[0] == 1.0 and l32[0] == 0.0


def test_mlp_fp32_close_to_fp64_at_full_size():
    dims = S.mlp_dims(32, 8, 2)
    assert dims == [88, 2048, 1024, 512, 256, 128, 64, 64, 8]        # seven hidden layers, 2048 down to 64
    ws, bs, sc, sh = S.mlp_params(dims, 5)
    s = np.abs(S.normal_f32((dims[0],), 5, 998, 0.3))
    l32, l64 = oracle.mlp_forward(s, ws, bs, sc, sh)
    assert np.abs(l32 - l64).max() <= 1e-4 * max(1.0, np.abs(l64).max())
    assert list(oracle.top_m(l32, 3)) == sorted(range(8), key=lambda e: (-l64[e], e))[:3]


def test_top_m_breaks_ties_by_index():
    assert list(oracle.top_m(np.array([1.0, 3.0, 3.0, 2.0]), 3)) == [1, 2, 3]
