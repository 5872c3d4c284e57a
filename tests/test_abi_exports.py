"""The C-ABI library loads without a GPU and exports every function the header declares."""
import pytest
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "moe_offload.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:int|size_t|const char \*)\s*\*?\s*(\w+)\s*\(", text)
    return sorted(set(n for n in names if n.startswith(("moe_", "expert_cache_", "predictor_"))))


def test_header_functions_are_exported():
    from paper_2509_07379_amd import binding
    assert os.path.exists(binding.LIB_PATH), "build first: python -m paper_2509_07379_amd.build"
    lib = ctypes.CDLL(binding.LIB_PATH)
    names = declared_functions()
    assert {"moe_prefill_layer", "moe_decode_layer", "expert_cache_prefetch", "predictor_score"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_internal_hooks_are_declared_apart_from_the_public_header():
    from paper_2509_07379_amd import binding
    lib = ctypes.CDLL(binding.LIB_PATH)
    text = open(os.path.join(ROOT, "paper_2509_07379_amd", "csrc", "moe_tuning.h")).read()
    public = declared_functions()
    for n in binding.INTERNAL_EXPORTS:
        assert hasattr(lib, n) and re.search(r"\b%s\s*\(" % n, text) and n not in public, n


def test_limits_of_the_argument_block_are_refused_at_create():
    """A slot index travels to the kernels in 16 bits and the gate stages token vectors in LDS: a cache
    of more slots, or a wider hidden size, is refused before any HIP call (so this runs without a GPU)."""
    from paper_2509_07379_amd import binding
    lib = binding.load()
    h = ctypes.c_void_p()
    for cfg, word in ((binding.MoeConfig(256, 128, 8, 2, 28, 40000, 0, 1, 1, 0), b"cache_slots"),
                      (binding.MoeConfig(16392, 128, 8, 2, 1, 8, 0, 1, 0, 0), b"d = 16392")):
        assert lib.moe_create(ctypes.byref(cfg), ctypes.byref(h)) == -2
        assert word in lib.moe_last_error()
        assert lib.moe_workspace_bytes(ctypes.byref(cfg), 4) == 0


def test_gemm_kernel_choice_keeps_31_bit_offsets_in_reach():
    """The ping-pong kernel (12) addresses a gathered activation matrix with 31-bit byte offsets from its
    first row: every row the permutation can name must be in reach, however few rows one group has."""
    from paper_2509_07379_amd import binding
    lib = binding.load()
    d, I = 4096, 14336
    pick = lambda mode, gathered, a_rows, lda, N, ldb, K, gap, rows, groups: lib.moe_debug_gemm_choice(
        mode, gathered, a_rows, lda, N, ldb, K, gap, rows, groups)
    # gate/up GEMM of one expert with 600 rows out of T tokens
    assert pick(0, 1, 2048, d, I, d, d, 2 * I * d, 600, 1) == 12
    assert pick(0, 1, 262143, d, I, d, d, 2 * I * d, 600, 1) == 12      # (T - 1) * d * 2 < 2^31
    assert pick(0, 1, 262144, d, I, d, d, 2 * I * d, 600, 1) == 6       # one more token: out of reach
    assert pick(0, 1, 1 << 22, d, I, d, d, 2 * I * d, 600, 1) == 6
    # the down GEMM reads H in place, tile by tile: any number of rows
    assert pick(1, 0, 1 << 22, I, d, I, I, 0, 600, 1) == 12
    # small groups take the 128 x 128 tiles, a ragged K the padding kernel
    assert pick(0, 1, 2048, d, I, d, d, 2 * I * d, 600, 60) == 1
    assert pick(1, 0, 2048, 1000, 512, 1000, 1000, 0, 600, 1) == 100


def test_argument_errors_without_gpu():
    from paper_2509_07379_amd import binding
    lib = binding.load()
    cfg = binding.MoeConfig(256, 128, 8, 9, 1, 8, 0, 1)  # k > E: rejected before any HIP call
    h = ctypes.c_void_p()
    assert lib.moe_create(ctypes.byref(cfg), ctypes.byref(h)) == -1
    assert b"exceeds" in lib.moe_last_error()
    assert lib.moe_workspace_bytes(ctypes.byref(cfg), 4) == 0
    ok = binding.MoeConfig(4096, 14336, 8, 2, 1, 2, 0, 1)
    assert lib.moe_workspace_bytes(ctypes.byref(ok), 2048) > 2048 * 2 * 14336 * 2


def test_state_constructor_matches_the_oracle():
    """Host-only bookkeeping (no GPU call): the predictor's input vector, Eq. 4-5."""
    import numpy as np
    import torch
    from oracle import predictor as P
    from paper_2509_07379_amd import binding, synth as S
    w = S.Workload("state", d=64, I=64, E=8, k=2, T=1, seed=9, L=5, steps=300, p_stay=0.6)
    trace = S.markov_trace(w)
    trace = trace[:, :, 0, :] if trace.ndim == 4 else trace
    pop, aff = P.popularity(trace, w.E), P.affinity(trace, w.E)
    st = binding.MoeState(w.L, w.E, w.k, pop, aff)
    dim = st.moe_state_dim()
    assert dim == P.state_dim(w.L, w.E, w.k)
    out = torch.zeros(dim, dtype=torch.float32)
    pop32, aff32 = pop.astype(np.float32).astype(np.float64), aff.astype(np.float32).astype(np.float64)
    for episode in (3, 17):
        st.moe_state_clear()
        with pytest.raises(binding.MoeError):
            st.moe_state_vector(1, out)              # layer 0 not recorded yet in this decode step
        history = []
        for l in range(w.L):
            st.moe_state_vector(l, out)
            want = P.state_vector(history, l, pop32, aff32, w.k)
            np.testing.assert_array_equal(out.numpy(), want)
            st.moe_state_record(l, trace[episode, l])
            history.append(list(trace[episode, l]))
    with pytest.raises(binding.MoeError):
        st.moe_state_record(0, [0, w.E])             # id out of range
    st.close()


def test_blob_and_cache_sizes_per_host_format():
    """Sizes the caller allocates by (no GPU call): the library's figures equal the layouts the seeded
    quantisers write, and unknown or unsupported formats are refused."""
    import ctypes as C
    from paper_2509_07379_amd import binding, synth as S
    lib = binding.load()
    d, I, slots = 256, 384, 3
    for fmt, want in ((0, 6 * d * I), (1, S.q8_blob_bytes(d, I)), (2, S.q4_blob_bytes(d, I)), (3, S.mx4_blob_bytes(d, I))):
        cfg = binding.MoeConfig(d, I, 8, 2, 1, slots, 0, 1, 0, fmt)
        assert lib.moe_host_blob_bytes(C.byref(cfg)) == want
        stage = 0 if fmt == 0 else (want + 255) // 256 * 256
        bf16_slot = 0 if fmt in (1, 3) else 6 * d * I      # an e4m3 or MXFP4 cache holds the quantised blobs and nothing else
        assert lib.moe_cache_bytes(C.byref(cfg)) == slots * (bf16_slot + stage)
    assert lib.moe_host_blob_bytes(C.byref(binding.MoeConfig(d, I, 8, 2, 1, slots, 0, 1, 0, 4))) == 0
    assert b"not a known format" in lib.moe_last_error()
    assert lib.moe_host_blob_bytes(C.byref(binding.MoeConfig(264, I, 8, 2, 1, slots, 0, 1, 0, 2))) == 0
    assert b"multiples of 128" in lib.moe_last_error()
    for fmt in (1, 3):
        assert lib.moe_host_blob_bytes(C.byref(binding.MoeConfig(d, 136, 8, 2, 1, slots, 0, 1, 0, fmt))) == 0
        assert b"multiples of 64" in lib.moe_last_error()
