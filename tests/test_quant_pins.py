"""Pins for the 8-bit expert format (OCP e4m3 codes, one fp32 scale per output row): the oracle's
decode and expansion against the format's published values and torch's float8_e4m3fn, and the
seeded quantiser (input preparation) against brute force."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2509_07379_amd import synth as S


@pytest.fixture(scope="module", autouse=True)
def _built():
    oracle.build()
    S.build()


def test_e4m3_values_the_format_fixes():
    # OCP 8-bit floating point specification, E4M3: bias 7, max normal 448 = S.1111.110,
    # min normal 2^-6, min subnormal 2^-9, S.1111.111 is NaN, no infinities
    assert oracle.e4m3_value(0x7E) == 448.0
    assert oracle.e4m3_value(0x08) == 2.0 ** -6
    assert oracle.e4m3_value(0x01) == 2.0 ** -9
    assert oracle.e4m3_value(0x38) == 1.0
    assert oracle.e4m3_value(0x00) == 0.0
    assert oracle.e4m3_value(0xC0) == -2.0
    assert math.isnan(oracle.e4m3_value(0x7F)) and math.isnan(oracle.e4m3_value(0xFF))
    vals = [oracle.e4m3_value(c) for c in range(127)]
    assert all(b > a for a, b in zip(vals, vals[1:]))          # codes 0..126 ascend strictly
    assert all(oracle.e4m3_value(c | 0x80) == -v for c, v in enumerate(vals))


def test_e4m3_values_match_torch_float8():
    codes = torch.arange(256, dtype=torch.uint8)
    want = codes.view(torch.float8_e4m3fn).float().numpy()
    got = np.array([oracle.e4m3_value(c) for c in range(256)], dtype=np.float32)
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    np.testing.assert_array_equal(got[ok], want[ok])


def _quantize_rows(w_bf16_bits, rows, cols):
    scales = np.empty(rows, dtype=np.float32)
    q = np.empty(rows * cols, dtype=np.uint8)
    import ctypes
    S._load().synth_quantize_e4m3_rows(ctypes.c_void_p(w_bf16_bits.ctypes.data), rows, cols,
                                       ctypes.c_void_p(scales.ctypes.data), ctypes.c_void_p(q.ctypes.data))
    return scales, q.reshape(rows, cols)


def test_quantiser_picks_the_nearest_code_and_the_row_scale():
    rows, cols = 7, 64
    w = S.normal_bf16((rows * cols,), 3, 11, 0.05)
    w[2 * cols:3 * cols] = 0                                   # an all-zero row: scale 1, codes 0
    scales, q = _quantize_rows(w, rows, cols)
    wf = S.bf16_to_f32(w).reshape(rows, cols)
    table = np.array([oracle.e4m3_value(c) for c in range(127)], dtype=np.float64)
    for r in range(rows):
        amax = np.abs(wf[r]).max()
        assert scales[r] == (np.float32(amax) / np.float32(448.0) if amax > 0 else 1.0)
        x = (wf[r] / scales[r]).astype(np.float32).astype(np.float64)
        for c in range(cols):
            code = int(q[r, c])
            assert (code & 0x7F) != 0x7F
            assert (code >> 7) == (1 if x[c] < 0 else 0)
            dist = np.abs(table - abs(x[c]))
            best = dist.min()
            assert dist[code & 0x7F] == best                   # nearest value
            ties = np.flatnonzero(dist == best)
            if len(ties) > 1:
                assert (code & 1) == 0                         # ties go to the even code
        assert np.abs(q[r] & 0x7F).max() == (0x7E if amax > 0 else 0)   # the row maximum lands on 448


def test_quantiser_agrees_with_torch_float8_rounding():
    rows, cols = 4, 256
    w = S.normal_bf16((rows * cols,), 5, 2, 0.02)
    scales, q = _quantize_rows(w, rows, cols)
    wf = torch.from_numpy(S.bf16_to_f32(w).reshape(rows, cols))
    x = wf / torch.from_numpy(scales)[:, None]
    want = x.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(q, want)


def test_dequant_blob_layout_and_rounding_order():
    d, I = 32, 16
    blob = S.normal_bf16((3 * d * I,), 8, 4, 0.03)
    raw = np.zeros(S.q8_blob_bytes(d, I), dtype=np.uint8)
    S.quantize_blob_into(raw.ctypes.data, blob, d, I)
    got = oracle.dequant_blob(raw, d, I)
    sb = 4 * (2 * I + d)
    scales = torch.from_numpy(raw[:sb].view(np.float32).copy())
    codes = torch.from_numpy(raw[sb:].copy())
    vals = codes.view(torch.float8_e4m3fn).float()
    up = (vals[:2 * I * d].view(2 * I, d) * scales[:2 * I, None]).to(torch.bfloat16)     # fp32 product, then bf16
    down = (vals[2 * I * d:].view(d, I) * scales[2 * I:, None]).to(torch.bfloat16)
    want = torch.cat([up.reshape(-1), down.reshape(-1)]).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(got, want)
    # W_down rows use the LAST d scales: swapping the two scale groups must change the result
    assert not np.array_equal(scales[:d].numpy(), scales[2 * I:2 * I + d].numpy())


def test_dequantised_weights_stay_within_the_format_error_bound():
    d, I = 64, 40
    blob = S.normal_bf16((3 * d * I,), 1, 9, 0.02)
    raw = np.zeros(S.q8_blob_bytes(d, I), dtype=np.uint8)
    S.quantize_blob_into(raw.ctypes.data, blob, d, I)
    a = S.bf16_to_f32(blob).astype(np.float64)
    b = S.bf16_to_f32(oracle.dequant_blob(raw, d, I)).astype(np.float64)
    sb = 4 * (2 * I + d)
    scales = raw[:sb].view(np.float32).astype(np.float64)
    row_scale = np.concatenate([np.repeat(scales[:2 * I], d), np.repeat(scales[2 * I:], I)])
    # 3 mantissa bits: half an ulp is 2^-4 relative for normals, 2^-10 * scale in the subnormal range;
    # the two roundings that follow (fp32 product, bf16) add at most 2^-8 relative
    bound = np.maximum(np.abs(a) * 2.0 ** -4, row_scale * 2.0 ** -10) * (1 + 2.0 ** -7) + np.abs(a) * 2.0 ** -8
    assert np.all(np.abs(a - b) <= bound)
