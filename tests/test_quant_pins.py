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


# ---------------------------------------------------------------- 4-bit integers, groups of 128
def test_int4_dequant_by_hand():
    """One row of 256 columns = two groups.  Group 0: scale 0.5, zero 8, codes 0..15 repeating -> values
    (code - 8) / 2; group 1: scale 0.25, zero 0.  Two codes per byte, the even column in the low nibble."""
    import ctypes
    cols = 256
    code = np.arange(cols) % 16
    packed = (code[0::2] | (code[1::2] << 4)).astype(np.uint8)
    scales = np.array([0.5, 0.25], dtype=np.float32)
    zeros = np.array([8, 0], dtype=np.uint8)
    out = np.empty(cols, dtype=np.uint16)
    vp = lambda a: ctypes.c_void_p(a.ctypes.data)
    oracle._load().ref_dequant_int4_g128_rows(vp(packed), vp(scales), vp(zeros), 1, cols, vp(out))
    got = S.bf16_to_f32(out)
    want = np.concatenate([(code[:128] - 8) * 0.5, code[128:] * 0.25]).astype(np.float32)
    np.testing.assert_array_equal(got, want)
    assert got[1] == -3.5 and got[0] == -4.0          # column 1 came from the HIGH nibble of byte 0


def test_int4_blob_layout_and_rounding_against_torch():
    d, I = 256, 128
    blob = S.normal_bf16((3 * d * I,), 8, 4, 0.03)
    raw = np.zeros(S.q4_blob_bytes(d, I), dtype=np.uint8)
    S.quantize4_blob_into(raw.ctypes.data, blob, d, I)
    got = oracle.dequant4_blob(raw, d, I)
    lay = S.q4_layout(d, I)
    n_up, n_dn = 2 * I * (d // 128), d * (I // 128)

    def expand(codes_off, rows, cols, scales_off, zeros_off, n):
        b = torch.from_numpy(raw[codes_off:codes_off + rows * cols // 2].astype(np.int32))
        q = torch.stack([b & 15, b >> 4], dim=1).reshape(rows, cols)          # even column = low nibble
        s = torch.from_numpy(raw[scales_off:scales_off + 4 * n].view(np.float32).copy()).reshape(rows, cols // 128)
        z = torch.from_numpy(raw[zeros_off:zeros_off + n].astype(np.int32)).reshape(rows, cols // 128)
        val = (q - z.repeat_interleave(128, dim=1)).float() * s.repeat_interleave(128, dim=1)   # fp32 product
        return val.to(torch.bfloat16).reshape(-1)

    up = expand(lay["codes_up"], 2 * I, d, lay["scales_up"], lay["zeros_up"], n_up)
    down = expand(lay["codes_down"], d, I, lay["scales_down"], lay["zeros_down"], n_dn)
    want = torch.cat([up, down]).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(got, want)


def test_int4_quantiser_error_bound_and_exact_zero():
    d, I = 128, 256
    blob = S.normal_bf16((3 * d * I,), 2, 7, 0.02)
    blob[5:40] = 0                                               # zero weights must come back as zero
    raw = np.zeros(S.q4_blob_bytes(d, I), dtype=np.uint8)
    S.quantize4_blob_into(raw.ctypes.data, blob, d, I)
    a = S.bf16_to_f32(blob).astype(np.float64)
    b = S.bf16_to_f32(oracle.dequant4_blob(raw, d, I)).astype(np.float64)
    assert np.all(b[5:40] == 0.0)
    lay = S.q4_layout(d, I)
    n_up, n_dn = 2 * I * (d // 128), d * (I // 128)
    scales = raw[:4 * (n_up + n_dn)].view(np.float32).astype(np.float64)
    per_w = np.concatenate([np.repeat(scales[:n_up], 128), np.repeat(scales[n_up:], 128)])
    # round-to-nearest on a grid of step `scale` that covers [min, max] up to the zero point's own rounding
    # (half a step more at the ends); the fp32 and bf16 roundings add 2^-8 relative
    assert np.all(np.abs(a - b) <= per_w * 1.0 + np.abs(a) * 2.0 ** -7)
    assert np.sqrt(np.mean((a - b) ** 2)) < 0.4 * np.mean(per_w)   # typical error is step / sqrt(12)
    assert lay["total"] == raw.size and lay["meta"] % 16 == 0


# ---------------------------------------------------------------- MXFP4 (e2m1 codes, blocks of 32, 2^k scales)
def test_e2m1_values_the_format_fixes():
    # OCP microscaling formats, FP4 E2M1: exponent bias 1, max normal 6.0 = S.11.1, min normal 1.0, subnormal 0.5
    want = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    assert [oracle.e2m1_value(c) for c in range(8)] == want
    assert [oracle.e2m1_value(8 + c) for c in range(1, 8)] == [-v for v in want[1:]]
    assert math.copysign(1.0, oracle.e2m1_value(8)) == -1.0 and oracle.e2m1_value(8) == 0.0   # negative zero


def test_mxfp4_dequant_by_hand_and_exactness():
    """One row of 64 columns = two blocks: scale bytes 128 (x 2) and 120 (x 2^-7); codes 0..15 repeating.
    Every product is one mantissa bit times a power of two: exact in bf16, no rounding anywhere."""
    import ctypes
    cols = 64
    code = np.arange(cols) % 16
    packed = (code[0::2] | (code[1::2] << 4)).astype(np.uint8)
    scales = np.array([128, 120], dtype=np.uint8)
    out = np.empty(cols, dtype=np.uint16)
    vp = lambda a: ctypes.c_void_p(a.ctypes.data)
    oracle._load().ref_dequant_mxfp4_rows(vp(packed), vp(scales), 1, cols, vp(out))
    table = np.array([0, .5, 1, 1.5, 2, 3, 4, 6, -0.0, -.5, -1, -1.5, -2, -3, -4, -6])
    want = table[code] * np.repeat([2.0, 2.0 ** -7], 32)
    got = S.bf16_to_f32(out).astype(np.float64)
    np.testing.assert_array_equal(got, want)                     # exact, not "close"
    assert got[1] == 1.0 and got[2] == 2.0                       # column 1 = high nibble of byte 0: 0.5 * 2
    assert out[8] == 0x8000                                      # code 8 stays a negative zero


def test_mxfp4_blob_layout_against_numpy():
    d, I = 128, 96
    blob = S.normal_bf16((3 * d * I,), 8, 4, 0.03)
    raw = np.zeros(S.mx4_blob_bytes(d, I), dtype=np.uint8)
    S.quantize_mx4_blob_into(raw.ctypes.data, blob, d, I)
    got = S.bf16_to_f32(oracle.dequant_mx4_blob(raw, d, I)).astype(np.float64)
    lay = S.mx4_layout(d, I)
    table = np.array([0, .5, 1, 1.5, 2, 3, 4, 6, -0.0, -.5, -1, -1.5, -2, -3, -4, -6])

    def expand(codes_off, rows, cols, scales_off):
        b = raw[codes_off:codes_off + rows * cols // 2].astype(np.int64)
        q = np.stack([b & 15, b >> 4], axis=1).reshape(rows, cols)
        s = raw[scales_off:scales_off + rows * cols // 32].astype(np.float64).reshape(rows, cols // 32)
        return (table[q] * np.repeat(2.0 ** (s - 127), 32, axis=1)).ravel()

    want = np.concatenate([expand(lay["codes_up"], 2 * I, d, lay["scales_up"]),
                           expand(lay["codes_down"], d, I, lay["scales_down"])])
    np.testing.assert_array_equal(got, want)


def test_mxfp4_quantiser_scale_rule_and_nearest_code():
    rows, cols = 3, 128
    w = S.normal_bf16((rows * cols,), 4, 6, 0.05)
    w[40:72] = 0                                                   # an all-zero block
    import ctypes
    scales = np.empty(rows * cols // 32, dtype=np.uint8)
    codes = np.empty(rows * cols // 2, dtype=np.uint8)
    vp = lambda a: ctypes.c_void_p(a.ctypes.data)
    S._load().synth_quantize_mxfp4(vp(w), rows, cols, vp(scales), vp(codes))
    wf = S.bf16_to_f32(w).astype(np.float64).reshape(-1, 32)
    q = np.stack([codes & 15, codes >> 4], axis=1).reshape(-1, 32)
    table = np.array([0, .5, 1, 1.5, 2, 3, 4, 6])
    for blk in range(wf.shape[0]):
        amax = np.abs(wf[blk]).max()
        if amax == 0:
            assert scales[blk] == 127 and np.all((q[blk] & 7) == 0)
            continue
        assert int(scales[blk]) - 127 == math.floor(math.log2(amax)) - 2      # the block maximum lands in [4, 8) -> code 6 or 7
        x = np.abs(wf[blk]) / 2.0 ** (int(scales[blk]) - 127)
        for i in range(32):
            dist = np.abs(table - x[i])
            assert dist[q[blk, i] & 7] == dist.min()
            assert (q[blk, i] >> 3) == (1 if wf[blk, i] < 0 else 0)
        assert (q[blk] & 7).max() >= 6
