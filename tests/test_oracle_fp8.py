"""Pins for the 8-bit KV oracle (oracle_fp8.c).

The paper leaves the cache's number format open; this variant stores it as OCP E4M3 codes with
one scale per tensor.  What can go wrong is a wrong decode table, a wrong rounding rule, a scale
applied on the wrong side or to the wrong tensor, and a wrong placement of appended rows.  Each
pin below gets its expected values from somewhere other than oracle_fp8.c: the format's published
constants and structure, PyTorch's own float8_e4m3fn type, exact rationals, oracle.c (already
pinned) on a cache that holds the same values in bf16, and plain Python loops."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from workloads import gen

ALL = np.arange(256, dtype=np.uint8)
FINITE_POS = np.arange(0, 0x7F, dtype=np.uint8)          # 0x00 .. 0x7e


def test_decode_constants_of_the_format():
    v = oracle.e4m3_decode(ALL)
    assert v[0x00] == 0.0 and not np.signbit(v[0x00])
    assert v[0x80] == 0.0 and np.signbit(v[0x80])
    assert v[0x01] == 2.0 ** -9                          # smallest subnormal
    assert v[0x07] == 0.875 * 2.0 ** -6                  # largest subnormal
    assert v[0x08] == 2.0 ** -6                          # smallest normal
    assert v[0x38] == 1.0
    assert v[0x7E] == 448.0                              # largest finite
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF])       # the only NaNs; no infinities
    assert np.isfinite(np.delete(v, [0x7F, 0xFF])).all()


def test_decode_structure_fixes_every_other_code():
    v = oracle.e4m3_decode(ALL)
    pos = v[:0x7F]
    assert (np.diff(pos) > 0).all()                      # strictly increasing in the code
    np.testing.assert_array_equal(v[0x80:0xFF], -pos)    # sign bit only flips the sign
    np.testing.assert_array_equal(pos[16:0x7F], 2.0 * pos[8:0x77])   # exponent field + 1 doubles
    for e in range(16):                                  # eight equal steps inside each binade
        seg = v[8 * e: min(8 * e + 9, 0x7F)]
        assert len(set(np.diff(seg))) == 1
    np.testing.assert_array_equal(pos[:9], np.arange(9) * 2.0 ** -9)  # subnormals: multiples of 2^-9


def test_decode_equals_the_library_type():
    lib = torch.from_numpy(ALL.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    v = oracle.e4m3_decode(ALL)
    np.testing.assert_array_equal(np.isnan(v), np.isnan(lib))
    ok = ~np.isnan(v)
    np.testing.assert_array_equal(v[ok], lib[ok])
    np.testing.assert_array_equal(np.signbit(v[ok]), np.signbit(lib[ok]))


def test_every_finite_code_is_a_fixed_point_of_rounding():
    codes = np.concatenate([FINITE_POS, FINITE_POS | np.uint8(0x80)])
    vals = oracle.e4m3_decode(codes).astype(np.float32)
    np.testing.assert_array_equal(oracle.e4m3_from_float(vals), codes)


def test_midpoints_go_to_the_even_code_and_their_neighbours_to_the_nearer_one():
    v = oracle.e4m3_decode(FINITE_POS)
    for c in range(0, 0x7E):
        mid = Fraction(v[c]) + (Fraction(v[c + 1]) - Fraction(v[c])) / 2
        m32 = np.float32(float(mid))
        assert Fraction(float(m32)) == mid               # midpoints are exact in fp32
        even = c if c % 2 == 0 else c + 1
        below, above = np.nextafter(m32, np.float32(0)), np.nextafter(m32, np.float32(1e9))
        got = oracle.e4m3_from_float(np.asarray([m32, below, above, -m32, -below, -above], dtype=np.float32))
        np.testing.assert_array_equal(got, [even, c, c + 1, even | 0x80, c | 0x80, (c + 1) | 0x80])


def test_saturation_nan_and_zero_signs():
    y = np.asarray([448.0, 449.0, 464.0, 465.0, 1e30, np.inf, -448.5, -np.inf, 0.0, -0.0,
                    2.0 ** -10, 2.0 ** -11, -(2.0 ** -11)], dtype=np.float32)
    got = oracle.e4m3_from_float(y)
    np.testing.assert_array_equal(got, [0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0xFE, 0x00, 0x80,
                                        0x00, 0x00, 0x80])           # 2^-10 ties to the even code 0
    assert oracle.e4m3_from_float(np.asarray([np.nan], dtype=np.float32))[0] & 0x7F == 0x7F
    up = np.nextafter(np.float32(2.0 ** -10), np.float32(1))
    assert oracle.e4m3_from_float(np.asarray([up], dtype=np.float32))[0] == 0x01


def test_rounding_equals_the_library_cast_inside_the_finite_range():
    rng = np.random.default_rng(5)
    y = np.concatenate([rng.standard_normal(200000) * 3.0, rng.standard_normal(50000) * 0.01,
                        rng.uniform(-463.9, 463.9, 50000)]).astype(np.float32)
    lib = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(oracle.e4m3_from_float(y), lib)


@pytest.mark.parametrize("scale", [1.0, 0.5, 0.37, 3.0e-3, 17.25])
def test_quantize_divides_by_the_scale_in_fp32_then_rounds(scale):
    x = gen.normal_bf16(901, 1, (40000,))
    xf = gen.bf16_bits_to_f32(x)
    y = (xf / np.float32(scale)).astype(np.float32)                  # numpy's IEEE fp32 division
    lib = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = oracle.e4m3_quantize(x, scale)
    inside = np.abs(y) < 464.0
    np.testing.assert_array_equal(got[inside], lib[inside])
    np.testing.assert_array_equal(got[~inside] & 0x7F, 0x7E)         # saturated, never NaN
    # the dequantised value is within half a step of the input: step <= |x|/8 for normals
    back = oracle.e4m3_decode(got) * scale
    ok = inside & (np.abs(y) >= 2.0 ** -6)
    assert (np.abs(back[ok] - xf[ok]) <= np.abs(xf[ok]) / 16 * (1 + 1e-6)).all()


def test_quantize_is_a_division_not_a_multiplication_by_the_reciprocal():
    """All finite bf16 inputs against several scales, one of them (the fp32 just below 7) chosen
    because there the two ways of scaling land on different codes for some inputs: the oracle
    sides with the division."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    xf = gen.bf16_bits_to_f32(bits)
    bits = bits[np.isfinite(xf)]
    xf = xf[np.isfinite(xf)]
    differing = 0
    for scale in (3.0, 0.37, 0.011, float(np.nextafter(np.float32(7.0), np.float32(0.0)))):
        s32 = np.float32(scale)
        with np.errstate(over="ignore"):
            y_div = (xf / s32).astype(np.float32)
            y_mul = (xf * (np.float32(1.0) / s32)).astype(np.float32)
        inside = (np.abs(y_div) < 464.0) & (np.abs(y_mul) < 464.0)
        c_div = torch.from_numpy(y_div).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        c_mul = torch.from_numpy(y_mul).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        got = oracle.e4m3_quantize(bits, scale)
        np.testing.assert_array_equal(got[inside], c_div[inside])
        differing += int((c_div[inside] != c_mul[inside]).sum())
    assert differing > 0


def _codes_as_bf16(codes):
    """Every E4M3 value is a bf16 value: widen exactly (checked), return the bf16 bits."""
    v = oracle.e4m3_decode(codes)
    bits = gen.f32_to_bf16_bits(v.astype(np.float32))
    np.testing.assert_array_equal(gen.bf16_bits_to_f32(bits).astype(np.float64), v)
    return bits


SEGS = [(1, 1), (1, 37), (5, 5), (19, 50), (1, 130), (33, 64)]


@pytest.mark.parametrize("Hq,Hkv,D", [(4, 1, 64), (8, 2, 128)])
def test_attention_equals_the_bf16_oracle_on_the_widened_cache(Hq, Hkv, D):
    b = gen.make_batch_fp8kv("f8a", 311, Hq, Hkv, D, SEGS, k_scale=1.0, v_scale=1.0)
    got = oracle.attn_mixed_batch_fp8kv(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets,
                                        b.ctx_lens, b.scale, 1.0, 1.0)
    ref = oracle.attn_mixed_batch(b.q, _codes_as_bf16(b.k_pool), _codes_as_bf16(b.v_pool),
                                  b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_power_of_two_scales_equal_the_bf16_oracle_on_scaled_values():
    b = gen.make_batch_fp8kv("f8b", 312, 4, 2, 64, SEGS)
    ks, vs = 0.25, 8.0
    kb = gen.f32_to_bf16_bits((oracle.e4m3_decode(b.k_pool) * ks).astype(np.float32))   # exact
    vb = gen.f32_to_bf16_bits((oracle.e4m3_decode(b.v_pool) * vs).astype(np.float32))
    got = oracle.attn_mixed_batch_fp8kv(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets,
                                        b.ctx_lens, b.scale, ks, vs)
    ref = oracle.attn_mixed_batch(b.q, kb, vb, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-11)


def test_k_scale_acts_on_the_scores_and_v_scale_on_the_output():
    b = gen.make_batch_fp8kv("f8c", 313, 4, 1, 64, SEGS)
    args = (b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens)
    base = oracle.attn_mixed_batch_fp8kv(*args, b.scale, 0.37, 1.0)
    folded = oracle.attn_mixed_batch_fp8kv(*args, b.scale * 0.37, 1.0, 1.0)
    np.testing.assert_allclose(base, folded, rtol=0, atol=1e-12)
    scaled = oracle.attn_mixed_batch_fp8kv(*args, b.scale, 0.37, 2.5)
    np.testing.assert_allclose(scaled, 2.5 * base, rtol=0, atol=1e-12)
    # the two scales are not interchangeable: swapping them changes the result
    swapped = oracle.attn_mixed_batch_fp8kv(*args, b.scale, 2.5, 0.37)
    assert np.abs(swapped - scaled).max() > 1e-3


def test_selected_rows_equal_the_same_rows_of_the_whole_batch():
    b = gen.make_batch_fp8kv("f8d", 314, 4, 2, 64, SEGS)
    args = (b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale, 0.5, 0.5)
    full = oracle.attn_mixed_batch_fp8kv(*args)
    rows = np.asarray([(3, 18, 1), (0, 0, 3), (5, 7, 2), (4, 0, 0)], dtype=np.int32)
    sel = oracle.attn_rows_fp8kv(*args, rows)
    for r, (i, j, h) in enumerate(rows):
        np.testing.assert_array_equal(sel[r], full[b.q_offsets[i] + j, h])


def test_append_quantises_and_places_rows_like_a_python_loop():
    b = gen.make_batch_fp8kv("f8e", 315, 4, 2, 64, [(7, 30), (1, 1), (20, 21), (1, 40)])
    total_q = b.total_q
    k_new = gen.normal_bf16(316, 1, (total_q, 2, 64))
    v_new = gen.normal_bf16(316, 2, (total_q, 2, 64))
    ks, vs = 0.011, 0.02
    kp, vp = b.k_pool.copy(), b.v_pool.copy()
    oracle.kv_append_fp8(k_new, v_new, kp, vp, b.block_tables, b.q_offsets, b.ctx_lens, ks, vs)
    want_k, want_v = b.k_pool.copy(), b.v_pool.copy()
    kq = torch.from_numpy((gen.bf16_bits_to_f32(k_new) / np.float32(ks)).astype(np.float32)).clamp(-448, 448)
    vq = torch.from_numpy((gen.bf16_bits_to_f32(v_new) / np.float32(vs)).astype(np.float32)).clamp(-448, 448)
    kq = kq.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    vq = vq.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    r = 0
    for i in range(b.num_seqs):
        q_len = int(b.q_offsets[i + 1] - b.q_offsets[i])
        for j in range(q_len):
            p = int(b.ctx_lens[i]) - q_len + j
            blk = int(b.block_tables[i, p // 16])
            want_k[blk, p % 16] = kq[r]
            want_v[blk, p % 16] = vq[r]
            r += 1
    np.testing.assert_array_equal(kp, want_k)
    np.testing.assert_array_equal(vp, want_v)
    assert (kp != b.k_pool).any() and (kp != vp).any()


def test_invalid_scales_are_rejected():
    b = gen.make_batch_fp8kv("f8f", 317, 4, 1, 64, [(1, 5)])
    args = (b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    for ks, vs in [(0.0, 1.0), (1.0, -1.0), (float("nan"), 1.0)]:
        with pytest.raises(ValueError):
            oracle.attn_mixed_batch_fp8kv(*args, ks, vs)
    with pytest.raises(ValueError):
        oracle.e4m3_quantize(np.zeros(4, dtype=np.uint16), 0.0)
