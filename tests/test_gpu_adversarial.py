"""Parity on inputs far from N(0,1): keys whose magnitude rises or falls along the context by a
factor of 128 (the maxima of neighbouring context partitions differ by hundreds of log2 units,
most partitions' weights underflow to zero in the merge), values of magnitude 100, 8-bit codes
over the format's whole range, and the bf16 output of every store path at head_dim 128.
All element-wise against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
from workloads import gen

pytestmark = pytest.mark.gpu
TOL = 1e-2

# Which kernels serve the prefill spans: in one launch with the row work (one work item per
# workgroup), or in a launch of their own, by persistent workgroups or by one workgroup per item.
LAUNCHES = {"one_launch": {}, "apart_persistent": {"DSV_MIXED_LAUNCH": "0"},
            "apart_one_item": {"DSV_MIXED_LAUNCH": "0", "DSV_TILES_PERSISTENT": "0"}}


def _scale_rows_by_position(b, pool, shift_of):
    """Multiplies token t of every sequence by 2**shift_of(t, ctx) exactly (exponent bits of the
    bf16 patterns; N(0,1) draws stay far from the ends of the exponent range)."""
    out = pool.copy()
    for i in range(b.num_seqs):
        ctx = int(b.ctx_lens[i])
        t = np.arange(ctx)
        sh = shift_of(t, ctx).astype(np.uint16)
        blk, slot = b.block_tables[i, t // 16], t % 16
        rows = pool[blk, slot]                                          # [ctx, Hkv, D] bf16 bits
        nonzero = (rows & np.uint16(0x7fff)) != 0
        out[blk, slot] = np.where(nonzero, rows + (sh[:, None, None] << np.uint16(7)), rows)
    return out


RISING = lambda t, ctx: (8 * t) // max(ctx, 1)              # x1 at the start ... x128 at the end
FALLING = lambda t, ctx: 7 - (8 * t) // max(ctx, 1)         # x128 at the start ... x1 at the end

SEGS = [(1, 3000), (1, 5000), (3, 2600), (1, 257), (1, 100), (200, 700), (70, 5000), (1, 1), (40, 40)]


@pytest.mark.parametrize("launch", list(LAUNCHES))
@pytest.mark.parametrize("direction", ["rising", "falling"])
@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (8, 2, 64)])
def test_partition_maxima_hundreds_of_log2_units_apart(monkeypatch, direction, Hq, Hkv, D, launch):
    """Rows split into 256-token partitions and query tiles cut into partitions of two KV tiles,
    with keys scaled by position: scores reach several hundred log2 units, so the row kernel's
    running rescale, the MFMA kernel's robust pass and both merge kernels combine partials whose
    reference values are far apart (rising: every later partition dwarfs the earlier ones;
    falling: the first one dwarfs the rest)."""
    from gpu_harness import run_attention
    monkeypatch.setenv("DSV_PART_TOKENS", "256")
    monkeypatch.setenv("DSV_TILE_PART_TILES", "2")
    for k, v in LAUNCHES[launch].items():
        monkeypatch.setenv(k, v)
    b = gen.make_batch("adv_" + direction, 810 + D, Hq, Hkv, D, SEGS)
    kp = _scale_rows_by_position(b, b.k_pool, RISING if direction == "rising" else FALLING)
    # the scaled keys really do what the test is about: the raw scores of one decode row span
    # hundreds of log2 units between its first and last partitions
    i = 1
    q = gen.bf16_bits_to_f32(b.q[b.q_offsets[i], 0]).astype(np.float64)
    t = np.arange(int(b.ctx_lens[i]))
    k = gen.bf16_bits_to_f32(kp[b.block_tables[i, t // 16], t % 16][:, 0]).astype(np.float64)
    s = (k @ q) * b.scale * np.log2(np.e)
    part_max = np.array([s[p:p + 256].max() for p in range(0, len(s), 256)])
    assert part_max.max() - part_max.min() > 150
    got = run_attention(b, k_pool=kp)
    ref = oracle.attn_mixed_batch(b.q, kp, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    assert err.max() <= TOL, (float(err.max()), np.unravel_index(int(err.argmax()), err.shape))


def test_values_of_magnitude_100():
    """V scaled by 128 (exactly, exponent bits): the output is linear in V, so the error bound
    scales with it: |got - ref| <= 1e-2 * 128 everywhere, and relative to the row's largest
    output component it stays at the level of bf16 probabilities."""
    from gpu_harness import run_attention
    b = gen.make_batch("adv_bigv", 820, 32, 8, 128, SEGS)
    vp = _scale_rows_by_position(b, b.v_pool, lambda t, ctx: np.full_like(t, 7))
    got = run_attention(b, v_pool=vp)
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, vp, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    assert err.max() <= TOL * 128
    row_scale = np.abs(ref).max(axis=-1, keepdims=True)
    assert (err / np.maximum(row_scale, 1.0)).max() <= TOL


@pytest.mark.parametrize("launch", list(LAUNCHES))
@pytest.mark.parametrize("env", [{}, {"DSV_PART_TOKENS": "256", "DSV_TILE_PART_TILES": "3"}])
def test_bf16_output_is_rne_of_the_fp32_output_on_every_store_path(monkeypatch, env, launch):
    """head_dim 128, 32/8 heads: rows with one partition (row kernel's store), split rows (merge
    kernel's store), prefill tiles (MFMA kernel's epilogue) and, with the knobs set, query tiles
    cut along the context (the merge kernel's second instantiation).  The bf16 result must be the
    fp32 result rounded to nearest even, bit for bit."""
    from gpu_harness import run_attention
    import torch
    for k, v in list(env.items()) + list(LAUNCHES[launch].items()):
        monkeypatch.setenv(k, v)
    b = gen.make_batch("adv_rne", 830, 32, 8, 128, [(1, 50), (1, 3000), (100, 300), (70, 5000), (5, 900), (1, 1025)])
    f32 = run_attention(b)
    bf = run_attention(b, out_dtype=torch.bfloat16)
    np.testing.assert_array_equal(bf, gen.f32_to_bf16_bits(f32))
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.abs(f32 - ref).max() <= TOL


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (4, 1, 64)])
def test_8bit_codes_over_the_whole_finite_range(Hq, Hkv, D):
    """Every finite E4M3 code, magnitudes 2^-9 ... 448, both signs, uniformly: with k_scale = v_scale
    = 1/128 the cached values reach 3.5 and the outputs stay O(1).  Decodes (codes widened in
    registers), short spans and prefill spans (staged bf16 copy)."""
    from gpu_harness import run_attention_fp8kv
    segs = [(1, 700), (1, 2100), (40, 300), (3, 90), (130, 131), (1, 17)]
    b = gen.make_batch_fp8kv("adv_f8", 840 + D, Hq, Hkv, D, segs, k_scale=1.0 / 128, v_scale=1.0 / 128)
    rng = np.random.default_rng(841)
    finite = np.array([c for c in range(256) if (c & 0x7f) != 0x7f], np.uint8)       # 254 codes, no NaN
    kp = finite[rng.integers(0, len(finite), b.k_pool.shape)]
    vp = finite[rng.integers(0, len(finite), b.v_pool.shape)]
    assert (kp & 0x7f).max() == 0x7e and (vp & 0x7f).max() == 0x7e                   # +-448 present
    got = run_attention_fp8kv(b, k_pool=kp, v_pool=vp)
    ref = oracle.attn_mixed_batch_fp8kv(b.q, kp, vp, b.block_tables, b.q_offsets, b.ctx_lens, b.scale,
                                        b.meta["k_scale"], b.meta["v_scale"])
    assert np.isfinite(got).all() and np.abs(ref).max() < 4.0
    assert np.abs(got - ref).max() <= TOL


@pytest.mark.parametrize("Hq,Hkv,D,out", [(32, 8, 128, "f32"), (8, 2, 64, "bf16"), (40, 8, 128, "f32")])
@pytest.mark.parametrize("keys", ["plain", "rising"])
def test_hundreds_of_short_spans_through_the_persistent_workgroups(monkeypatch, Hq, Hkv, D, out, keys):
    """No decodes, so the spans run in the MFMA launch of their own: persistent workgroups that take
    many work items each.  600 spans of 16-300 tokens on prefixes of 0-400: items of one to eleven
    KV tiles in every order, among them runs of items shorter than the request look-ahead, and
    query tiles cut in two-tile partitions on top.  With rising keys most items repeat in the robust
    pass, which restarts the tile stream in mid-flight.  Every output against the oracle."""
    import torch
    from gpu_harness import run_attention
    monkeypatch.setenv("DSV_TILE_PART_TILES", "2")
    rng = np.random.default_rng(851)
    segs = [(int(q), int(q + p)) for q, p in zip(rng.integers(16, 301, 600), rng.integers(0, 401, 600))]
    b = gen.make_batch("adv_short_" + keys, 850 + D + Hq, Hq, Hkv, D, segs)
    kp = _scale_rows_by_position(b, b.k_pool, RISING) if keys == "rising" else b.k_pool
    ref = oracle.attn_mixed_batch(b.q, kp, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    if out == "f32":
        got = run_attention(b, k_pool=kp)
        assert np.isfinite(got).all()
        err = np.abs(got - ref)
        assert err.max() <= TOL, (float(err.max()), np.unravel_index(int(err.argmax()), err.shape))
    else:
        got = gen.bf16_bits_to_f32(run_attention(b, k_pool=kp, out_dtype=torch.bfloat16))
        assert np.isfinite(got).all()
        assert np.abs(got - ref).max() <= TOL + np.abs(ref).max() * 2.0 ** -8      # bf16 rounding of the output
