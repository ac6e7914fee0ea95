"""GPU parity of attn_mixed_batch against the fp64 CPU oracle, element by element on the same
seeded inputs, through the C ABI.  Tolerance: max abs error <= 1e-2 on the fp32 output (bf16
inputs, fp32 accumulation); the bf16 output must be the round-to-nearest-even of the fp32 one."""
import numpy as np
import pytest

import oracle
from workloads import gen

pytestmark = pytest.mark.gpu
TOL = 1e-2


def oracle_out(b, **over):
    a = dict(q=b.q, k_pool=b.k_pool, v_pool=b.v_pool, block_tables=b.block_tables,
             q_offsets=b.q_offsets, ctx_lens=b.ctx_lens, scale=b.scale)
    a.update(over)
    return oracle.attn_mixed_batch(**a)


def check(b, tol=TOL):
    from gpu_harness import run_attention
    got = run_attention(b)
    ref = oracle_out(b)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    assert err <= tol, "max abs err %.3e" % err
    return got, ref


def test_config1_tiny_mixed_batch():
    b, _ = gen.config1()
    check(b)


def test_bf16_output_is_rne_of_fp32_output():
    import torch
    from gpu_harness import run_attention
    b, _ = gen.config1()
    f32 = run_attention(b)
    bf = run_attention(b, out_dtype=torch.bfloat16)
    np.testing.assert_array_equal(bf, gen.f32_to_bf16_bits(f32))


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (4, 1, 64), (8, 8, 128), (16, 8, 64), (64, 8, 128),
                                      (6, 2, 128), (16, 1, 64), (24, 2, 128), (5, 5, 64)])
def test_decode_ragged_contexts(Hq, Hkv, D):
    """Contexts around block and partition boundaries: single token, one short of / exactly / one
    past a block and a 128-token partition, and several partitions with a ragged tail."""
    ctx = [1, 2, 15, 16, 17, 31, 33, 127, 128, 129, 255, 256, 257, 300, 1000, 2047]
    b = gen.make_batch("ragged", 51, Hq, Hkv, D, [(1, c) for c in ctx])
    check(b)


def test_short_prefill_spans_mixed_with_decodes():
    """Sub-block prefill pieces (1..15 tokens) resuming on prefixes, interleaved with decodes in
    arbitrary order (Alg. 2 emits partial prefill requests next to all decodes)."""
    segs = [(3, 3), (1, 70), (15, 200), (7, 7), (1, 1), (2, 130), (9, 25), (1, 513), (12, 12), (5, 1029)]
    b = gen.make_batch("short", 52, 32, 8, 128, segs)
    check(b)


def test_constant_v_and_ctx1_closed_forms():
    from gpu_harness import run_attention
    b = gen.make_batch("cf", 53, 8, 2, 128, [(1, 1), (1, 300), (4, 40), (1, 1)])
    one = gen.f32_to_bf16_bits(np.float32([1.0]))[0]
    got = run_attention(b, v_pool=np.full_like(b.v_pool, one))
    np.testing.assert_allclose(got, 1.0, rtol=0, atol=1e-5)
    got = run_attention(b)
    for i in (0, 3):                                        # ctx = 1 -> V[0], exactly
        v0 = gen.bf16_bits_to_f32(b.v_pool[b.block_tables[i, 0], 0])          # [Hkv, D]
        np.testing.assert_array_equal(got[b.q_offsets[i]], np.repeat(v0, 4, axis=0))


def test_poisoned_unowned_blocks_and_tail_slots():
    """Pools are never zeroed: NaN/Inf in blocks the batch does not own, in slots past each
    context, and behind the padding of the block table must not reach the output."""
    from gpu_harness import run_attention
    segs = [(1, 5), (1, 16), (1, 100), (6, 50), (1, 129), (1, 1000), (3, 3)]
    b = gen.make_batch("poison", 54, 16, 4, 128, segs, free_frac=0.5)
    ref = run_attention(b)
    owned = np.zeros(b.k_pool.shape[:2], bool)
    for i in range(b.num_seqs):
        t = np.arange(int(b.ctx_lens[i]))
        owned[b.block_tables[i, t // 16], t % 16] = True
    kp, vp = b.k_pool.copy(), b.v_pool.copy()
    kp[~owned] = 0x7FC0          # NaN
    vp[~owned] = 0x7F80          # +Inf
    free_block = int(np.setdiff1d(np.arange(b.k_pool.shape[0]), b.block_tables.ravel())[0])
    bt = b.block_tables.copy()
    for i in range(b.num_seqs):
        bt[i, (int(b.ctx_lens[i]) + 15) // 16:] = free_block
    got = run_attention(b, k_pool=kp, v_pool=vp, block_tables=bt)
    assert np.isfinite(got).all()
    np.testing.assert_array_equal(got, ref)
    assert np.abs(got - oracle_out(b)).max() <= TOL


def test_decode_equals_last_row_of_short_prefill():
    from gpu_harness import run_attention
    L = 12
    full = gen.make_batch("req", 55, 8, 2, 128, [(L, L)])
    a = run_attention(full)
    dec = gen.AttnBatch("dec", 8, 2, 128, full.scale, full.q[L - 1:L], full.k_pool, full.v_pool,
                        full.block_tables, np.array([0, 1], np.int32), np.array([L], np.int32))
    d = run_attention(dec)
    assert np.abs(d[0] - a[L - 1]).max() <= 2e-2
    assert np.abs(d - oracle_out(dec)).max() <= TOL


def test_config2_decode_heavy_shrunk():
    check(gen.config2(shrink=4))


def test_config2_decode_heavy_full():
    b = gen.config2()
    assert b.num_seqs == 256 and b.Hq == 32 and b.Hkv == 8 and b.D == 128
    check(b)


def test_config5_long_context_shrunk():
    check(gen.config5_attention(shrink=16))


def test_invalid_arguments_are_refused():
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceBatch
    b = gen.make_batch("bad", 56, 8, 2, 128, [(1, 40), (2, 20)])
    d = DeviceBatch(b)
    out = torch.empty(d.q.shape, dtype=torch.float32, device="cuda")

    def call(**kw):
        a = dict(q=d.q, out=out, pool=d.pool, layer=0, block_tables=d.block_tables,
                 q_offsets=d.q_offsets, ctx_lens=d.ctx_lens, q_offsets_host=b.q_offsets,
                 ctx_lens_host=b.ctx_lens, num_q_heads=b.Hq, softmax_scale=b.scale,
                 workspace=d.workspace)
        a.update(kw)
        dsv.attn_mixed_batch(**a)

    call()
    for kw, code in [(dict(ctx_lens_host=np.array([40, 1], np.int32)), -1),      # ctx < q_len
                     (dict(ctx_lens_host=np.array([40, 4000], np.int32)), -1),   # table too short
                     (dict(layer=1), -1), (dict(num_q_heads=7), -1),
                     (dict(workspace=d.workspace[:256]), -3)]:
        with pytest.raises(dsv.DsvError) as e:
            call(**kw)
        assert e.value.code == code
