"""GPU parity of the 8-bit KV variant (attn_mixed_batch_fp8kv, kv_append_fp8, kv_pack_chunks_fp8,
kv_unpack_chunks_fp8) against the fp64 / bit-level CPU oracle on the same seeded inputs, through
the C ABI.  Attention: max abs error <= 1e-2 on the fp32 output, as for the bf16 cache (the
codes are widened exactly, so the arithmetic after the load is the same).  Append: the stored
codes must be the oracle's, byte for byte - both decide the code in fp32.  Copies: byte-exact."""
import numpy as np
import pytest

import oracle
from workloads import gen

pytestmark = pytest.mark.gpu
TOL = 1e-2


def oracle_out(b, rows=None):
    args = (b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale,
            b.meta["k_scale"], b.meta["v_scale"])
    if rows is None:
        return oracle.attn_mixed_batch_fp8kv(*args)
    return oracle.attn_rows_fp8kv(*args, rows)


def check(b, tol=TOL):
    from gpu_harness import run_attention_fp8kv
    got = run_attention_fp8kv(b)
    ref = oracle_out(b)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    assert err <= tol, "max abs err %.3e" % err
    return got, ref


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (4, 1, 64), (8, 8, 128), (16, 8, 64), (64, 8, 128),
                                      (6, 2, 128), (40, 2, 64)])
def test_decodes_with_ragged_contexts(Hq, Hkv, D):
    ctx = [1, 2, 15, 16, 17, 31, 33, 100, 255, 256, 257, 700, 1025, 2100]
    b = gen.make_batch_fp8kv("f8dec", 4100 + D + Hq, Hq, Hkv, D, [(1, c) for c in ctx])
    check(b)


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (4, 1, 64), (16, 2, 64)])
def test_short_spans_mixed_with_decodes(Hq, Hkv, D):
    segs = [(3, 3), (1, 50), (15, 15), (7, 300), (1, 1), (12, 1500), (2, 18), (1, 777)]
    b = gen.make_batch_fp8kv("f8short", 4200 + D, Hq, Hkv, D, segs)
    check(b)


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (4, 1, 64), (8, 8, 128), (6, 2, 128), (16, 8, 64)])
def test_prefill_spans_read_the_staged_copy(Hq, Hkv, D):
    """Spans of 16 and more tokens take the matrix-core path on a bf16 copy of their contexts:
    spans with and without prefix, ragged tails, several tiles, next to decodes and short spans."""
    segs = [(16, 16), (1, 90), (64, 64), (65, 130), (100, 1000), (3, 40), (130, 131), (17, 600), (1, 2000)]
    b = gen.make_batch_fp8kv("f8pre", 4300 + D + Hq, Hq, Hkv, D, segs)
    check(b)


def test_more_segments_than_one_planner_pass():
    """2,600 segments with prefill spans in the planner's second and third pass of 1,024: the
    staged segments' indices and block offsets carry across passes."""
    rng = np.random.default_rng(11)
    segs = [(1, int(c)) for c in rng.integers(1, 180, 2600)]
    for i, s in {5: (20, 50), 1030: (70, 200), 1500: (3, 90), 2047: (64, 64), 2300: (130, 131), 2599: (7, 7)}.items():
        segs[i] = s
    check(gen.make_batch_fp8kv("f8many", 4350, 8, 2, 64, segs))


def test_mixed_launch_equals_the_two_kernels_apart(monkeypatch):
    """Prefill tiles (on the staged copy) and row items (on the codes) in one launch: forced on,
    forced off and left to the library give bit-equal outputs, and they match the oracle."""
    from gpu_harness import run_attention_fp8kv
    for Hq, Hkv, D, segs in [(32, 8, 128, [(300, 420), (1, 900), (64, 64), (1, 17), (3, 200), (1, 5000)]),
                             (16, 2, 64, [(70, 70), (1, 33), (2, 40)]),
                             (64, 8, 128, [(129, 300), (1, 2500)])]:
        b = gen.make_batch_fp8kv("f8mixed", 4360, Hq, Hkv, D, segs)
        monkeypatch.setenv("DSV_MIXED_LAUNCH", "1")
        one = run_attention_fp8kv(b)
        monkeypatch.setenv("DSV_MIXED_LAUNCH", "0")
        two = run_attention_fp8kv(b)
        monkeypatch.delenv("DSV_MIXED_LAUNCH", raising=False)
        auto = run_attention_fp8kv(b)
        np.testing.assert_array_equal(one, two)
        np.testing.assert_array_equal(auto, two)
        assert np.abs(one - oracle_out(b)).max() <= TOL


def test_query_tiles_cut_along_the_context_forced(monkeypatch):
    """Context partitions of the query tiles on the staged copy of an 8-bit cache."""
    monkeypatch.setenv("DSV_TILE_PART_TILES", "2")
    segs = [(64, 64), (65, 130), (100, 1000), (3, 40), (130, 131), (1, 2000)]
    check(gen.make_batch_fp8kv("f8cut", 4370, 16, 2, 128, segs))


def test_only_prefill_spans_and_bf16_output():
    import torch
    from gpu_harness import run_attention_fp8kv
    b = gen.make_batch_fp8kv("f8only", 4400, 8, 2, 128, [(200, 200), (96, 400)])
    f32, _ = check(b)
    b16 = run_attention_fp8kv(b, out_dtype=torch.bfloat16)
    np.testing.assert_array_equal(b16, gen.f32_to_bf16_bits(f32))


def test_scales_other_than_the_default():
    b = gen.make_batch_fp8kv("f8sc", 4500, 8, 2, 128, [(1, 300), (40, 90), (5, 5), (1, 1100)],
                             k_scale=0.37, v_scale=1.7)
    check(b, tol=4e-2)        # the outputs are 3.4 times larger than with the default v_scale
    b2 = gen.make_batch_fp8kv("f8sc", 4500, 8, 2, 128, [(1, 300), (40, 90), (5, 5), (1, 1100)],
                              k_scale=0.011, v_scale=0.02)
    check(b2)


def test_nan_codes_in_unowned_blocks_and_tail_slots_do_not_reach_the_output():
    from gpu_harness import run_attention_fp8kv
    segs = [(1, 5), (1, 33), (20, 41), (70, 100), (1, 250)]
    b = gen.make_batch_fp8kv("f8nan", 4600, 8, 2, 64, segs)
    kp, vp = b.k_pool.copy(), b.v_pool.copy()
    owned = np.zeros(kp.shape[:2], dtype=bool)                     # (block, slot) read by some row
    for i, (_, ctx) in enumerate(segs):
        for t in range(ctx):
            owned[b.block_tables[i, t // 16], t % 16] = True
    kp[~owned] = 0x7F
    vp[~owned] = 0xFF
    got = run_attention_fp8kv(b, k_pool=kp, v_pool=vp)
    assert np.isfinite(got).all()
    assert np.abs(got - oracle_out(b)).max() <= TOL


def test_decode_heavy_shape_sampled_rows():
    """Config 2's shape (256 decodes, lognormal contexts, 32 query / 8 KV heads, D=128) on an
    8-bit cache, in the launch configuration the benchmark times; rows sampled for the oracle."""
    from gpu_harness import run_attention_fp8kv
    ctx = gen.lognormal_lengths(gen.seed_for(2), 256, 1024.0, 0.8, 64, 8192)
    b = gen.make_batch_fp8kv("f8c2", gen.seed_for(2), 32, 8, 128, [(1, int(c)) for c in ctx])
    got = run_attention_fp8kv(b)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(7)
    longest = int(np.argmax(b.ctx_lens))
    rows = [(longest, 0, h) for h in (0, 31)] + [(int(i), 0, int(h)) for i, h in
                                                 zip(rng.integers(0, 256, 60), rng.integers(0, 32, 60))]
    ref = oracle_out(b, np.asarray(rows, dtype=np.int32))
    for r, (i, j, h) in enumerate(rows):
        err = np.abs(got[b.q_offsets[i] + j, h] - ref[r]).max()
        assert err <= TOL, (i, j, h, err)


def test_prefill_heavy_shape_sampled_rows():
    """Config 3's shape: four 2048-token spans on prefixes 0/512/1024/4096 plus 16 decodes."""
    from gpu_harness import run_attention_fp8kv
    segs = [(2048, 2048 + p) for p in (0, 512, 1024, 4096)]
    ctx = gen.lognormal_lengths(gen.seed_for(3), 16, 2048.0, 0.8, 64, 16384)
    segs += [(1, int(c)) for c in ctx]
    b = gen.make_batch_fp8kv("f8c3", gen.seed_for(3), 32, 8, 128, segs)
    got = run_attention_fp8kv(b)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(8)
    rows = [(3, 2047, 31), (0, 0, 0), (0, 63, 5), (1, 64, 9), (2, 1000, 17)]
    rows += [(int(i), int(j), int(h)) for i, j, h in zip(rng.integers(0, 4, 40), rng.integers(0, 2048, 40),
                                                         rng.integers(0, 32, 40))]
    rows += [(int(i), 0, int(h)) for i, h in zip(rng.integers(4, 20, 10), rng.integers(0, 32, 10))]
    ref = oracle_out(b, np.asarray(rows, dtype=np.int32))
    for r, (i, j, h) in enumerate(rows):
        err = np.abs(got[b.q_offsets[i] + j, h] - ref[r]).max()
        assert err <= TOL, (i, j, h, err)


# ---- quantising append -------------------------------------------------------------------------

def _append_case(segs, Hkv, D, k_scale, v_scale, seed, k_new=None, v_new=None):
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import dev_bf16, dev_u8
    b = gen.make_batch_fp8kv("f8app", seed, 2 * Hkv, Hkv, D, segs)
    total_q = b.total_q
    if k_new is None:
        k_new = gen.normal_bf16(seed, 31, (total_q, Hkv, D))
        v_new = gen.normal_bf16(seed, 32, (total_q, Hkv, D))
    want_k, want_v = b.k_pool.copy(), b.v_pool.copy()
    oracle.kv_append_fp8(k_new, v_new, want_k, want_v, b.block_tables, b.q_offsets, b.ctx_lens,
                         k_scale, v_scale)
    pool = dsv.KVPool(dev_u8(b.k_pool[None]), dev_u8(b.v_pool[None]))
    bt = torch.from_numpy(b.block_tables).cuda()
    dsv.kv_append_fp8(dev_bf16(k_new), dev_bf16(v_new), pool, 0, bt, torch.from_numpy(b.q_offsets).cuda(),
                      torch.from_numpy(b.ctx_lens).cuda(), b.q_offsets, b.ctx_lens, k_scale, v_scale)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(pool.k.cpu().numpy()[0], want_k)
    np.testing.assert_array_equal(pool.v.cpu().numpy()[0], want_v)
    assert (want_k != b.k_pool).any()


@pytest.mark.parametrize("Hkv,D", [(8, 128), (1, 64), (2, 128), (3, 64)])
@pytest.mark.parametrize("scales", [(1.0, 1.0), (0.011, 0.02), (0.37, 17.25)])
def test_append_stores_the_oracles_codes(Hkv, D, scales):
    segs = [(7, 30), (1, 1), (20, 21), (1, 400), (130, 300), (1, 16), (2, 17)]
    _append_case(segs, Hkv, D, scales[0], scales[1], 4700 + Hkv + D)


def test_append_every_bf16_input_against_awkward_scales():
    """All finite bf16 bit patterns as inputs (ties, subnormal range, saturation, both zeros), with
    scales that include the fp32 just below 7, where dividing and multiplying by the reciprocal
    give different codes."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    bits = bits[np.isfinite(gen.bf16_bits_to_f32(bits))]
    n = bits.size // 128 * 128                                  # whole rows of 1 head x 128 dims
    rng = np.random.default_rng(3)
    k_new = np.ascontiguousarray(rng.permutation(bits)[:n].reshape(-1, 1, 128))
    v_new = np.ascontiguousarray(rng.permutation(bits)[:n].reshape(-1, 1, 128))
    below7 = float(np.nextafter(np.float32(7.0), np.float32(0.0)))
    for ks, vs in [(below7, 1.0), (3.0, 0.37), (2.0 ** -20, 2.0 ** 20)]:
        _append_case([(k_new.shape[0], k_new.shape[0] + 5)], 1, 128, ks, vs, 4800, k_new, v_new)


def test_append_then_attention_equals_the_oracles_chain():
    """kv_append_fp8 followed by attn_mixed_batch_fp8kv on the same stream, against the oracle's
    append followed by the oracle's attention."""
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceBatchFp8, dev_bf16
    segs = [(33, 70), (1, 129), (5, 5), (1, 900)]
    b = gen.make_batch_fp8kv("f8chain", 4900, 8, 2, 128, segs, k_scale=0.02, v_scale=0.02)
    k_new = gen.normal_bf16(4900, 31, (b.total_q, 2, 128))
    v_new = gen.normal_bf16(4900, 32, (b.total_q, 2, 128))
    want_k, want_v = b.k_pool.copy(), b.v_pool.copy()
    oracle.kv_append_fp8(k_new, v_new, want_k, want_v, b.block_tables, b.q_offsets, b.ctx_lens, 0.02, 0.02)
    ref = oracle.attn_mixed_batch_fp8kv(b.q, want_k, want_v, b.block_tables, b.q_offsets, b.ctx_lens,
                                        b.scale, 0.02, 0.02)
    d = DeviceBatchFp8(b)
    dsv.kv_append_fp8(dev_bf16(k_new), dev_bf16(v_new), d.pool, 0, d.block_tables, d.q_offsets, d.ctx_lens,
                      b.q_offsets, b.ctx_lens, 0.02, 0.02)
    got = d.run().cpu().numpy()
    assert np.abs(got - ref).max() <= TOL


# ---- chunked hand-off of 1-byte elements ----------------------------------------------------------

@pytest.mark.parametrize("L,Hkv,D,chunk_tokens", [(1, 1, 64, 32), (3, 8, 128, 64), (2, 2, 128, 100), (4, 3, 64, 7)])
def test_pack_and_unpack_of_codes_are_byte_exact(L, Hkv, D, chunk_tokens):
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import dev_u8
    seed = 5000 + L + D
    req = [130, 64, 17, 300]
    ranges = [(0, 0, 130), (1, 16, 64), (2, 3, 17), (3, 100, 300)]
    src_tables, nb_s = gen.build_block_tables(seed, gen.TID_SRC_PERM, req, 0.10)
    dst_tables, nb_d = gen.build_block_tables(seed, gen.TID_DST_PERM, req, 0.10)
    src_k = gen.e4m3_codes(seed, 41, (L, nb_s, 16, Hkv, D))
    src_v = gen.e4m3_codes(seed, 42, (L, nb_s, 16, Hkv, D))
    dst_k = gen.e4m3_codes(seed, 43, (L, nb_d, 16, Hkv, D))
    dst_v = gen.e4m3_codes(seed, 44, (L, nb_d, 16, Hkv, D))
    chunks, n_el = gen.make_chunks(ranges, chunk_tokens, L, Hkv, D)
    # Chunk offsets must be multiples of 16 bytes: pad each chunk's start up (the layout inside a
    # chunk is unchanged).
    off = 0
    for c in chunks:
        c[3] = off
        off += (2 * L * int(c[2]) * Hkv * D + 15) // 16 * 16
    n_el = off
    # The oracle's copies move 2-byte elements: the same bytes seen as [.., D/2] uint16.
    as16 = lambda a: np.ascontiguousarray(a).view(np.uint16)
    chunks16 = chunks.copy()
    chunks16[:, 3] //= 2
    want_buf = np.full(n_el // 2, 0xABCD, dtype=np.uint16)
    oracle.kv_pack_chunks(as16(src_k), as16(src_v), src_tables, chunks16, want_buf)
    want_dk, want_dv = as16(dst_k).copy(), as16(dst_v).copy()
    oracle.kv_unpack_chunks(want_buf, chunks16, want_dk, want_dv, dst_tables)

    src = dsv.KVPool(dev_u8(src_k), dev_u8(src_v))
    dst = dsv.KVPool(dev_u8(dst_k), dev_u8(dst_v))
    descs = dsv.ChunkDescs(chunks)
    buf = torch.from_numpy(np.full(n_el // 2, 0xABCD, dtype=np.uint16).view(np.uint8).copy()).cuda()
    dsv.kv_pack_chunks_fp8(src, torch.from_numpy(src_tables).cuda(), descs, buf)
    dsv.kv_unpack_chunks_fp8(buf, descs, dst, torch.from_numpy(dst_tables).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(buf.cpu().numpy().view(np.uint16), want_buf)
    np.testing.assert_array_equal(dst.k.cpu().numpy().view(np.uint16), want_dk)
    np.testing.assert_array_equal(dst.v.cpu().numpy().view(np.uint16), want_dv)
    assert (want_dk != as16(dst_k)).any()


@pytest.mark.parametrize("nbuf", ["4", "8"])
def test_deeper_lds_rings_of_the_row_kernel_8bit(monkeypatch, nbuf):
    """DSV_ROW_NBUF on the 8-bit cache: four slots (eight waves) or eight slots (four waves) per wave."""
    from gpu_harness import run_attention_fp8kv
    monkeypatch.setenv("DSV_ROW_NBUF", nbuf)
    monkeypatch.setenv("DSV_PART_TOKENS", "128")
    segs = [(1, 1), (1, 16), (1, 17), (1, 33), (1, 48), (1, 130), (1, 700), (1, 1025), (3, 40), (70, 90), (1, 64)]
    for Hq, Hkv, D in ((32, 8, 128), (12, 3, 64)):
        b = gen.make_batch_fp8kv("ring8_%s_%d" % (nbuf, D), 72, Hq, Hkv, D, segs)
        got = run_attention_fp8kv(b)
        ref = oracle.attn_mixed_batch_fp8kv(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens,
                                            b.scale, b.meta["k_scale"], b.meta["v_scale"])
        assert np.isfinite(got).all()
        assert np.abs(got - ref).max() <= TOL
