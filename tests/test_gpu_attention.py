"""GPU parity of attn_mixed_batch against the fp64 CPU oracle, element by element on the same
seeded inputs, through the C ABI.  Tolerance: max abs error <= 1e-2 on the fp32 output (bf16
inputs, fp32 accumulation); the bf16 output must be the round-to-nearest-even of the fp32 one."""
import os

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


@pytest.mark.parametrize("min_qlen", ["2", "16", "300"])
def test_short_and_long_spans_on_either_path(monkeypatch, min_qlen):
    """DSV_MFMA_MIN_QLEN moves the boundary between the row path (one pass over the context per
    query token) and the matrix-core path: spans of 2-15 tokens on both, and spans of up to 299
    tokens on the row path."""
    monkeypatch.setenv("DSV_MFMA_MIN_QLEN", min_qlen)
    segs = [(2, 2), (3, 50), (15, 15), (7, 1300), (1, 1), (12, 1500), (2, 2048), (1, 777), (40, 90), (299, 320)]
    for Hq, Hkv, D in [(32, 8, 128), (4, 1, 64)]:
        check(gen.make_batch("either", 97, Hq, Hkv, D, segs))


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
                     (dict(layer=1), -1),
                     (dict(num_q_heads=7, q=d.q[:, :7].contiguous(), out=out[:, :7].contiguous()), -1),   # 7 % 2
                     (dict(workspace=d.workspace[:256]), -3)]:
        with pytest.raises(dsv.DsvError) as e:
            call(**kw)
        assert e.value.code == code
    # What the C ABI cannot see (it carries no tensor shapes) the binding refuses before the call.
    for kw in [dict(num_q_heads=7), dict(q=d.q[:2].contiguous()), dict(out=out[:, :4].contiguous()),
               dict(q_offsets_host=np.array([0, 1, 3, 4], np.int32)),
               dict(block_tables=d.block_tables.to(torch.int64)), dict(block_tables=d.block_tables[:1].contiguous())]:
        with pytest.raises(ValueError):
            call(**kw)


# ------------------------------------------------------------------ long prefill spans (MFMA path)
@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (4, 1, 64), (8, 8, 128), (64, 8, 128), (6, 2, 128),
                                      (16, 1, 64), (2, 1, 128)])
def test_prefill_ragged_spans(Hq, Hkv, D):
    """Span lengths around the 32-token query tile and the 64-token KV tile, on prefixes that are
    empty, sub-block, block-aligned and unaligned; decodes interleaved."""
    segs = [(16, 16), (17, 18), (31, 46), (32, 32), (33, 49), (1, 77), (63, 113), (64, 264),
            (65, 65), (100, 103), (1, 300), (47, 1047), (129, 192)]
    b = gen.make_batch("pre_ragged", 61, Hq, Hkv, D, segs)
    check(b)


def test_split_at_token_boundaries_is_invariant_on_gpu():
    """Section 3.1: a request cut at any token gives the same outputs as the unsplit request.
    The two GPU results may differ by rounding (different tiling), each stays within tolerance."""
    from gpu_harness import run_attention
    L = 200
    full = gen.make_batch("req", 62, 8, 2, 128, [(L, L)])
    ref = oracle_out(full)
    whole = run_attention(full)
    assert np.abs(whole - ref).max() <= TOL
    tbl = np.concatenate([full.block_tables, full.block_tables], axis=0)
    for s in (1, 15, 16, 17, 63, 64, 100, 184, 199):
        split = gen.AttnBatch("split", 8, 2, 128, full.scale, full.q, full.k_pool, full.v_pool, tbl,
                              np.array([0, s, L], np.int32), np.array([s, L], np.int32))
        got = run_attention(split)
        assert np.abs(got - ref).max() <= TOL, s
        assert np.abs(got - whole).max() <= 2e-2, s


def test_prefill_poisoned_pool():
    from gpu_harness import run_attention
    segs = [(40, 40), (33, 70), (1, 90), (64, 129), (20, 21)]
    b = gen.make_batch("pre_poison", 63, 16, 4, 128, segs, free_frac=0.5)
    ref = run_attention(b)
    owned = np.zeros(b.k_pool.shape[:2], bool)
    for i in range(b.num_seqs):
        t = np.arange(int(b.ctx_lens[i]))
        owned[b.block_tables[i, t // 16], t % 16] = True
    kp, vp = b.k_pool.copy(), b.v_pool.copy()
    kp[~owned] = 0x7FC0
    vp[~owned] = 0x7FC0
    free_block = int(np.setdiff1d(np.arange(b.k_pool.shape[0]), b.block_tables.ravel())[0])
    bt = b.block_tables.copy()
    for i in range(b.num_seqs):
        bt[i, (int(b.ctx_lens[i]) + 15) // 16:] = free_block
    got = run_attention(b, k_pool=kp, v_pool=vp, block_tables=bt)
    assert np.isfinite(got).all()
    np.testing.assert_array_equal(got, ref)
    assert np.abs(got - oracle_out(b)).max() <= TOL


def test_prefill_constant_v():
    from gpu_harness import run_attention
    b = gen.make_batch("pre_cf", 64, 8, 2, 128, [(70, 150), (33, 33)])
    one = gen.f32_to_bf16_bits(np.float32([1.0]))[0]
    got = run_attention(b, v_pool=np.full_like(b.v_pool, one))
    np.testing.assert_allclose(got, 1.0, rtol=0, atol=1e-2)


def test_prefill_scores_far_above_first_subtile():
    """Keys from token 96 on are 64 times larger than the first ones, so later scores exceed the
    maximum over the first 32 tokens by hundreds of log2 units: the MFMA kernel's fast pass
    (reference value fixed after the first sub-tile) must notice that its sums leave the safe
    range and the robust pass must deliver the result.  Rows whose large scores are all negative
    stay on the fast pass within the same workgroups."""
    from gpu_harness import run_attention
    b = gen.make_batch("pre_growing", 65, 8, 2, 128, [(200, 300), (64, 64), (130, 260)])
    kp = b.k_pool.copy()
    for i in range(b.num_seqs):
        t = np.arange(96, int(b.ctx_lens[i])) if b.ctx_lens[i] > 96 else np.arange(0)
        rows = kp[b.block_tables[i, t // 16], t % 16]                  # bf16 bits [n, Hkv, D]
        kp[b.block_tables[i, t // 16], t % 16] = rows + np.uint16(6 << 7)   # exponent + 6: x64
    got = run_attention(b, k_pool=kp)
    ref = oracle_out(b, k_pool=kp)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= TOL


def test_mixed_launch_equals_the_two_kernels_apart(monkeypatch):
    """A batch with prefill tiles and row items can run both in one launch (DSV_MIXED_LAUNCH=1
    forces it, =0 forces the two kernels one after the other; unset, the library chooses).  Same
    kernel bodies, so the outputs are bit-equal."""
    from gpu_harness import run_attention
    for Hq, Hkv, D, segs in [(32, 8, 128, [(300, 420), (1, 900), (64, 64), (1, 17), (3, 200), (1, 5000)]),
                             (16, 2, 64, [(70, 70), (1, 33), (2, 40)]),
                             (64, 8, 128, [(129, 300), (1, 2500)])]:
        b = gen.make_batch("mixed_eq", 66, Hq, Hkv, D, segs)
        monkeypatch.setenv("DSV_MIXED_LAUNCH", "1")
        one = run_attention(b)
        monkeypatch.setenv("DSV_MIXED_LAUNCH", "0")
        two = run_attention(b)
        monkeypatch.delenv("DSV_MIXED_LAUNCH", raising=False)
        auto = run_attention(b)
        np.testing.assert_array_equal(one, two)
        np.testing.assert_array_equal(auto, two)
        assert np.abs(one - oracle_out(b)).max() <= TOL


def _many_segments():
    """2,600 segments: the planner's scans run three passes of 1,024 with carries between them,
    and prefill spans (tile work) sit in the second and third pass."""
    rng = np.random.default_rng(11)
    segs = [(1, int(c)) for c in rng.integers(1, 180, 2600)]
    for i, s in {5: (20, 50), 1030: (70, 200), 1500: (3, 90), 2047: (64, 64), 2300: (130, 131), 2599: (7, 7)}.items():
        segs[i] = s
    return segs


def test_more_segments_than_one_planner_pass():
    b = gen.make_batch("many", 91, 8, 2, 64, _many_segments())
    check(b)


@pytest.mark.parametrize("part_tiles", [1, 2, 3, 5])
def test_query_tiles_cut_along_the_context_forced(monkeypatch, part_tiles):
    """DSV_TILE_PART_TILES forces every query tile's context into partitions of that many KV
    tiles (production only cuts when query tiles are scarce, and never below 16): partials +
    merge must reproduce the oracle on spans with and without prefix, ragged tails, partitions
    of one tile, and rows that see nothing of their last partition."""
    monkeypatch.setenv("DSV_TILE_PART_TILES", str(part_tiles))
    segs = [(16, 16), (1, 90), (64, 64), (65, 130), (100, 1000), (3, 40), (130, 131), (17, 600),
            (1, 2000), (200, 777)]
    for Hq, Hkv, D in [(32, 8, 128), (4, 1, 64), (6, 2, 128)]:
        check(gen.make_batch("cut", 93 + part_tiles, Hq, Hkv, D, segs))


def test_short_span_on_a_long_prefix_is_cut_by_the_library():
    """Two query tiles on 20,000 cached tokens: 16 workgroups uncut; the library cuts the context
    so that the device is filled, and the result matches the oracle (all rows)."""
    import paper_2504_09285_amd as dsv
    b = gen.make_batch("long_prefix", 94, 32, 8, 128, [(128, 20128), (1, 300)])
    cut = dsv.attn_mixed_batch_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
    os.environ["DSV_TILE_PART_TILES"] = "-1"
    try:
        uncut = dsv.attn_mixed_batch_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
    finally:
        del os.environ["DSV_TILE_PART_TILES"]
    assert cut > uncut                  # partials of the cut q-tiles
    check(b)


def test_scale_zero_gives_the_mean_of_the_visible_values():
    """softmax_scale = 0: uniform weights over the causal context (masked scores must not turn
    into NaN when multiplied by a zero scale)."""
    b = gen.make_batch("scale0", 95, 8, 2, 128, [(70, 100), (1, 50), (5, 5), (1, 600)])
    b.scale = 0.0
    check(b)


def test_more_prefill_spans_than_the_planner_lists():
    """1,100 spans of 16-20 tokens: more segments with tile work than the planner's cooperative
    list holds, so every thread walks the query tiles of its own segments."""
    rng = np.random.default_rng(12)
    segs = [(int(q), int(q + p)) for q, p in zip(rng.integers(16, 21, 1100), rng.integers(0, 60, 1100))]
    segs += [(1, 100), (3, 50)]
    check(gen.make_batch("many_spans", 96, 4, 1, 64, segs))


def test_config3_prefill_heavy_shrunk():
    check(gen.config3(shrink=8))


def test_config3_prefill_heavy_full_sampled_rows():
    """Full-size prefill-heavy batch in the configuration bench.py times; the oracle recomputes a
    seeded sample of output rows (first/last rows of spans, tile edges, random rows, decodes)."""
    from gpu_harness import run_attention
    b = gen.config3()
    assert b.total_q == 8208 and b.ctx_lens[:4].tolist() == [2048, 2560, 3072, 6144]
    got = run_attention(b)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(3)
    rows = []
    for i in range(4):
        for j in (0, 1, 31, 32, 33, 1023, 2047):
            rows.append((i, j, int(rng.integers(b.Hq))))
        for _ in range(24):
            rows.append((i, int(rng.integers(2048)), int(rng.integers(b.Hq))))
    for i in range(4, b.num_seqs):
        rows.append((i, 0, int(rng.integers(b.Hq))))
    ref = oracle.attn_rows(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale, rows)
    for r, (i, j, h) in enumerate(rows):
        err = np.abs(got[b.q_offsets[i] + j, h] - ref[r]).max()
        assert err <= TOL, (i, j, h, err)


def test_thousands_of_row_items_of_every_length(monkeypatch):
    """400 decodes and short spans with contexts of 1 to 3,000 tokens, cut into 256-token
    partitions: about 2,500 row items of 1 to 16 blocks (several passes of the plan kernel's item
    loop, every bin of the dispatch order in use), listed longest first.  Every item must be
    processed exactly once whatever the order: sampled rows against the oracle, all rows finite."""
    from gpu_harness import run_attention
    monkeypatch.setenv("DSV_PART_TOKENS", "256")
    rng = np.random.default_rng(11)
    segs = [(1, int(c)) for c in rng.integers(1, 3000, 380)]
    segs += [(int(q), int(q) + int(c)) for q, c in zip(rng.integers(2, 9, 20), rng.integers(0, 100, 20))]
    order = rng.permutation(len(segs))
    segs = [segs[k] for k in order]
    b = gen.make_batch("many_items", 68, 16, 2, 128, segs)
    got = run_attention(b)
    assert np.isfinite(got).all()
    rows = [(int(i), 0, int(rng.integers(b.Hq))) for i in rng.choice(b.num_seqs, 120, replace=False)]
    shortest, longest = int(np.argmin(b.ctx_lens)), int(np.argmax(b.ctx_lens))
    rows += [(shortest, 0, 0), (longest, 0, b.Hq - 1)]
    for i in range(b.num_seqs):
        q_len = int(b.q_offsets[i + 1] - b.q_offsets[i])
        if q_len > 1:
            rows.append((i, q_len - 1, int(rng.integers(b.Hq))))
    ref = oracle.attn_rows(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale, rows)
    for r, (i, j, h) in enumerate(rows):
        err = np.abs(got[b.q_offsets[i] + j, h] - ref[r]).max()
        assert err <= TOL, (i, j, h, err)


def test_long_prefill_on_a_long_prefix_sampled_rows():
    """A 8,192-token span resuming on a 24,576-token prefix (ctx 32,768: 512 KV tiles for the last
    query tile), an unaligned one (ctx 20,011) and a few decodes, 64/8 heads: many tiles per work
    item, the tile list sorted across spans, the mixed launch.  Sampled rows against the oracle."""
    from gpu_harness import run_attention
    b = gen.make_batch("long_prefill", 67, 64, 8, 128, [(8192, 32768), (1, 30000), (3011, 20011), (1, 777), (5, 9000)])
    got = run_attention(b)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(4)
    rows = [(0, j, int(rng.integers(b.Hq))) for j in (0, 1, 63, 64, 4095, 8127, 8128, 8191)]
    rows += [(0, int(rng.integers(8192)), int(rng.integers(b.Hq))) for _ in range(10)]
    rows += [(2, j, int(rng.integers(b.Hq))) for j in (0, 10, 2999, 3010)]
    rows += [(2, int(rng.integers(3011)), int(rng.integers(b.Hq))) for _ in range(6)]
    rows += [(1, 0, 5), (3, 0, 63), (4, 0, 0), (4, 4, 17)]
    ref = oracle.attn_rows(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale, rows)
    for r, (i, j, h) in enumerate(rows):
        err = np.abs(got[b.q_offsets[i] + j, h] - ref[r]).max()
        assert err <= TOL, (i, j, h, err)


def _config4_inputs(shrink):
    """Config 4 placement, CPU side: row 0 holds the prompt; row 1's tokens [k,L) are made equal to
    row 0's; tokens [0,k) reach row 1 by pack/unpack (done by the caller, oracle or GPU)."""
    b, sp = gen.config4(shrink=shrink)
    t = np.arange(sp.k, sp.total)
    for pool in (b.k_pool, b.v_pool):
        pool[b.block_tables[1, t // 16], t % 16] = pool[b.block_tables[0, t // 16], t % 16]
    return b, sp


def test_config4_micro_request_shrunk():
    """The split prompt's second span attends to a prefix that arrived through the GPU hand-off
    (pack from row 0, unpack into row 1); result equals the oracle's unsplit 4096/shrink prefill."""
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceBatch, host_u16
    b, sp = _config4_inputs(8)
    d = DeviceBatch(b)
    descs = dsv.ChunkDescs(sp.chunks)
    buf = torch.zeros(sp.chunk_elems, dtype=torch.bfloat16, device="cuda")
    src_tbl = d.block_tables[0:1].contiguous()
    dst_tbl = d.block_tables[1:2].contiguous()
    dsv.kv_pack_chunks(d.pool, src_tbl, descs, buf)
    dsv.kv_unpack_chunks(buf, descs, d.pool, dst_tbl)
    got = d.run().cpu().numpy()
    torch.cuda.synchronize()
    # oracle side: same hand-off with the oracle's copy routines, then attention
    kp, vp = b.k_pool.copy()[None], b.v_pool.copy()[None]
    obuf = np.zeros(sp.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(kp, vp, b.block_tables[0:1], sp.chunks, obuf)
    oracle.kv_unpack_chunks(obuf, sp.chunks, kp, vp, b.block_tables[1:2])
    np.testing.assert_array_equal(host_u16(d.pool.k), kp)
    np.testing.assert_array_equal(host_u16(d.pool.v), vp)
    ref = oracle_out(b, k_pool=kp[0], v_pool=vp[0])
    assert np.abs(got - ref).max() <= TOL
    # the two spans together are the unsplit prompt
    unsplit = gen.AttnBatch("unsplit", b.Hq, b.Hkv, b.D, b.scale, b.q[:sp.total], kp[0], vp[0],
                            b.block_tables[0:1], np.array([0, sp.total], np.int32),
                            np.array([sp.total], np.int32))
    ref_unsplit = oracle_out(unsplit)
    assert np.abs(got[:sp.total] - ref_unsplit).max() <= TOL


# ------------------------------------------------------------------ full-size spot checks
def _sampled_rows_check(b, rows, got):
    ref = oracle.attn_rows(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale, rows)
    for r, (i, j, h) in enumerate(rows):
        err = np.abs(got[b.q_offsets[i] + j, h] - ref[r]).max()
        assert err <= TOL, (i, j, h, err)


@pytest.mark.timeout(600)
def test_config4_micro_request_full_sampled_rows():
    """Config 4 at full size (64/8 heads, 4096-token prompt split at the seeded boundary, 128 decodes
    with contexts up to 32768), hand-off through the GPU pack/unpack, sampled rows vs the oracle."""
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceBatch, host_u16
    b, sp = _config4_inputs(1)
    assert b.Hq == 64 and sp.total == 4096 and b.num_seqs == 130
    d = DeviceBatch(b)
    descs = dsv.ChunkDescs(sp.chunks)
    buf = torch.zeros(sp.chunk_elems, dtype=torch.bfloat16, device="cuda")
    dsv.kv_pack_chunks(d.pool, d.block_tables[0:1].contiguous(), descs, buf)
    dsv.kv_unpack_chunks(buf, descs, d.pool, d.block_tables[1:2].contiguous())
    got = d.run().cpu().numpy()
    assert np.isfinite(got).all()
    kp, vp = b.k_pool[None].copy(), b.v_pool[None].copy()
    obuf = np.zeros(sp.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(kp, vp, b.block_tables[0:1], sp.chunks, obuf)
    oracle.kv_unpack_chunks(obuf, sp.chunks, kp, vp, b.block_tables[1:2])
    np.testing.assert_array_equal(host_u16(buf), obuf)
    np.testing.assert_array_equal(host_u16(d.pool.k), kp)
    moved = gen.AttnBatch(b.name, b.Hq, b.Hkv, b.D, b.scale, b.q, kp[0], vp[0], b.block_tables,
                          b.q_offsets, b.ctx_lens)
    rng = np.random.default_rng(4)
    rows = [(0, 0, 0), (0, sp.k - 1, 63), (1, 0, 5), (1, sp.total - sp.k - 1, 17)]
    rows += [(0, int(rng.integers(sp.k)), int(rng.integers(64))) for _ in range(20)]
    rows += [(1, int(rng.integers(sp.total - sp.k)), int(rng.integers(64))) for _ in range(20)]
    rows += [(int(i), 0, int(rng.integers(64))) for i in rng.choice(np.arange(2, 130), 24, replace=False)]
    rows.append((2 + int(np.argmax(b.ctx_lens[2:])), 0, 7))
    _sampled_rows_check(moved, rows, got)


@pytest.mark.timeout(900)
def test_config5_long_context_full_sampled_rows():
    """Config 5's attention at full size (64 decodes, contexts 16K..128K, one layer's pool of
    ~0.24M blocks: block offsets exceed 2^32 elements); sampled (sequence, head) rows vs the oracle."""
    from gpu_harness import run_attention
    b = gen.config5_attention(threads=16)
    assert b.num_seqs == 64 and int(b.k_pool.size) > 2 ** 31
    got = run_attention(b)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(5)
    rows = [(int(i), 0, int(rng.integers(32))) for i in rng.choice(64, 20, replace=False)]
    rows += [(int(np.argmax(b.ctx_lens)), 0, h) for h in (0, 31)]
    rows += [(int(np.argmin(b.ctx_lens)), 0, 13)]
    far = int(np.argmax(b.block_tables.max(axis=1)))          # the sequence owning the highest block id
    rows.append((far, 0, 3))
    _sampled_rows_check(b, rows, got)


# ------------------------------------------------------------------ full size, every output
def _all_outputs_check(b, got):
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert got.shape == ref.shape and np.isfinite(got).all()
    err = np.abs(got - ref)
    assert err.max() <= TOL, (float(err.max()), np.unravel_index(int(err.argmax()), err.shape))
    return ref


@pytest.mark.timeout(900)
def test_config3_prefill_heavy_full_every_output():
    """Config 3 at its stated size, in the launch configuration bench.py times: every one of the
    8,208 x 32 output rows against the oracle (about 330 GFLOP of fp64 on the host cores)."""
    from gpu_harness import run_attention
    b = gen.config3(threads=16)
    assert b.total_q == 8208 and b.Hq == 32 and b.ctx_lens[:4].tolist() == [2048, 2560, 3072, 6144]
    _all_outputs_check(b, run_attention(b))


@pytest.mark.timeout(900)
def test_config4_micro_request_full_every_output():
    """Config 4 at its stated size: the prompt's first k tokens reach the second span's table through
    GPU pack/unpack in 64-token chunks, then one mixed batch (two spans + 128 decodes, 64/8 heads).
    Every output against the oracle, and the two spans together against the unsplit prompt."""
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceBatch, host_u16
    b, sp = _config4_inputs(1)
    assert b.Hq == 64 and sp.total == 4096 and b.num_seqs == 130 and b.total_q == 4224
    d = DeviceBatch(b)
    descs = dsv.ChunkDescs(sp.chunks)
    buf = torch.zeros(sp.chunk_elems, dtype=torch.bfloat16, device="cuda")
    dsv.kv_pack_chunks(d.pool, d.block_tables[0:1].contiguous(), descs, buf)
    dsv.kv_unpack_chunks(buf, descs, d.pool, d.block_tables[1:2].contiguous())
    got = d.run(fill=float("nan")).cpu().numpy()
    kp, vp = b.k_pool[None].copy(), b.v_pool[None].copy()
    obuf = np.zeros(sp.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(kp, vp, b.block_tables[0:1], sp.chunks, obuf)
    oracle.kv_unpack_chunks(obuf, sp.chunks, kp, vp, b.block_tables[1:2])
    np.testing.assert_array_equal(host_u16(buf), obuf)
    np.testing.assert_array_equal(host_u16(d.pool.k), kp)
    np.testing.assert_array_equal(host_u16(d.pool.v), vp)
    moved = gen.AttnBatch(b.name, b.Hq, b.Hkv, b.D, b.scale, b.q, kp[0], vp[0], b.block_tables,
                          b.q_offsets, b.ctx_lens)
    ref = _all_outputs_check(moved, got)
    unsplit = gen.AttnBatch("unsplit", b.Hq, b.Hkv, b.D, b.scale, b.q[:sp.total], kp[0], vp[0],
                            b.block_tables[0:1], np.array([0, sp.total], np.int32),
                            np.array([sp.total], np.int32))
    ref_unsplit = oracle_out(unsplit)
    assert np.abs(got[:sp.total] - ref_unsplit).max() <= TOL
    assert np.abs(ref[:sp.total] - ref_unsplit).max() <= 1e-12      # the oracle's own split invariant


@pytest.mark.timeout(900)
def test_config5_long_context_full_every_output():
    """Config 5's attention at its stated size (64 decodes on 16K-128K contexts, a pool of 0.24M
    blocks whose offsets pass 2^32 elements): all 64 x 32 output rows against the oracle."""
    from gpu_harness import run_attention
    b = gen.config5_attention(threads=16)
    assert b.num_seqs == 64 and int(b.k_pool.size) > 2 ** 31
    _all_outputs_check(b, run_attention(b))


@pytest.mark.parametrize("nbuf", ["3", "4"])
def test_deeper_lds_rings_of_the_row_kernel(monkeypatch, nbuf):
    """DSV_ROW_NBUF selects three or four LDS ring slots per wave (four waves per workgroup instead
    of eight, two workgroups per item with eight KV heads; tiles and rows then run in launches of
    their own).  Contexts shorter than the ring, of exactly one block, ragged, and split rows."""
    from gpu_harness import run_attention
    monkeypatch.setenv("DSV_ROW_NBUF", nbuf)
    monkeypatch.setenv("DSV_PART_TOKENS", "128")
    segs = [(1, 1), (1, 16), (1, 17), (1, 33), (1, 48), (1, 130), (1, 700), (1, 1025), (3, 40), (70, 90), (1, 64)]
    for Hq, Hkv, D in ((32, 8, 128), (12, 3, 64)):
        b = gen.make_batch("ring%s_%d" % (nbuf, D), 71, Hq, Hkv, D, segs)
        got = run_attention(b)
        ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
        assert np.isfinite(got).all()
        assert np.abs(got - ref).max() <= TOL


@pytest.mark.parametrize("G,Hkv,D,cut", [(5, 8, 128, None), (5, 2, 64, "2"), (6, 1, 128, None), (7, 2, 128, "3"),
                                         (9, 1, 64, None), (10, 2, 128, "1"), (3, 3, 128, None), (13, 1, 128, None)])
def test_head_groups_that_are_not_four_heads(monkeypatch, G, Hkv, D, cut):
    """Query heads per KV head that do not fill groups of four (the paper's Qwen-2.5 models have
    40 query and 8 KV heads): a work item of the MFMA path then takes (token, head) pairs of a
    group of up to eight heads for fewer tokens (51 x 5, 42 x 6, 36 x 7, 32 x 8), so query tiles
    are not 64 tokens long.  Spans shorter and longer than a tile, with and without prefix,
    ragged ends, decodes in between; with and without query tiles cut along the context."""
    from gpu_harness import run_attention
    if cut is not None:
        monkeypatch.setenv("DSV_TILE_PART_TILES", cut)
    segs = [(200, 200), (1, 300), (51, 51), (52, 700), (36, 36), (17, 17), (130, 1000), (1, 40), (32, 95), (64, 64)]
    b = gen.make_batch("flat%d_%d" % (G, D), 90 + G, G * Hkv, Hkv, D, segs)
    got = run_attention(b)
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    assert err.max() <= TOL, (err.max(), np.unravel_index(err.argmax(), err.shape))
