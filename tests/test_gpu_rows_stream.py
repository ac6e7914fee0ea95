"""The row path as one stream per workgroup (large decode-only launches): the rows' blocks are cut
into equal runs, one per persistent workgroup, and a row that straddles a cut is partitioned
there.  DSV_ROWS_STREAM forces the form (1: one run per compute unit, n > 1: n runs) on batches far
smaller than those it is chosen for, so that every path of the run logic is crossed: rows much
shorter than a run (many items per workgroup, one-block items among them), rows cut many times,
cuts that fall on row starts, more runs than rows.  Every output against the fp64 oracle."""
import numpy as np
import pytest

import oracle
from workloads import gen

pytestmark = pytest.mark.gpu
TOL = 1e-2

RAGGED = [(1, 1), (1, 15), (1, 16), (1, 17), (1, 3000), (1, 31), (1, 32), (1, 33), (1, 700), (1, 5000),
          (1, 2), (1, 1024), (1, 1025), (1, 255), (1, 48), (1, 9000), (1, 1), (1, 64)]


@pytest.mark.parametrize("runs", [1, 2, 3, 7, 40, 256, 1000])
@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (8, 2, 64), (16, 1, 128), (5, 5, 64)])
def test_decodes_of_every_length_in_any_number_of_runs(monkeypatch, runs, Hq, Hkv, D):
    from gpu_harness import run_attention
    import paper_2504_09285_amd as dsv
    monkeypatch.setenv("DSV_ROWS_STREAM", str(runs))
    b = gen.make_batch("stream_ragged", 900 + runs + D, Hq, Hkv, D, RAGGED)
    blocks = int(((b.ctx_lens + 15) // 16).sum())
    assert dsv.attn_mixed_batch_plan_info(b.q_offsets, b.ctx_lens, Hq, Hkv, D)["row_streams"] == min(runs, blocks)
    got = run_attention(b)
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    assert err.max() <= TOL, (float(err.max()), np.unravel_index(int(err.argmax()), err.shape))


@pytest.mark.parametrize("runs", [1, 5, 256])
def test_short_spans_on_the_row_path_and_a_span_on_the_mfma_path(monkeypatch, runs):
    """Spans of 2-15 tokens whose rows each have their own causal context, next to decodes; with a
    long span in the batch the row work is streamed only when the two kernels are launched apart."""
    from gpu_harness import run_attention
    monkeypatch.setenv("DSV_ROWS_STREAM", str(runs))
    monkeypatch.setenv("DSV_MIXED_LAUNCH", "0")
    segs = [(3, 40), (1, 900), (15, 70), (2, 2), (7, 130), (1, 4000), (200, 260), (4, 100), (1, 16)]
    b = gen.make_batch("stream_spans", 910 + runs, 32, 8, 128, segs)
    got = run_attention(b)
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.isfinite(got).all() and np.abs(got - ref).max() <= TOL


@pytest.mark.parametrize("runs", [3, 256])
def test_bf16_output_and_8bit_cache(monkeypatch, runs):
    import torch
    from gpu_harness import run_attention, run_attention_fp8kv
    monkeypatch.setenv("DSV_ROWS_STREAM", str(runs))
    b = gen.make_batch("stream_bf16", 920 + runs, 32, 8, 128, RAGGED)
    f32 = run_attention(b)
    bf = run_attention(b, out_dtype=torch.bfloat16)
    np.testing.assert_array_equal(bf, gen.f32_to_bf16_bits(f32))
    b8 = gen.make_batch_fp8kv("stream_f8", 930 + runs, 32, 8, 128, RAGGED)
    got = run_attention_fp8kv(b8)
    ref = oracle.attn_mixed_batch_fp8kv(b8.q, b8.k_pool, b8.v_pool, b8.block_tables, b8.q_offsets, b8.ctx_lens, b8.scale,
                                        b8.meta["k_scale"], b8.meta["v_scale"])
    assert np.abs(got - ref).max() <= TOL


def test_one_run_and_the_item_form_agree(monkeypatch):
    """One run: no row is cut and every row is one item, as in the item form with a partition that
    covers the whole row; the two forms share the per-block arithmetic, so the results are equal
    bit for bit."""
    from gpu_harness import run_attention
    b = gen.make_batch("stream_same", 940, 32, 8, 128, [(1, c) for c in (1, 100, 1000, 1024, 513)])
    monkeypatch.setenv("DSV_ROWS_STREAM", "0")
    monkeypatch.setenv("DSV_PART_TOKENS", "1024")
    items = run_attention(b)
    monkeypatch.delenv("DSV_PART_TOKENS")
    monkeypatch.setenv("DSV_ROWS_STREAM", "1")
    stream = run_attention(b)
    np.testing.assert_array_equal(stream, items)
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.abs(stream - ref).max() <= TOL


MIXED = [(300, 900), (1, 3000), (1, 17), (64, 64), (1, 5000), (2, 40), (1, 1), (1, 700), (130, 2130), (1, 2048), (9, 300)]


@pytest.mark.parametrize("runs", [8, 64, 200])
@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (64, 8, 128), (8, 2, 64)])
def test_row_streams_and_prefill_tiles_in_one_launch(monkeypatch, runs, Hq, Hkv, D):
    """A batch with prefill spans and decodes: the row work runs as `runs` persistent streams at the
    head of the grid, the spans' tiles as one workgroup per item behind them."""
    from gpu_harness import run_attention
    import paper_2504_09285_amd as dsv
    monkeypatch.setenv("DSV_ROWS_STREAM", str(runs))
    b = gen.make_batch("stream_mixed", 950 + runs + D + Hq, Hq, Hkv, D, MIXED)
    info = dsv.attn_mixed_batch_plan_info(b.q_offsets, b.ctx_lens, Hq, Hkv, D)
    assert info["row_streams"] == runs and info["one_launch"] == 1 and info["tile_items"] > 0
    got = run_attention(b)
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    assert err.max() <= TOL, (float(err.max()), np.unravel_index(int(err.argmax()), err.shape))


def test_row_streams_and_prefill_tiles_on_an_8bit_cache(monkeypatch):
    from gpu_harness import run_attention_fp8kv
    monkeypatch.setenv("DSV_ROWS_STREAM", "16")
    b8 = gen.make_batch_fp8kv("stream_mixed_f8", 960, 32, 8, 128, MIXED)
    got = run_attention_fp8kv(b8)
    ref = oracle.attn_mixed_batch_fp8kv(b8.q, b8.k_pool, b8.v_pool, b8.block_tables, b8.q_offsets, b8.ctx_lens, b8.scale,
                                        b8.meta["k_scale"], b8.meta["v_scale"])
    assert np.abs(got - ref).max() <= TOL
