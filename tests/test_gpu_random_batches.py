"""Seeded random mixed batches against the oracle: head geometries (also group sizes that are not
powers of two), head_dim 64 and 128, decodes, short spans, long spans with and without prefix in
any order, and the library's tuning knobs (partition sizes of rows and of query tiles, mixed
launch on or off, the row work as streams) drawn at random as well.  bf16 cache and 8-bit cache.  Tolerance as for the
fixed cases: max abs error <= 1e-2 on the fp32 output."""
import numpy as np
import pytest

import oracle
from workloads import gen

pytestmark = pytest.mark.gpu
TOL = 1e-2


def random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    Hkv = int(rng.choice([1, 2, 3, 8]))
    G = int(rng.choice([1, 2, 4, 5, 8, 16]))
    D = int(rng.choice([64, 128]))
    segs = []
    for _ in range(int(rng.integers(1, 11))):
        kind = rng.integers(0, 4)
        if kind == 0:
            segs.append((1, int(rng.integers(1, 1500))))
        elif kind == 1:
            q = int(rng.integers(2, 16))
            segs.append((q, q + int(rng.integers(0, 600))))
        elif kind == 2:
            q = int(rng.integers(16, 200))
            segs.append((q, q))
        else:
            q = int(rng.integers(16, 200))
            segs.append((q, q + int(rng.integers(1, 1200))))
    env = {}
    if rng.random() < 0.5:
        env["DSV_TILE_PART_TILES"] = str(int(rng.choice([1, 2, 3, 7])))
    if rng.random() < 0.5:
        env["DSV_PART_TOKENS"] = str(int(rng.choice([16, 64, 256])))
    if rng.random() < 0.6:
        env["DSV_MIXED_LAUNCH"] = str(int(rng.integers(0, 2)))
    if rng.random() < 0.5:
        env["DSV_MFMA_MIN_QLEN"] = str(int(rng.choice([2, 16, 64])))
    return Hkv * G, Hkv, D, segs, env


@pytest.mark.parametrize("seed", range(24))
def test_random_batch_bf16_cache(monkeypatch, seed):
    from gpu_harness import run_attention
    Hq, Hkv, D, segs, env = random_case(seed)
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    b = gen.make_batch("rnd%d" % seed, 7000 + seed, Hq, Hkv, D, segs)
    got = run_attention(b)
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.isfinite(got).all(), (Hq, Hkv, D, segs, env)
    err = np.abs(got - ref).max()
    assert err <= TOL, (err, Hq, Hkv, D, segs, env)


@pytest.mark.parametrize("seed", range(24, 40))
def test_random_batch_8bit_cache(monkeypatch, seed):
    from gpu_harness import run_attention_fp8kv
    Hq, Hkv, D, segs, env = random_case(seed)
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    b = gen.make_batch_fp8kv("rnd8_%d" % seed, 7000 + seed, Hq, Hkv, D, segs)
    got = run_attention_fp8kv(b)
    ref = oracle.attn_mixed_batch_fp8kv(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens,
                                        b.scale, b.meta["k_scale"], b.meta["v_scale"])
    assert np.isfinite(got).all(), (Hq, Hkv, D, segs, env)
    err = np.abs(got - ref).max()
    assert err <= TOL, (err, Hq, Hkv, D, segs, env)


def stream_knob(seed, env):
    """The row work as n streams (forced on batches far smaller than those it is chosen for), drawn
    from a generator of its own so that the cases above keep their draws."""
    rng = np.random.default_rng(5000 + seed)
    env = dict(env)
    env.pop("DSV_PART_TOKENS", None)                   # a forced partition size keeps the item form
    env["DSV_ROWS_STREAM"] = str(int(rng.choice([1, 2, 5, 8, 16, 24, 64, 256])))
    return env


@pytest.mark.parametrize("seed", range(40, 56))
def test_random_batch_row_streams(monkeypatch, seed):
    """Row streams next to whatever else the batch holds: alone, launched apart from the prefill
    tiles, or (stream counts that are multiples of eight) in one launch with them."""
    from gpu_harness import run_attention, run_attention_fp8kv
    Hq, Hkv, D, segs, env = random_case(seed)
    if not any(q == 1 for q, _ in segs):
        segs = segs + [(1, 700 + 13 * seed)]
    for k, v in stream_knob(seed, env).items():
        monkeypatch.setenv(k, v)
    import paper_2504_09285_amd as dsv
    qo = np.concatenate([[0], np.cumsum([q for q, _ in segs])]).astype(np.int32)
    cl = np.asarray([c for _, c in segs], np.int32)
    info = dsv.attn_mixed_batch_plan_info(qo, cl, Hq, Hkv, D, 2 - seed % 2)
    # (In one launch with prefill tiles the stream count is cut to a multiple of eight below the
    # number of compute units, which may leave none: then the item form runs.)
    assert info["rows"] >= 1, info
    if info["tile_items"] == 0 or env.get("DSV_MIXED_LAUNCH") == "0":
        assert info["row_streams"] >= 1, info
    if seed % 2 == 0:
        b = gen.make_batch("rnds%d" % seed, 7000 + seed, Hq, Hkv, D, segs)
        got = run_attention(b)
        ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    else:
        b = gen.make_batch_fp8kv("rnds8_%d" % seed, 7000 + seed, Hq, Hkv, D, segs)
        got = run_attention_fp8kv(b)
        ref = oracle.attn_mixed_batch_fp8kv(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens,
                                            b.scale, b.meta["k_scale"], b.meta["v_scale"])
    assert np.isfinite(got).all(), (Hq, Hkv, D, segs, env)
    err = np.abs(got - ref).max()
    assert err <= TOL, (err, Hq, Hkv, D, segs, env)
