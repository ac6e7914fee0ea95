"""Pins for the attention oracle: every check compares it with something that is not itself
(dense brute force, torch's library attention, hand-derived values, closed forms, invariances).
CPU only."""
import math
import os

import numpy as np
import pytest

import oracle
from workloads import gen
from dense_ref import bf16_to_f64, dense_attention, dense_batch, gather_sequence

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_oracle(b, **over):
    a = dict(q=b.q, k_pool=b.k_pool, v_pool=b.v_pool, block_tables=b.block_tables,
             q_offsets=b.q_offsets, ctx_lens=b.ctx_lens, scale=b.scale)
    a.update(over)
    return oracle.attn_mixed_batch(**a)


def small_mixed(seed=7, Hq=4, Hkv=2, D=16):
    segs = [(5, 5), (1, 1), (7, 40), (1, 33), (16, 16), (3, 19), (1, 16), (1, 17)]
    return gen.make_batch("small", seed, Hq, Hkv, D, segs)


# ---------------------------------------------------------------- hand-derived golden values
def _parse_scale(tok):
    tok = tok.strip()
    return math.log(float(tok[2:])) if tok.startswith("ln") else float(tok)


def _rows(txt):
    return np.array([[float(x) for x in r.split()] for r in txt.split(";")], dtype=np.float32)


def test_hand_derived_cases():
    n = 0
    for line in open(os.path.join(GOLDEN, "hand_softmax_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, scale, q, K, V, O = [x.strip() for x in line.split("|")]
        K, V = _rows(K), _rows(V)
        ctx, D = K.shape
        qb = gen.f32_to_bf16_bits(_rows(q)).reshape(1, 1, D)
        # place tokens in blocks of 16 through a non-trivial table
        nblk = (ctx + 15) // 16
        table = np.array([[3, 1, 2][:nblk]], dtype=np.int32)
        kp = np.zeros((4, 16, 1, D), np.uint16)
        vp = np.zeros((4, 16, 1, D), np.uint16)
        for t in range(ctx):
            kp[table[0, t // 16], t % 16, 0] = gen.f32_to_bf16_bits(K[t])
            vp[table[0, t // 16], t % 16, 0] = gen.f32_to_bf16_bits(V[t])
        out = oracle.attn_mixed_batch(qb, kp, vp, table, [0, 1], [ctx], _parse_scale(scale))
        np.testing.assert_allclose(out[0, 0], _rows(O)[0].astype(np.float64), rtol=0, atol=1e-12,
                                   err_msg="case " + name)
        n += 1
    assert n >= 4


# ---------------------------------------------------------------- brute force / library
def test_matches_dense_bruteforce_small_mixed():
    b = small_mixed()
    np.testing.assert_allclose(run_oracle(b), dense_batch(b), rtol=0, atol=1e-12)


def test_matches_dense_bruteforce_config1():
    b, _ = gen.config1()
    assert b.q.shape == (51, 4, 64) and b.k_pool.shape == (256, 16, 1, 64)
    np.testing.assert_allclose(run_oracle(b), dense_batch(b), rtol=0, atol=1e-12)


def test_matches_torch_sdpa_fp64():
    """Single contiguous sequence == torch's scaled_dot_product_attention with a boolean mask."""
    import torch
    import torch.nn.functional as F
    b = gen.make_batch("sdpa", 11, 6, 3, 32, [(9, 37)])
    ctx, q_len, G = 37, 9, 2
    k = torch.from_numpy(gather_sequence(b.k_pool, b.block_tables[0], ctx))   # [ctx,Hkv,D]
    v = torch.from_numpy(gather_sequence(b.v_pool, b.block_tables[0], ctx))
    q = torch.from_numpy(bf16_to_f64(b.q))                                    # [q,Hq,D]
    k = k.repeat_interleave(G, dim=1).permute(1, 0, 2)                        # [Hq,ctx,D]
    v = v.repeat_interleave(G, dim=1).permute(1, 0, 2)
    mask = torch.arange(ctx)[None, :] <= (ctx - q_len + torch.arange(q_len))[:, None]
    ref = F.scaled_dot_product_attention(q.permute(1, 0, 2), k, v, attn_mask=mask, scale=b.scale)
    np.testing.assert_allclose(run_oracle(b), ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- softmax normalisation
def test_softmax_rows_sum_to_one():
    b = small_mixed()
    for i in range(b.num_seqs):
        for j in (0, int(b.q_lens[i]) - 1):
            for h in range(b.Hq):
                w, _ = oracle.attn_row_weights(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets,
                                               b.ctx_lens, b.scale, i, j, h)
                assert len(w) == b.ctx_lens[i] - b.q_lens[i] + j + 1
                assert abs(w.sum() - 1.0) <= 1e-12 and (w >= 0).all()


def test_constant_v_gives_constant_output():
    b = small_mixed()
    ones = np.full_like(b.v_pool, gen.f32_to_bf16_bits(np.float32([1.0]))[0])
    np.testing.assert_allclose(run_oracle(b, v_pool=ones), 1.0, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- closed forms
def test_ctx1_returns_v0_exactly():
    b = gen.make_batch("one", 3, 4, 2, 16, [(1, 1), (1, 1)])
    out = run_oracle(b)
    for i in range(2):
        v0 = bf16_to_f64(b.v_pool[b.block_tables[i, 0], 0])                   # [Hkv, D]
        np.testing.assert_array_equal(out[i], np.repeat(v0, 2, axis=0))


def test_zero_query_gives_running_mean_of_v():
    b = gen.make_batch("zq", 5, 2, 1, 8, [(6, 20)])
    out = run_oracle(b, q=np.zeros_like(b.q))
    v = gather_sequence(b.v_pool, b.block_tables[0], 20)[:, 0, :]
    for j in range(6):
        p = 14 + j
        np.testing.assert_allclose(out[j, 0], v[:p + 1].mean(axis=0), rtol=0, atol=1e-13)
        np.testing.assert_allclose(out[j, 1], v[:p + 1].mean(axis=0), rtol=0, atol=1e-13)


def test_equal_keys_give_mean_of_v():
    b = gen.make_batch("eqk", 6, 2, 2, 8, [(1, 30)])
    kp = b.k_pool.copy()
    kp[:] = kp[0, 0]          # every key row identical (per head)
    out = run_oracle(b, k_pool=kp)
    v = gather_sequence(b.v_pool, b.block_tables[0], 30)
    np.testing.assert_allclose(out[0], v.mean(axis=0), rtol=0, atol=1e-13)


def test_dominant_key_selects_its_value():
    D = 8
    b = gen.make_batch("dom", 8, 1, 1, D, [(1, 25)])
    kp = np.zeros_like(b.k_pool)
    star = 13
    big = gen.f32_to_bf16_bits(np.float32([64.0]))[0]
    kp[b.block_tables[0, star // 16], star % 16, 0, 0] = big
    q = np.zeros_like(b.q)
    q[0, 0, 0] = big          # score 4096*scale for the star key, 0 for the rest
    out = run_oracle(b, q=q, k_pool=kp)
    vstar = bf16_to_f64(b.v_pool[b.block_tables[0, star // 16], star % 16, 0])
    np.testing.assert_allclose(out[0, 0], vstar, rtol=0, atol=1e-12)


def test_score_shift_invariance():
    """Adding the same constant to every score of a row leaves the output unchanged: append one
    dimension where q=1 and every key holds the same value c."""
    b = gen.make_batch("shift", 9, 2, 1, 8, [(4, 21)])
    base = run_oracle(b)
    one = gen.f32_to_bf16_bits(np.float32([1.0]))[0]
    c = gen.f32_to_bf16_bits(np.float32([3.5]))[0]
    q2 = np.concatenate([b.q, np.full(b.q.shape[:2] + (1,), one, np.uint16)], axis=2)
    k2 = np.concatenate([b.k_pool, np.full(b.k_pool.shape[:3] + (1,), c, np.uint16)], axis=3)
    v2 = np.concatenate([b.v_pool, np.zeros(b.v_pool.shape[:3] + (1,), np.uint16)], axis=3)
    out = oracle.attn_mixed_batch(q2, k2, v2, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    np.testing.assert_allclose(out[..., :8], base, rtol=0, atol=1e-12)


def test_scale_is_applied_to_scores():
    """Doubling scale == doubling q (exact in bf16: exponent shift)."""
    b = gen.make_batch("scale", 10, 2, 2, 8, [(3, 18)])
    q2 = gen.f32_to_bf16_bits(gen.bf16_bits_to_f32(b.q) * np.float32(2.0))
    np.testing.assert_allclose(run_oracle(b, scale=2 * b.scale), run_oracle(b, q=q2),
                               rtol=0, atol=1e-12)


# ---------------------------------------------------------------- causal / prefix / split
def _one_request(seed, L, Hq=4, Hkv=2, D=16):
    """A request of L tokens with one query row per token."""
    return gen.make_batch("req", seed, Hq, Hkv, D, [(L, L)])


def test_decode_equals_last_prefill_row():
    L = 45
    full = _one_request(21, L)
    ref = run_oracle(full)
    dec = oracle.attn_mixed_batch(full.q[L - 1:L], full.k_pool, full.v_pool, full.block_tables,
                                  [0, 1], [L], full.scale)
    np.testing.assert_array_equal(dec[0], ref[L - 1])


def test_split_at_every_token_boundary_is_invariant():
    """A request cut at any boundary s gives the same rows (section 3.1: tokens 1..s and s+1..L)."""
    L = 37
    full = _one_request(22, L)
    ref = run_oracle(full)
    tbl = np.concatenate([full.block_tables, full.block_tables], axis=0)
    for s in range(1, L):
        out = oracle.attn_mixed_batch(full.q, full.k_pool, full.v_pool, tbl, [0, s, L], [s, L],
                                      full.scale)
        np.testing.assert_array_equal(out, ref)


def test_prefix_rows_equal_rows_of_the_unsplit_prefill():
    L, p = 50, 23
    full = _one_request(23, L)
    ref = dense_batch(full)
    out = oracle.attn_mixed_batch(full.q[p:], full.k_pool, full.v_pool, full.block_tables,
                                  [0, L - p], [L], full.scale)
    np.testing.assert_allclose(out, ref[p:], rtol=0, atol=1e-12)


def test_future_tokens_are_invisible():
    """Changing K/V of tokens after position p must not change row p."""
    L = 40
    full = _one_request(24, L)
    ref = run_oracle(full)
    kp, vp = full.k_pool.copy(), full.v_pool.copy()
    nan = np.uint16(0x7FC0)
    cut = 17
    for t in range(cut + 1, L):
        kp[full.block_tables[0, t // 16], t % 16] = nan
        vp[full.block_tables[0, t // 16], t % 16] = nan
    out = run_oracle(full, k_pool=kp, v_pool=vp)
    np.testing.assert_array_equal(out[:cut + 1], ref[:cut + 1])
    assert np.isnan(out[cut + 1:]).all()


def test_unowned_blocks_and_tail_slots_are_never_read():
    b = small_mixed()
    ref = run_oracle(b)
    owned = np.zeros(b.k_pool.shape[:2], bool)
    for i in range(b.num_seqs):
        t = np.arange(int(b.ctx_lens[i]))
        owned[b.block_tables[i, t // 16], t % 16] = True
    kp, vp = b.k_pool.copy(), b.v_pool.copy()
    kp[~owned] = 0x7FC0
    vp[~owned] = 0x7F80      # +inf
    np.testing.assert_array_equal(run_oracle(b, k_pool=kp, v_pool=vp), ref)


# ---------------------------------------------------------------- paging / GQA / order
def test_block_permutation_invariance():
    b = small_mixed()
    ref = run_oracle(b)
    nb = b.k_pool.shape[0]
    perm = np.random.default_rng(0).permutation(nb)          # new id of old block x is perm[x]
    kp, vp = np.empty_like(b.k_pool), np.empty_like(b.v_pool)
    kp[perm], vp[perm] = b.k_pool, b.v_pool
    np.testing.assert_array_equal(run_oracle(b, k_pool=kp, v_pool=vp,
                                             block_tables=perm[b.block_tables].astype(np.int32)), ref)


def test_gqa_equals_expanded_mha():
    b = small_mixed(Hq=6, Hkv=2)
    ref = run_oracle(b)
    kp = np.repeat(b.k_pool, 3, axis=2)
    vp = np.repeat(b.v_pool, 3, axis=2)
    np.testing.assert_array_equal(run_oracle(b, k_pool=kp, v_pool=vp), ref)


def test_gqa_head_mapping_is_contiguous_groups():
    """Head h must read KV head h // G, not h % Hkv: make KV head 1 the only one with signal."""
    b = gen.make_batch("gqa", 12, 4, 2, 8, [(1, 9)])
    vp = b.v_pool.copy()
    one = gen.f32_to_bf16_bits(np.float32([1.0]))[0]
    vp[:, :, 0, :] = 0
    vp[:, :, 1, :] = one
    out = run_oracle(b, v_pool=vp)
    np.testing.assert_allclose(out[0, :2], 0.0, atol=1e-13)
    np.testing.assert_allclose(out[0, 2:], 1.0, atol=1e-12)


def test_decode_kv_order_invariance():
    """For a decode token, permuting the order of its KV tokens leaves the output unchanged."""
    b = gen.make_batch("perm", 13, 4, 2, 16, [(1, 48)])
    ref = run_oracle(b)
    ctx = 48
    order = np.random.default_rng(1).permutation(ctx)
    kp, vp = b.k_pool.copy(), b.v_pool.copy()
    row = b.block_tables[0]
    for new_t, old_t in enumerate(order):
        kp[row[new_t // 16], new_t % 16] = b.k_pool[row[old_t // 16], old_t % 16]
        vp[row[new_t // 16], new_t % 16] = b.v_pool[row[old_t // 16], old_t % 16]
    np.testing.assert_allclose(run_oracle(b, k_pool=kp, v_pool=vp), ref, rtol=0, atol=1e-13)


def test_selected_rows_match_full():
    b = small_mixed()
    ref = run_oracle(b)
    rows = [(0, 4, 3), (2, 0, 0), (2, 6, 1), (3, 0, 2), (7, 0, 3)]
    out = oracle.attn_rows(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens,
                           b.scale, rows)
    for r, (i, j, h) in enumerate(rows):
        np.testing.assert_array_equal(out[r], ref[b.q_offsets[i] + j, h])


def test_rejects_bad_problems():
    b = small_mixed()
    with pytest.raises(ValueError):
        run_oracle(b, ctx_lens=np.where(np.arange(b.num_seqs) == 0, 1, b.ctx_lens))   # ctx < q_len
    with pytest.raises(ValueError):
        run_oracle(b, block_tables=b.block_tables[:, :1])                              # table too short
