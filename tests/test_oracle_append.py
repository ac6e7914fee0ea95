"""Pins for the KV-append oracle (paper section 2.1: the new tokens' keys/values enter the cache
before attention reads it).  The definition is a scatter through the block table, so the pins
rebuild its result by other means: a gather written independently with numpy indexing, the
generator's own pool (which holds every token), and byte counts of what may and may not change."""
import numpy as np
import pytest

import oracle
from workloads import gen


def new_token_slots(b):
    """(block, slot) of every new token of the batch, in q order: plain Python loop."""
    blk, slot = [], []
    for i in range(b.num_seqs):
        q_len = int(b.q_offsets[i + 1] - b.q_offsets[i])
        for j in range(q_len):
            p = int(b.ctx_lens[i]) - q_len + j
            blk.append(int(b.block_tables[i, p // 16]))
            slot.append(p % 16)
    return np.asarray(blk), np.asarray(slot)


@pytest.mark.parametrize("segs", [[(1, 1)], [(5, 5), (1, 17), (16, 48), (3, 35)],
                                  [(48, 80), (1, 70), (1, 129), (1, 200)], [(33, 33), (1, 16), (2, 18)]])
def test_append_rebuilds_the_generators_pool(segs):
    b = gen.make_batch("app", 71, 4, 2, 64, segs)
    blk, slot = new_token_slots(b)
    k_new = np.ascontiguousarray(b.k_pool[blk, slot])          # gather: what the step produced
    v_new = np.ascontiguousarray(b.v_pool[blk, slot])
    kp, vp = b.k_pool.copy(), b.v_pool.copy()
    kp[blk, slot] = 0x7FC0                                     # the slots are not written yet
    vp[blk, slot] = 0xFFFF
    oracle.kv_append(k_new, v_new, kp, vp, b.block_tables, b.q_offsets, b.ctx_lens)
    np.testing.assert_array_equal(kp, b.k_pool)                # every byte, touched or not
    np.testing.assert_array_equal(vp, b.v_pool)


def test_append_touches_exactly_the_new_rows_and_keeps_k_v_apart():
    b = gen.make_batch("app2", 72, 8, 2, 128, [(7, 30), (1, 1), (20, 21)])
    total_q = int(b.q_offsets[-1])
    k_new = (np.arange(total_q * 2 * 128, dtype=np.uint32) % 60000 + 1).astype(np.uint16).reshape(total_q, 2, 128)
    v_new = (k_new + np.uint16(5000)).astype(np.uint16)
    kp, vp = b.k_pool.copy(), b.v_pool.copy()
    oracle.kv_append(k_new, v_new, kp, vp, b.block_tables, b.q_offsets, b.ctx_lens)
    changed_k = (kp != b.k_pool).any(axis=(2, 3))
    changed_v = (vp != b.v_pool).any(axis=(2, 3))
    blk, slot = new_token_slots(b)
    expect = np.zeros_like(changed_k)
    expect[blk, slot] = True
    assert (changed_k <= expect).all() and (changed_v <= expect).all()
    np.testing.assert_array_equal(kp[blk, slot], k_new)        # row r of k_new is token r
    np.testing.assert_array_equal(vp[blk, slot], v_new)


def test_append_then_attention_equals_attention_on_the_full_pool():
    b = gen.make_batch("app3", 73, 4, 1, 64, [(9, 20), (1, 40), (12, 12)])
    blk, slot = new_token_slots(b)
    k_new, v_new = np.ascontiguousarray(b.k_pool[blk, slot]), np.ascontiguousarray(b.v_pool[blk, slot])
    kp, vp = b.k_pool.copy(), b.v_pool.copy()
    kp[blk, slot] = 0
    vp[blk, slot] = 0
    oracle.kv_append(k_new, v_new, kp, vp, b.block_tables, b.q_offsets, b.ctx_lens)
    args = dict(q=b.q, block_tables=b.block_tables, q_offsets=b.q_offsets, ctx_lens=b.ctx_lens, scale=b.scale)
    np.testing.assert_array_equal(oracle.attn_mixed_batch(k_pool=kp, v_pool=vp, **args),
                                  oracle.attn_mixed_batch(k_pool=b.k_pool, v_pool=b.v_pool, **args))


def test_append_rejects_bad_problems():
    b = gen.make_batch("app4", 74, 4, 1, 64, [(3, 10)])
    k_new = np.zeros((3, 1, 64), np.uint16)
    with pytest.raises(ValueError):
        oracle.kv_append(k_new, k_new, b.k_pool.copy(), b.v_pool.copy(), b.block_tables,
                         np.array([0, 3], np.int32), np.array([2], np.int32))        # ctx < q_len
    with pytest.raises(ValueError):
        oracle.kv_append(k_new, k_new, b.k_pool.copy(), b.v_pool.copy(), b.block_tables[:, :0],
                         b.q_offsets, b.ctx_lens)                                    # table too short
