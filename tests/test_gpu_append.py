"""GPU parity of kv_append against the CPU oracle through the C ABI: bit-exact on the whole
pool (written rows and every untouched byte), on mixed batches, multi-layer pools, both head
dims, and followed by attention on the same stream."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_09285_amd as dsv
from workloads import gen

pytestmark = pytest.mark.gpu


def dev_u16(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)


def host_u16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def new_rows(seed, total_q, Hkv, D):
    rng = np.random.default_rng(seed)
    return (rng.integers(0, 0x7F80, size=(total_q, Hkv, D), dtype=np.uint16),
            rng.integers(0x8000, 0xFF80, size=(total_q, Hkv, D), dtype=np.uint16))


def run_append(b, k_new, v_new, layers=1, layer=0):
    kp = np.stack([b.k_pool] * layers) if layers > 1 else b.k_pool[None]
    vp = np.stack([b.v_pool] * layers) if layers > 1 else b.v_pool[None]
    pool = dsv.KVPool(dev_u16(kp), dev_u16(vp))
    bt = torch.from_numpy(np.ascontiguousarray(b.block_tables, dtype=np.int32)).cuda()
    dsv.kv_append(dev_u16(k_new), dev_u16(v_new), pool, layer, bt, torch.from_numpy(b.q_offsets).cuda(),
                  torch.from_numpy(b.ctx_lens).cuda(), b.q_offsets, b.ctx_lens)
    torch.cuda.synchronize()
    return host_u16(pool.k), host_u16(pool.v)


@pytest.mark.parametrize("Hq,Hkv,D,segs", [
    (4, 1, 64, [(48, 80), (1, 70), (1, 129), (1, 200)]),
    (32, 8, 128, [(1, c) for c in (1, 16, 17, 31, 32, 33, 500, 1023)]),
    (32, 8, 128, [(200, 300), (1, 77), (64, 64), (17, 4000), (1, 16)]),
    (16, 2, 128, [(5, 5), (3, 35)]),
    (8, 8, 64, [(130, 131), (1, 2)]),
])
def test_append_matches_oracle_bit_for_bit(Hq, Hkv, D, segs):
    b = gen.make_batch("gapp", 81, Hq, Hkv, D, segs)
    k_new, v_new = new_rows(5, int(b.q_offsets[-1]), Hkv, D)
    gk, gv = run_append(b, k_new, v_new)
    ok, ov = b.k_pool.copy(), b.v_pool.copy()
    oracle.kv_append(k_new, v_new, ok, ov, b.block_tables, b.q_offsets, b.ctx_lens)
    np.testing.assert_array_equal(gk[0], ok)
    np.testing.assert_array_equal(gv[0], ov)


def test_append_writes_only_the_chosen_layer():
    b = gen.make_batch("gapp_l", 82, 8, 2, 128, [(40, 100), (1, 9)])
    k_new, v_new = new_rows(6, int(b.q_offsets[-1]), 2, 128)
    gk, gv = run_append(b, k_new, v_new, layers=3, layer=1)
    ok, ov = b.k_pool.copy(), b.v_pool.copy()
    oracle.kv_append(k_new, v_new, ok, ov, b.block_tables, b.q_offsets, b.ctx_lens)
    for l in (0, 2):
        np.testing.assert_array_equal(gk[l], b.k_pool)
        np.testing.assert_array_equal(gv[l], b.v_pool)
    np.testing.assert_array_equal(gk[1], ok)
    np.testing.assert_array_equal(gv[1], ov)


def test_append_then_attention_on_one_stream():
    """The new tokens' K/V are cut out of the generator's pool, the slots are poisoned, and
    kv_append + attn_mixed_batch run back to back on a side stream: the result must equal the
    oracle's attention on the full pool."""
    b = gen.make_batch("gapp_attn", 83, 32, 8, 128, [(150, 260), (1, 700), (1, 33), (40, 40)])
    blk, slot = [], []
    for i in range(b.num_seqs):
        q_len = int(b.q_offsets[i + 1] - b.q_offsets[i])
        p = int(b.ctx_lens[i]) - q_len + np.arange(q_len)
        blk.append(b.block_tables[i, p // 16]); slot.append(p % 16)
    blk, slot = np.concatenate(blk), np.concatenate(slot)
    k_new, v_new = np.ascontiguousarray(b.k_pool[blk, slot]), np.ascontiguousarray(b.v_pool[blk, slot])
    kp, vp = b.k_pool.copy(), b.v_pool.copy()
    kp[blk, slot] = 0x7FC0
    vp[blk, slot] = 0x7FC0
    pool = dsv.KVPool(dev_u16(kp[None]), dev_u16(vp[None]))
    bt = torch.from_numpy(np.ascontiguousarray(b.block_tables, dtype=np.int32)).cuda()
    qo, cl = torch.from_numpy(b.q_offsets).cuda(), torch.from_numpy(b.ctx_lens).cuda()
    q = dev_u16(b.q)
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(dsv.attn_mixed_batch_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D),
                     dtype=torch.uint8, device="cuda")
    dk, dv = dev_u16(k_new), dev_u16(v_new)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        dsv.kv_append(dk, dv, pool, 0, bt, qo, cl, b.q_offsets, b.ctx_lens, stream=s)
        dsv.attn_mixed_batch(q, out, pool, 0, bt, qo, cl, b.q_offsets, b.ctx_lens, b.Hq, b.scale, ws, stream=s)
    s.synchronize()
    np.testing.assert_array_equal(host_u16(pool.k)[0], b.k_pool)
    ref = oracle.attn_mixed_batch(q=b.q, k_pool=b.k_pool, v_pool=b.v_pool, block_tables=b.block_tables,
                                  q_offsets=b.q_offsets, ctx_lens=b.ctx_lens, scale=b.scale)
    got = out.cpu().numpy()
    assert np.isfinite(got).all() and np.abs(got - ref).max() <= 1e-2


def test_append_refuses_invalid_arguments():
    b = gen.make_batch("gapp_bad", 84, 4, 1, 64, [(3, 10)])
    k_new, v_new = new_rows(7, 3, 1, 64)
    pool = dsv.KVPool(dev_u16(b.k_pool[None]), dev_u16(b.v_pool[None]))
    bt = torch.from_numpy(np.ascontiguousarray(b.block_tables, dtype=np.int32)).cuda()
    qo, cl = torch.from_numpy(b.q_offsets).cuda(), torch.from_numpy(b.ctx_lens).cuda()
    dk, dv = dev_u16(k_new), dev_u16(v_new)
    before = host_u16(pool.k).copy()
    with pytest.raises(dsv.DsvError):
        dsv.kv_append(dk, dv, pool, 1, bt, qo, cl, b.q_offsets, b.ctx_lens)                     # layer out of range
    with pytest.raises(dsv.DsvError):
        dsv.kv_append(dk, dv, pool, 0, bt, qo, cl, b.q_offsets, np.array([2], np.int32))        # ctx < q_len
    with pytest.raises(dsv.DsvError):
        dsv.kv_append(dk, dv, pool, 0, bt, qo, cl, np.array([1, 4], np.int32), b.ctx_lens)      # offsets not from 0
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host_u16(pool.k), before)                                     # nothing was enqueued
