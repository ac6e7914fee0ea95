"""Seeded random hand-offs and appends against the oracle, bit for bit: layer counts, head
geometries, request lengths, token ranges that start and end anywhere, chunk sizes from one token
to several hundred, for the bf16 cache; random appends (with quantisation) for the 8-bit cache."""
import numpy as np
import pytest

import oracle
from workloads import gen

pytestmark = pytest.mark.gpu


def random_handoff(seed):
    rng = np.random.default_rng(2000 + seed)
    L = int(rng.integers(1, 5))
    Hkv = int(rng.choice([1, 2, 3, 8]))
    D = int(rng.choice([64, 128]))
    n_req = int(rng.integers(1, 6))
    toks = [int(rng.integers(1, 700)) for _ in range(n_req)]
    ranges = []
    for r, n in enumerate(toks):
        if rng.random() < 0.85:
            lo = int(rng.integers(0, n))
            hi = int(rng.integers(lo + 1, n + 1))
            ranges.append((r, lo, hi))
    if not ranges:
        ranges.append((0, 0, toks[0]))
    chunk = int(rng.choice([1, 3, 16, 17, 64, 100, 256, 512]))
    return gen.make_handoff("rh%d" % seed, 8000 + seed, L, Hkv, D, toks, ranges, chunk)


@pytest.mark.parametrize("seed", range(16))
def test_random_handoff(seed):
    from test_gpu_handoff import check
    check(random_handoff(seed))


@pytest.mark.parametrize("seed", range(12))
def test_random_append_bf16_and_8bit(seed):
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import dev_bf16, dev_u8, host_u16
    rng = np.random.default_rng(3000 + seed)
    Hkv = int(rng.choice([1, 2, 3, 8]))
    D = int(rng.choice([64, 128]))
    segs = []
    for _ in range(int(rng.integers(1, 9))):
        q = int(rng.choice([1, 1, 2, 15, 16, 17, 64, 130]))
        segs.append((q, q + int(rng.integers(0, 500))))
    ks, vs = float(rng.choice([1.0, 0.37, 0.011, 3.0])), float(rng.choice([1.0, 0.02, 0.5]))
    b = gen.make_batch("ra%d" % seed, 9000 + seed, Hkv, Hkv, D, segs)
    b8 = gen.make_batch_fp8kv("ra8_%d" % seed, 9000 + seed, Hkv, Hkv, D, segs)
    k_new = gen.normal_bf16(9000 + seed, 31, (b.total_q, Hkv, D))
    v_new = gen.normal_bf16(9000 + seed, 32, (b.total_q, Hkv, D))
    bt = torch.from_numpy(b.block_tables).cuda()
    qo, cl = torch.from_numpy(b.q_offsets).cuda(), torch.from_numpy(b.ctx_lens).cuda()
    # bf16 cache
    want_k, want_v = b.k_pool.copy(), b.v_pool.copy()
    oracle.kv_append(k_new, v_new, want_k, want_v, b.block_tables, b.q_offsets, b.ctx_lens)
    pool = dsv.KVPool(dev_bf16(b.k_pool[None]), dev_bf16(b.v_pool[None]))
    dsv.kv_append(dev_bf16(k_new), dev_bf16(v_new), pool, 0, bt, qo, cl, b.q_offsets, b.ctx_lens)
    # 8-bit cache
    want_k8, want_v8 = b8.k_pool.copy(), b8.v_pool.copy()
    oracle.kv_append_fp8(k_new, v_new, want_k8, want_v8, b8.block_tables, b8.q_offsets, b8.ctx_lens, ks, vs)
    pool8 = dsv.KVPool(dev_u8(b8.k_pool[None]), dev_u8(b8.v_pool[None]))
    bt8 = torch.from_numpy(b8.block_tables).cuda()
    dsv.kv_append_fp8(dev_bf16(k_new), dev_bf16(v_new), pool8, 0, bt8, qo, cl, b8.q_offsets, b8.ctx_lens, ks, vs)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host_u16(pool.k)[0], want_k)
    np.testing.assert_array_equal(host_u16(pool.v)[0], want_v)
    np.testing.assert_array_equal(pool8.k.cpu().numpy()[0], want_k8)
    np.testing.assert_array_equal(pool8.v.cpu().numpy()[0], want_v8)
