"""The entry points under HIP graph capture: kv_append + attn_mixed_batch recorded once on a side
stream and replayed.  The library allocates nothing and synchronises nothing on that path, and
clears its work lists with its own kernels, so a replay must give what the eager call gives.
Every replay is checked (against the eager result bit for bit and against the oracle), with
eager work of the same library and synchronisations between the replays; the device-side inputs
are changed between two replays to show that a replay reads them afresh.  What is frozen at
capture is what the host decides from the host-side lists: grid sizes and the workspace layout."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_09285_amd as dsv
from gpu_harness import DeviceBatch, dev_bf16
from workloads import gen

pytestmark = pytest.mark.gpu


def dev_u16(a):
    return dev_bf16(a)


def test_append_and_attention_replayed_from_a_graph():
    # decodes whose context is split into partitions (merge kernel), prefill spans (MFMA tiles),
    # short spans on either path
    segs = [(150, 260), (1, 2000), (1, 33), (40, 40), (1, 700), (5, 300), (1, 1500), (9, 9)]
    b = gen.make_batch("graph_capture", 4242, 32, 8, 128, segs)
    other = DeviceBatch(gen.make_batch("graph_other", 4243, 32, 8, 128, [(1, 900), (70, 70), (1, 17)]))

    # the new tokens' K/V are cut out of the pool and appended by the captured call
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
    poisoned_k, poisoned_v = dev_u16(kp[None]), dev_u16(vp[None])
    pool = dsv.KVPool(poisoned_k.clone(), poisoned_v.clone())
    bt = torch.from_numpy(np.ascontiguousarray(b.block_tables, dtype=np.int32)).cuda()
    qo, cl = torch.from_numpy(b.q_offsets).cuda(), torch.from_numpy(b.ctx_lens).cuda()
    q = dev_u16(b.q)
    dk, dv = dev_u16(k_new), dev_u16(v_new)
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(dsv.attn_mixed_batch_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D),
                     dtype=torch.uint8, device="cuda")

    def step(stream):
        dsv.kv_append(dk, dv, pool, 0, bt, qo, cl, b.q_offsets, b.ctx_lens, stream=stream)
        dsv.attn_mixed_batch(q, out, pool, 0, bt, qo, cl, b.q_offsets, b.ctx_lens, b.Hq, b.scale, ws,
                             stream=stream)

    def reset():
        pool.k.copy_(poisoned_k)
        pool.v.copy_(poisoned_v)
        out.fill_(float("nan"))
        ws.fill_(0xA5)                           # whatever the last call left is not relied upon

    s = torch.cuda.Stream()
    reset()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        step(s)                                  # eager: first-call set-up happens outside the capture
    torch.cuda.synchronize()
    eager = out.clone()
    ref = oracle.attn_mixed_batch(q=b.q, k_pool=b.k_pool, v_pool=b.v_pool, block_tables=b.block_tables,
                                  q_offsets=b.q_offsets, ctx_lens=b.ctx_lens, scale=b.scale)
    assert np.abs(eager.cpu().numpy() - ref).max() <= 1e-2

    g = torch.cuda.CUDAGraph()
    reset()
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        step(s)
    torch.cuda.synchronize()

    for rep in range(4):
        reset()
        other.run()                              # the library's own eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = out.clone()
        assert torch.equal(got, eager), f"replay {rep} differs from the eager call"
        assert torch.equal(pool.k.view(torch.int16), dev_u16(b.k_pool[None]).view(torch.int16))
        assert np.abs(got.cpu().numpy() - ref).max() <= 1e-2

    # new query values on the device: the same graph must follow them
    q2 = gen.make_batch("graph_capture_q2", 777, 32, 8, 128, segs).q
    q.copy_(dev_u16(q2))
    reset()
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    ref2 = oracle.attn_mixed_batch(q=q2, k_pool=b.k_pool, v_pool=b.v_pool, block_tables=b.block_tables,
                                   q_offsets=b.q_offsets, ctx_lens=b.ctx_lens, scale=b.scale)
    got2 = out.cpu().numpy()
    assert np.isfinite(got2).all() and np.abs(got2 - ref2).max() <= 1e-2
    assert np.abs(ref2 - ref).max() > 0.05       # the two query sets really differ
