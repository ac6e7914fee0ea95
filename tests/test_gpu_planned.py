"""One plan for all layers: attn_mixed_batch_plan builds the work lists of a batch once, and the
planned calls run single layers on them.  The result of a planned call must equal, bit for bit,
what the full call gives for the same layer (same kernels, same lists), and the oracle within
the attention tolerance; planned calls whose arguments do not match the plan are refused."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_09285_amd as dsv
from gpu_harness import dev_bf16, dev_u8
from workloads import gen

pytestmark = pytest.mark.gpu
TOL = 1e-2
SEGS = [(150, 260), (1, 2000), (1, 33), (40, 40), (1, 700), (5, 300), (1, 1500), (9, 9), (300, 1324)]


def _device_lists(b):
    bt = torch.from_numpy(np.ascontiguousarray(b.block_tables, dtype=np.int32)).cuda()
    return bt, torch.from_numpy(b.q_offsets).cuda(), torch.from_numpy(b.ctx_lens).cuda()


def test_one_plan_serves_every_layer_bf16():
    b = gen.make_batch("planned", 515, 32, 8, 128, SEGS)
    layers = 3
    k_layers = np.stack([np.roll(b.k_pool, l, axis=0) for l in range(layers)])
    v_layers = np.stack([np.roll(b.v_pool, 2 * l, axis=0) for l in range(layers)])
    pool = dsv.KVPool(dev_bf16(k_layers), dev_bf16(v_layers))
    bt, qo, cl = _device_lists(b)
    q = dev_bf16(b.q)
    nbytes = dsv.attn_mixed_batch_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
    ws_full = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ws_plan = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")

    full = []
    for l in range(layers):
        out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
        dsv.attn_mixed_batch(q, out, pool, l, bt, qo, cl, b.q_offsets, b.ctx_lens, b.Hq, b.scale, ws_full)
        full.append(out)
    plan = dsv.attn_mixed_batch_plan(bt, qo, cl, b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D, ws_plan)
    planned = []
    for l in (2, 0, 1, 2):                        # any order, a layer twice
        out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
        dsv.attn_mixed_batch_planned(plan, q, out, pool, l, bt, qo, cl, b.q_offsets, b.ctx_lens, b.Hq,
                                     b.scale, ws_plan)
        planned.append((l, out))
    torch.cuda.synchronize()
    for l, out in planned:
        assert torch.equal(out, full[l]), f"layer {l}: planned call differs from the full call"
    ref = oracle.attn_mixed_batch(q=b.q, k_pool=k_layers[1], v_pool=v_layers[1], block_tables=b.block_tables,
                                  q_offsets=b.q_offsets, ctx_lens=b.ctx_lens, scale=b.scale)
    got = full[1].cpu().numpy()
    assert np.isfinite(got).all() and np.abs(got - ref).max() <= TOL


def test_one_plan_serves_every_layer_fp8kv():
    b = gen.make_batch_fp8kv("planned8", 516, 32, 8, 128, SEGS)
    ks, vs = b.meta["k_scale"], b.meta["v_scale"]
    layers = 2
    k_layers = np.stack([np.roll(b.k_pool, l, axis=0) for l in range(layers)])
    v_layers = np.stack([np.roll(b.v_pool, 3 * l, axis=0) for l in range(layers)])
    pool = dsv.KVPool(dev_u8(k_layers), dev_u8(v_layers))
    bt, qo, cl = _device_lists(b)
    q = dev_bf16(b.q)
    nbytes = dsv.attn_mixed_batch_fp8kv_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
    ws_full = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ws_plan = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device="cuda")
    full = []
    for l in range(layers):
        out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
        dsv.attn_mixed_batch_fp8kv(q, out, pool, l, bt, qo, cl, b.q_offsets, b.ctx_lens, b.Hq, b.scale,
                                   ks, vs, ws_full)
        full.append(out)
    plan = dsv.attn_mixed_batch_plan(bt, qo, cl, b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D, ws_plan,
                                     kv_elem_bytes=1)
    for l in (1, 0):
        out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
        dsv.attn_mixed_batch_fp8kv_planned(plan, q, out, pool, l, bt, qo, cl, b.q_offsets, b.ctx_lens,
                                           b.Hq, b.scale, ks, vs, ws_plan)
        torch.cuda.synchronize()
        assert torch.equal(out, full[l]), f"layer {l}: planned call differs from the full call"
    ref = oracle.attn_mixed_batch_fp8kv(q=b.q, k_pool=k_layers[1], v_pool=v_layers[1],
                                        block_tables=b.block_tables, q_offsets=b.q_offsets,
                                        ctx_lens=b.ctx_lens, scale=b.scale, k_scale=ks, v_scale=vs)
    got = full[1].cpu().numpy()
    assert np.isfinite(got).all() and np.abs(got - ref).max() <= TOL


def test_planned_call_refuses_what_the_plan_was_not_made_for():
    b = gen.make_batch("planned_bad", 517, 16, 4, 64, [(1, 300), (20, 50), (1, 77)])
    pool = dsv.KVPool(dev_bf16(b.k_pool[None]), dev_bf16(b.v_pool[None]))
    bt, qo, cl = _device_lists(b)
    q = dev_bf16(b.q)
    out = torch.zeros(q.shape, dtype=torch.float32, device="cuda")
    nbytes = dsv.attn_mixed_batch_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    other_ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    plan = dsv.attn_mixed_batch_plan(bt, qo, cl, b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D, ws)

    def planned(**over):
        a = dict(plan=plan, q=q, out=out, pool=pool, layer=0, block_tables=bt, q_offsets=qo, ctx_lens=cl,
                 q_offsets_host=b.q_offsets, ctx_lens_host=b.ctx_lens, num_q_heads=b.Hq,
                 softmax_scale=b.scale, workspace=ws)
        a.update(over)
        dsv.attn_mixed_batch_planned(**a)

    planned()                                                        # as planned: accepted
    longer = b.ctx_lens.copy()
    longer[0] -= 1                                                   # another batch (still valid)
    for over in (dict(ctx_lens_host=longer), dict(workspace=other_ws), dict(ctx_lens=cl.clone()),
                 dict(block_tables=bt.clone()), dict(plan=dsv.AttnPlan())):
        with pytest.raises(dsv.DsvError) as e:
            planned(**over)
        assert e.value.code == -1, over.keys()
    # a plan for 1-byte elements does not serve the bf16 call
    plan8 = dsv.attn_mixed_batch_plan(bt, qo, cl, b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D,
                                      torch.empty(dsv.attn_mixed_batch_fp8kv_workspace_bytes(
                                          b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D), dtype=torch.uint8,
                                          device="cuda"), kv_elem_bytes=1)
    with pytest.raises(dsv.DsvError):
        planned(plan=plan8)
    torch.cuda.synchronize()
    ref = oracle.attn_mixed_batch(q=b.q, k_pool=b.k_pool, v_pool=b.v_pool, block_tables=b.block_tables,
                                  q_offsets=b.q_offsets, ctx_lens=b.ctx_lens, scale=b.scale)
    assert np.abs(out.cpu().numpy() - ref).max() <= TOL              # the refused calls left it alone
