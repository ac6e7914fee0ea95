"""attn_mixed_batch_static: the entry point for callers that cannot allocate (no workspace
argument; the library's own fixed device array holds work lists and partials).  It must give
what attn_mixed_batch gives, call after call, with the array keeping the previous call's
contents: here a larger batch first, then a smaller one, each compared with attn_mixed_batch on
the same inputs (same kernels, same lists: bit for bit) and with the oracle."""
import numpy as np
import pytest

import oracle
from workloads import gen

pytestmark = pytest.mark.gpu
TOL = 1e-2


def _both(b, out_dtype):
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceBatch
    d = DeviceBatch(b)
    want = d.run(out_dtype, fill=float("nan"))
    got = torch.full(d.q.shape, float("nan"), dtype=out_dtype, device="cuda")
    dsv.attn_mixed_batch_static(d.q, got, d.pool, 0, d.block_tables, d.q_offsets, d.ctx_lens,
                                b.q_offsets, b.ctx_lens, b.Hq, b.scale)
    torch.cuda.synchronize()
    return got, want


def test_two_calls_in_a_row_the_second_smaller():
    import torch
    import paper_2504_09285_amd as dsv
    assert dsv.attn_mixed_batch_static_max_bytes() == 64 << 20
    # First: prefill spans (one cut along its context), short spans on the row path, and decodes
    # whose contexts are split into several partitions, so work lists, partials of split rows and
    # partials of cut query tiles all land in the array.
    big = gen.make_batch("static_big", 701, 32, 8, 128,
                         [(300, 700), (1, 5000), (70, 9000), (1, 1), (3, 40), (1, 2500), (1, 17), (9, 2000)])
    # Second: fewer and shorter segments; the array still holds the first call's lists.
    small = gen.make_batch("static_small", 702, 32, 8, 128, [(1, 1300), (40, 90), (1, 33), (2, 2)])
    for b in (big, small):
        need = dsv.attn_mixed_batch_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
        assert 0 < need <= dsv.attn_mixed_batch_static_max_bytes()
        ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
        got, want = _both(b, torch.float32)
        got, want = got.cpu().numpy(), want.cpu().numpy()
        assert np.isfinite(got).all()
        np.testing.assert_array_equal(got, want)
        assert np.abs(got - ref).max() <= TOL
    # bf16 output through the same path
    got, want = _both(small, torch.bfloat16)
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))


def test_a_batch_beyond_the_fixed_array_is_refused_before_any_work():
    """4,096 decodes with 64 query heads need more partial-result space than the array holds: the
    call returns DSV_E_WORKSPACE and leaves the output untouched."""
    import torch
    import paper_2504_09285_amd as dsv
    n, ctx, Hq, Hkv, D = 4096, 4096, 64, 8, 128
    q_offsets = np.arange(n + 1, dtype=np.int32)
    ctx_lens = np.full(n, ctx, np.int32)
    assert dsv.attn_mixed_batch_workspace_bytes(q_offsets, ctx_lens, Hq, Hkv, D) > dsv.attn_mixed_batch_static_max_bytes()
    nblk = ctx // 16
    # The pool is never read (the call is refused on the host): one block stands in for all.
    k = torch.zeros((1, 1, 16, Hkv, D), dtype=torch.bfloat16, device="cuda")
    pool = dsv.KVPool(k, k.clone())
    bt = torch.zeros((n, nblk), dtype=torch.int32, device="cuda")
    q = torch.zeros((n, Hq, D), dtype=torch.bfloat16, device="cuda")
    out = torch.full((n, Hq, D), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(dsv.DsvError) as e:
        dsv.attn_mixed_batch_static(q, out, pool, 0, bt, torch.from_numpy(q_offsets).cuda(),
                                    torch.from_numpy(ctx_lens).cuda(), q_offsets, ctx_lens, Hq, 0.1)
    assert e.value.code == -3
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
