"""Hand-off on a second HIP stream while attention runs on the first (paper section 4.3: completed
KV is immutable, so chunks are shipped while computation continues).  Both results are checked
against the oracle, and the attention result must equal the one obtained without the concurrent
copy."""
import numpy as np
import pytest

import oracle
from workloads import gen

pytestmark = pytest.mark.gpu


def test_handoff_overlaps_attention_on_two_streams():
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceBatch, DeviceHandoff, host_u16
    b = gen.config5_attention(shrink=16)                   # 4 decodes, contexts 1K..8K
    h = gen.config5_handoff(shrink=8, layers=8)            # 2 requests x 1024 tokens x 8 layers, 256-token chunks
    d, dh = DeviceBatch(b), DeviceHandoff(h)
    alone = d.run().cpu().numpy()
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for _ in range(3):                                      # several rounds so the two streams really interleave
        with torch.cuda.stream(s1):
            outs.append(d.run(stream=s1))
        with torch.cuda.stream(s2):
            dh.pack(stream=s2)
            dh.unpack(stream=s2)
    torch.cuda.synchronize()
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    for o in outs:
        o = o.cpu().numpy()
        np.testing.assert_array_equal(o, alone)
        assert np.abs(o - ref).max() <= 1e-2
    buf = np.zeros(h.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, h.chunks, buf)
    dk, dv = h.dst_k.copy(), h.dst_v.copy()
    oracle.kv_unpack_chunks(buf, h.chunks, dk, dv, h.dst_tables)
    np.testing.assert_array_equal(host_u16(dh.chunk_buf), buf)
    np.testing.assert_array_equal(host_u16(dh.dst.k), dk)
    np.testing.assert_array_equal(host_u16(dh.dst.v), dv)


@pytest.mark.timeout(1500)
def test_config5_at_its_stated_size_on_two_streams():
    """Config 5 as stated: attention over 64 contexts of 16K-128K tokens on one stream while, on a
    second stream, 8 requests x 8,192 tokens x 32 layers (8.59 GB) are packed into 256-token
    chunks and unpacked into a second pool with another block table.  The event times must show
    the two streams' work overlapping; every attention output and every copied byte is compared
    with the oracle, and the attention result must equal the one obtained with the GPU to itself."""
    import torch
    from gpu_harness import DeviceBatch, DeviceHandoff, host_u16
    b = gen.config5_attention(threads=16)
    h = gen.config5_handoff(threads=16)
    assert b.num_seqs == 64 and h.L == 32 and h.chunks.shape[0] == 256
    assert h.payload_bytes == 8 * 8192 * 32 * 4096
    d, dh = DeviceBatch(b), DeviceHandoff(h)
    alone = d.run(fill=float("nan")).cpu().numpy()
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    ev = {k: torch.cuda.Event(enable_timing=True) for k in ("a0", "a1", "c0", "c1", "origin")}
    ev["origin"].record()
    torch.cuda.synchronize()
    outs = []
    with torch.cuda.stream(s2):
        ev["c0"].record(s2)
        dh.pack(stream=s2)
        dh.unpack(stream=s2)
        ev["c1"].record(s2)
    with torch.cuda.stream(s1):
        ev["a0"].record(s1)
        for _ in range(3):                                  # three steps fit inside one hand-off
            outs.append(d.run(stream=s1, fill=float("nan")))
        ev["a1"].record(s1)
    torch.cuda.synchronize()
    t = {k: ev["origin"].elapsed_time(ev[k]) for k in ("a0", "a1", "c0", "c1")}
    assert t["a0"] < t["c1"] and t["c0"] < t["a1"], t          # the two intervals intersect
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    for o in outs:
        o = o.cpu().numpy()
        np.testing.assert_array_equal(o, alone)
        assert np.abs(o - ref).max() <= 1e-2
    buf = np.zeros(h.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, h.chunks, buf)
    assert np.array_equal(host_u16(dh.chunk_buf), buf)
    oracle.kv_unpack_chunks(buf, h.chunks, h.dst_k, h.dst_v, h.dst_tables)      # in place: h.dst_* now expected
    for l in range(h.L):
        assert np.array_equal(host_u16(dh.dst.k[l]), h.dst_k[l]), l
        assert np.array_equal(host_u16(dh.dst.v[l]), h.dst_v[l]), l


def test_pack_reads_the_pool_attention_is_reading():
    """Pack may read the very pool (and blocks) an attention call is reading at the same time:
    read-read sharing of immutable KV.  Config 1 geometry: the hand-off source is the batch pool."""
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceBatch, dev_bf16, host_u16
    b, h = gen.config1()
    d = DeviceBatch(b)
    descs = dsv.ChunkDescs(h.chunks)
    buf = torch.zeros(h.chunk_elems, dtype=torch.bfloat16, device="cuda")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s1):
        out = d.run(stream=s1)
    with torch.cuda.stream(s2):
        dsv.kv_pack_chunks(d.pool, d.block_tables, descs, buf, stream=s2)
    torch.cuda.synchronize()
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.abs(out.cpu().numpy() - ref).max() <= 1e-2
    obuf = np.zeros(h.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, h.chunks, obuf)
    np.testing.assert_array_equal(host_u16(buf), obuf)
