"""GPU parity of kv_pack_chunks / kv_unpack_chunks against the CPU oracle: bit-exact, through
the C ABI, on the same seeded inputs."""
import numpy as np
import pytest

import oracle
from workloads import gen

pytestmark = pytest.mark.gpu


def oracle_handoff(h):
    buf = np.full(max(h.chunk_elems, 8), np.uint16(-21555 & 0xFFFF), np.uint16)
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, h.chunks, buf)
    dk, dv = h.dst_k.copy(), h.dst_v.copy()
    oracle.kv_unpack_chunks(buf, h.chunks, dk, dv, h.dst_tables)
    return buf, dk, dv


def check(h):
    import torch
    from gpu_harness import DeviceHandoff, host_u16
    d = DeviceHandoff(h)
    d.pack()
    d.unpack()
    torch.cuda.synchronize()
    buf, dk, dv = oracle_handoff(h)
    np.testing.assert_array_equal(host_u16(d.chunk_buf), buf)
    np.testing.assert_array_equal(host_u16(d.dst.k), dk)
    np.testing.assert_array_equal(host_u16(d.dst.v), dv)
    np.testing.assert_array_equal(host_u16(d.src.k), h.src_k)      # source untouched


def test_config1_handoff():
    _, h = gen.config1()
    check(h)


@pytest.mark.parametrize("L,Hkv,D,toks,ranges,chunk", [
    (3, 2, 64, (50, 17, 96), ((0, 3, 47), (1, 0, 17), (2, 16, 96)), 20),     # unaligned, short last chunks
    (2, 8, 128, (300, 1, 33), ((0, 0, 300), (1, 0, 1), (2, 5, 33)), 64),     # several tiles, 1-token chunk
    (1, 3, 128, (70,), ((0, 1, 70),), 7),                                    # row size not a power of two
    (4, 8, 128, (1024, 777), ((0, 0, 1024), (1, 13, 777)), 256),             # full-size rows, 256-token chunks
])
def test_handoff_shapes(L, Hkv, D, toks, ranges, chunk):
    check(gen.make_handoff("t", 41, L, Hkv, D, list(toks), list(ranges), chunk))


def test_config5_handoff_shrunk():
    check(gen.config5_handoff(shrink=16, layers=4))


def test_chunk_order_and_subsets_do_not_matter():
    """Chunks are independent units (section 4.3): packing/unpacking them in two calls, in reverse
    order, gives the same destination image."""
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceHandoff, host_u16
    h = gen.make_handoff("t", 43, 2, 8, 128, [200, 90], [(0, 0, 200), (1, 10, 90)], 48)
    d = DeviceHandoff(h)
    rev = h.chunks[::-1].copy()
    for part in (rev[: len(rev) // 2], rev[len(rev) // 2:]):
        descs = dsv.ChunkDescs(part)
        dsv.kv_pack_chunks(d.src, d.src_tables, descs, d.chunk_buf)
        dsv.kv_unpack_chunks(d.chunk_buf, descs, d.dst, d.dst_tables)
    torch.cuda.synchronize()
    _, dk, dv = oracle_handoff(h)
    np.testing.assert_array_equal(host_u16(d.dst.k), dk)
    np.testing.assert_array_equal(host_u16(d.dst.v), dv)


def test_empty_and_invalid():
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceHandoff
    h = gen.make_handoff("t", 44, 1, 2, 64, [40], [(0, 0, 40)], 16)
    d = DeviceHandoff(h)
    dsv.kv_pack_chunks(d.src, d.src_tables, dsv.ChunkDescs(np.zeros((0, 4))), d.chunk_buf)   # no-op
    bad = h.chunks.copy()
    bad[0, 1] = 16 * h.src_tables.shape[1]
    with pytest.raises(dsv.DsvError) as e:
        dsv.kv_pack_chunks(d.src, d.src_tables, dsv.ChunkDescs(bad), d.chunk_buf)
    assert e.value.code == -1
    bad = h.chunks.copy()
    bad[0, 3] = 4                      # misaligned chunk offset
    with pytest.raises(dsv.DsvError):
        dsv.kv_pack_chunks(d.src, d.src_tables, dsv.ChunkDescs(bad), d.chunk_buf)


@pytest.mark.timeout(1200)
def test_config5_handoff_full_size():
    """Config 5's hand-off at full size: 8 requests x 8192 tokens x 32 layers (8.59 GB payload) in
    256-token chunks from one paged pool into another with a different block table.  The copied
    bytes are compared layer by layer; untouched destination blocks must keep their bytes."""
    import torch
    from gpu_harness import DeviceHandoff, host_u16
    h = gen.config5_handoff(threads=16)
    assert h.L == 32 and h.chunks.shape[0] == 256 and h.payload_bytes == 8 * 8192 * 32 * 4096
    d = DeviceHandoff(h)
    d.pack()
    d.unpack()
    torch.cuda.synchronize()
    buf = np.zeros(h.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, h.chunks, buf)
    assert np.array_equal(host_u16(d.chunk_buf), buf)
    oracle.kv_unpack_chunks(buf, h.chunks, h.dst_k, h.dst_v, h.dst_tables)      # in place: h.dst_* now expected
    for l in range(h.L):
        assert np.array_equal(host_u16(d.dst.k[l]), h.dst_k[l]), l
        assert np.array_equal(host_u16(d.dst.v[l]), h.dst_v[l]), l


def test_an_error_left_by_an_unrelated_hip_call_is_not_reported_as_a_failed_launch():
    """The calling thread's HIP last-error state may hold an error from a call that has nothing to
    do with this library (here: the elapsed time of two events that were never recorded, a
    host-side error).  Every entry point must still do its work and return success."""
    import ctypes as C

    import torch

    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceBatch, DeviceHandoff, host_u16, loaded_hip_runtime
    hip = loaded_hip_runtime()
    hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
    hip.hipEventDestroy.argtypes = [C.c_void_p]
    e0, e1 = C.c_void_p(), C.c_void_p()
    assert hip.hipEventCreate(C.byref(e0)) == 0 and hip.hipEventCreate(C.byref(e1)) == 0

    def leave_an_error():
        ms = C.c_float()
        assert hip.hipEventElapsedTime(C.byref(ms), e0, e1) != 0

    b, h = gen.config1()
    d = DeviceHandoff(h)
    torch.cuda.synchronize()
    leave_an_error()
    d.pack()
    leave_an_error()
    d.unpack()
    db = DeviceBatch(b)
    k_new = db.q[:, :b.Hkv].contiguous()         # (torch's own launches do not survive a planted error)
    out = torch.empty(db.q.shape, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    leave_an_error()
    dsv.attn_mixed_batch(db.q, out, db.pool, 0, db.block_tables, db.q_offsets, db.ctx_lens, b.q_offsets,
                         b.ctx_lens, b.Hq, b.scale, db.workspace)
    leave_an_error()
    dsv.kv_append(k_new, k_new, db.pool, 0, db.block_tables, db.q_offsets, db.ctx_lens, b.q_offsets,
                  b.ctx_lens)
    hip.hipGetLastError()                        # leave the thread clean for torch
    torch.cuda.synchronize()
    buf, dk, dv = oracle_handoff(h)
    np.testing.assert_array_equal(host_u16(d.chunk_buf), buf)
    np.testing.assert_array_equal(host_u16(d.dst.k), dk)
    ref = oracle.attn_mixed_batch(b.q, b.k_pool, b.v_pool, b.block_tables, b.q_offsets, b.ctx_lens, b.scale)
    assert np.abs(out.cpu().numpy() - ref).max() <= 1e-2
    hip.hipEventDestroy(e0)
    hip.hipEventDestroy(e1)


# ------------------------------------------------------------------ unpack in destination order
def _unpack_ordered_check(h, expect_same_as_plain=True):
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceHandoff, host_u16
    d = DeviceHandoff(h)
    d.pack()
    ws = torch.full((dsv.kv_unpack_chunks_ordered_workspace_bytes(d.dst.NB) // 8,), -7, dtype=torch.int64, device="cuda")
    dsv.kv_unpack_chunks_ordered(d.chunk_buf, d.descs, d.dst, d.dst_tables, ws)
    torch.cuda.synchronize()
    buf, dk, dv = oracle_handoff(h)
    np.testing.assert_array_equal(host_u16(d.chunk_buf), buf)
    np.testing.assert_array_equal(host_u16(d.dst.k), dk)          # every byte of the pool: copied and untouched alike
    np.testing.assert_array_equal(host_u16(d.dst.v), dv)
    return d


@pytest.mark.parametrize("L,Hkv,D", [(3, 8, 128), (2, 1, 64), (1, 3, 128)])
def test_unpack_in_destination_order_dense_pool(L, Hkv, D):
    """Chunks on block boundaries that fill most of the destination pool: the ordered sweep runs.
    Requests of ragged length (last chunks and last blocks short), 48-token chunks."""
    req = [200, 77, 16, 1000, 333, 48]
    h = gen.make_handoff("ord_dense", 51 + D, L, Hkv, D, req, [(r, 0, n) for r, n in enumerate(req)], 48, free_frac=0.05)
    assert (h.chunks[:, 1] % 16 == 0).all()
    assert 2 * sum(-(-int(n) // 16) for n in h.chunks[:, 2]) >= h.dst_k.shape[1]
    _unpack_ordered_check(h)


def test_unpack_in_destination_order_config5_geometry():
    _unpack_ordered_check(gen.config5_handoff(shrink=8, layers=3))


def test_unpack_ordered_falls_back_for_sparse_or_unaligned_hand_offs():
    """A pool mostly untouched by the hand-off, and chunks that start inside blocks: the call runs
    the plain unpack and gives the same bytes."""
    req = [300, 90, 500]
    sparse = gen.make_handoff("ord_sparse", 52, 2, 2, 64, req, [(r, 0, n) for r, n in enumerate(req)], 64, free_frac=3.0)
    _unpack_ordered_check(sparse)
    unaligned = gen.make_handoff("ord_unaligned", 53, 2, 2, 64, req, [(0, 5, 290), (1, 17, 80), (2, 0, 500)], 40,
                                 free_frac=0.05)
    assert (unaligned.chunks[:, 1] % 16 != 0).any()
    _unpack_ordered_check(unaligned)


def test_unpack_ordered_refuses_a_short_workspace():
    import torch
    import paper_2504_09285_amd as dsv
    from gpu_harness import DeviceHandoff
    h = gen.make_handoff("ord_ws", 54, 1, 2, 64, [64], [(0, 0, 64)], 32)
    d = DeviceHandoff(h)
    ws = torch.zeros(1, dtype=torch.int64, device="cuda")
    with pytest.raises(dsv.DsvError) as e:
        dsv.kv_unpack_chunks_ordered(d.chunk_buf, d.descs, d.dst, d.dst_tables, ws)
    assert e.value.code == -3
