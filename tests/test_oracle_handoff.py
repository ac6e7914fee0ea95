"""Pins for the chunked KV hand-off oracle (paper section 4.3): numpy fancy-indexing gathers
written here independently, identities and chunk-boundary independence.  CPU only."""
import numpy as np
import pytest

import oracle
from workloads import gen


def small_handoff(seed=31, L=3, Hkv=2, D=8, toks=(50, 17, 96), chunk=20,
                  ranges=((0, 3, 47), (1, 0, 17), (2, 16, 96))):
    return gen.make_handoff("small", seed, L, Hkv, D, list(toks), list(ranges), chunk)


def gather_tokens(pool, table_row, t0, t1):
    """[L, t1-t0, Hkv, D] via numpy indexing (independent of the oracle's loops)."""
    t = np.arange(t0, t1)
    return pool[:, table_row[t // 16], t % 16]


def covered_mask(h, tables, nb):
    m = np.zeros((nb, 16), bool)
    for seq, tb, n, _ in h.chunks:
        t = np.arange(tb, tb + n)
        m[tables[seq, t // 16], t % 16] = True
    return m


def test_pack_matches_numpy_gather():
    h = small_handoff()
    buf = np.full(h.chunk_elems, 0xDEAD, np.uint16)
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, h.chunks, buf)
    row = h.Hkv * h.D
    for seq, tb, n, off in h.chunks:
        c = buf[off:off + 2 * h.L * n * row].reshape(h.L, 2, n, h.Hkv, h.D)
        np.testing.assert_array_equal(c[:, 0], gather_tokens(h.src_k, h.src_tables[seq], tb, tb + n))
        np.testing.assert_array_equal(c[:, 1], gather_tokens(h.src_v, h.src_tables[seq], tb, tb + n))
    assert not (buf == 0xDEAD).all()


def test_chunk_sizes_and_offsets():
    h = small_handoff()
    # (0,3,47): 20,20,4 ; (1,0,17): 17 ; (2,16,96): 20,20,20,20
    assert h.chunks[:, 2].tolist() == [20, 20, 4, 17, 20, 20, 20, 20]
    assert h.chunks[:, 1].tolist() == [3, 23, 43, 0, 16, 36, 56, 76]
    per_tok = 2 * h.L * h.Hkv * h.D
    assert h.chunks[:, 3].tolist() == (np.concatenate([[0], np.cumsum(h.chunks[:, 2])[:-1]]) * per_tok).tolist()
    assert h.chunk_elems == int(h.chunks[:, 2].sum()) * per_tok


def test_unpack_pack_identity_same_table():
    h = small_handoff()
    buf = np.zeros(h.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, h.chunks, buf)
    k2, v2 = h.src_k.copy(), h.src_v.copy()
    m = covered_mask(h, h.src_tables, h.src_k.shape[1])
    k2[:, m] = 0
    v2[:, m] = 0
    oracle.kv_unpack_chunks(buf, h.chunks, k2, v2, h.src_tables)
    np.testing.assert_array_equal(k2, h.src_k)
    np.testing.assert_array_equal(v2, h.src_v)


def test_unpack_into_different_table_moves_tokens_and_touches_nothing_else():
    h = small_handoff()
    buf = np.zeros(h.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, h.chunks, buf)
    dk, dv = h.dst_k.copy(), h.dst_v.copy()
    oracle.kv_unpack_chunks(buf, h.chunks, dk, dv, h.dst_tables)
    for seq, tb, n, _ in h.chunks:
        np.testing.assert_array_equal(gather_tokens(dk, h.dst_tables[seq], tb, tb + n),
                                      gather_tokens(h.src_k, h.src_tables[seq], tb, tb + n))
        np.testing.assert_array_equal(gather_tokens(dv, h.dst_tables[seq], tb, tb + n),
                                      gather_tokens(h.src_v, h.src_tables[seq], tb, tb + n))
    m = covered_mask(h, h.dst_tables, dk.shape[1])
    assert m.sum() == int(h.chunks[:, 2].sum())
    np.testing.assert_array_equal(dk[:, ~m], h.dst_k[:, ~m])
    np.testing.assert_array_equal(dv[:, ~m], h.dst_v[:, ~m])
    assert (dk[:, m] != h.dst_k[:, m]).any()


def test_chunk_boundary_independence():
    """pack [a,b) == pack [a,m) ++ pack [m,b) per (layer, K|V), for every m."""
    L, Hkv, D = 2, 2, 8
    a, b = 5, 44
    base = gen.make_handoff("cb", 33, L, Hkv, D, [60], [(0, a, b)], 1000)
    whole = np.zeros(base.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(base.src_k, base.src_v, base.src_tables, base.chunks, whole)
    whole = whole.reshape(L, 2, b - a, Hkv, D)
    for m in range(a + 1, b):
        chunks, n_el = gen.make_chunks([(0, a, m), (0, m, b)], 1000, L, Hkv, D)
        buf = np.zeros(n_el, np.uint16)
        oracle.kv_pack_chunks(base.src_k, base.src_v, base.src_tables, chunks, buf)
        c0 = buf[:chunks[1, 3]].reshape(L, 2, m - a, Hkv, D)
        c1 = buf[chunks[1, 3]:].reshape(L, 2, b - m, Hkv, D)
        np.testing.assert_array_equal(np.concatenate([c0, c1], axis=2), whole)


def test_k_and_v_and_layers_are_not_mixed_up():
    """K plane of layer l holds K of layer l, V plane holds V: tag pools with distinct constants."""
    L, Hkv, D = 3, 1, 8
    h = gen.make_handoff("tag", 34, L, Hkv, D, [40], [(0, 7, 33)], 13)
    k = np.empty_like(h.src_k)
    v = np.empty_like(h.src_v)
    for l in range(L):
        k[l] = 100 + l
        v[l] = 200 + l
    buf = np.zeros(h.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(k, v, h.src_tables, h.chunks, buf)
    for seq, tb, n, off in h.chunks:
        c = buf[off:off + 2 * L * n * D].reshape(L, 2, n, D)
        for l in range(L):
            assert (c[l, 0] == 100 + l).all() and (c[l, 1] == 200 + l).all()


def test_config1_handoff_shape():
    b, h = gen.config1()
    assert h.chunks.tolist() == [[2, 32, 32, 0], [2, 64, 32, 2 * 32 * 64]]
    assert b.ctx_lens[2] == 129
    buf = np.zeros(h.chunk_elems, np.uint16)
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, h.chunks, buf)
    assert buf.nbytes == 2 * 8192
    dk, dv = h.dst_k.copy(), h.dst_v.copy()
    oracle.kv_unpack_chunks(buf, h.chunks, dk, dv, h.dst_tables)
    np.testing.assert_array_equal(gather_tokens(dk, h.dst_tables[2], 32, 96),
                                  gather_tokens(h.src_k, h.src_tables[2], 32, 96))
    # relocation invariance (section 4.3: the receiver chooses placement): attention over the
    # moved range through the destination table equals attention through the source table
    q = b.q[48:49]
    src = oracle.attn_mixed_batch(q, h.src_k[0], h.src_v[0], h.src_tables[2:3] * 1, [0, 1], [96], b.scale)
    # make dst tokens [0,32) equal as well, then compare
    chunks0, n0 = gen.make_chunks([(2, 0, 32)], 32, 1, 1, 64)
    buf0 = np.zeros(n0, np.uint16)
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, chunks0, buf0)
    oracle.kv_unpack_chunks(buf0, chunks0, dk, dv, h.dst_tables)
    dst = oracle.attn_mixed_batch(q, dk[0], dv[0], h.dst_tables[2:3] * 1, [0, 1], [96], b.scale)
    np.testing.assert_array_equal(src, dst)


def test_rejects_out_of_table_ranges():
    h = small_handoff()
    bad = h.chunks.copy()
    bad[0, 1] = 16 * h.src_tables.shape[1]          # begins past the table
    with pytest.raises(ValueError):
        oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, bad, np.zeros(h.chunk_elems, np.uint16))
