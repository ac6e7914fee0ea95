"""fp64 CPU oracle (test infrastructure only).

Thin ctypes wrapper around ``oracle.c``.  Nothing on the product path may import
this package: only the tests, the smoke check and the benchmark's CPU-baseline
leg do.  It shares no code with the HIP library and does not import it.

All arrays are numpy; bf16 tensors are passed as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (OpenMP) into liboracle.so next to it."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
_u16p = np.ctypeslib.ndpointer(np.uint16, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")
_c = ctypes


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            attn_common = [_u16p, _u16p, _u16p, _i32p, _c.c_int32, _i32p, _i32p,
                           _c.c_int32, _c.c_int32, _c.c_int32, _c.c_int32, _c.c_int32, _c.c_double]
            lib.oracle_attn_mixed_batch.argtypes = attn_common + [_f64p]
            lib.oracle_attn_rows.argtypes = attn_common + [_c.c_int32, _i32p, _f64p]
            lib.oracle_attn_row_weights.argtypes = attn_common + [_c.c_int32] * 3 + [_f64p, _f64p]
            lib.oracle_kv_pack_chunks.argtypes = [
                _u16p, _u16p, _c.c_int64, _c.c_int32, _c.c_int32, _c.c_int32, _c.c_int32,
                _i32p, _c.c_int32, _c.c_int32, _c.c_int32, _i32p, _i32p, _i32p, _i64p, _u16p]
            lib.oracle_kv_unpack_chunks.argtypes = [
                _u16p, _c.c_int32, _i32p, _i32p, _i32p, _i64p, _u16p, _u16p, _c.c_int64,
                _c.c_int32, _c.c_int32, _c.c_int32, _c.c_int32, _i32p, _c.c_int32, _c.c_int32]
            lib.oracle_kv_append.argtypes = [
                _u16p, _u16p, _u16p, _u16p, _c.c_int32, _c.c_int32, _c.c_int32, _i32p, _c.c_int32,
                _c.c_int32, _i32p, _i32p]
            for f in (lib.oracle_attn_mixed_batch, lib.oracle_attn_rows,
                      lib.oracle_attn_row_weights, lib.oracle_kv_pack_chunks,
                      lib.oracle_kv_unpack_chunks, lib.oracle_kv_append, lib.oracle_num_threads):
                f.restype = _c.c_int
            _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _c32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _attn_args(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale):
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k_pool = np.ascontiguousarray(k_pool, dtype=np.uint16)
    v_pool = np.ascontiguousarray(v_pool, dtype=np.uint16)
    assert q.ndim == 3 and k_pool.ndim == 4 and k_pool.shape == v_pool.shape
    _, Hq, D = q.shape
    _, bs, Hkv, Dk = k_pool.shape
    assert D == Dk
    bt = _c32(block_tables)
    assert bt.ndim == 2
    qo, cl = _c32(q_offsets), _c32(ctx_lens)
    S = cl.shape[0]
    assert qo.shape[0] == S + 1 and bt.shape[0] == S and qo[-1] == q.shape[0]
    return (q, k_pool, v_pool, bt, bt.shape[1], qo, cl, S, Hq, Hkv, D, bs, float(scale))


def attn_mixed_batch(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale):
    """All rows.  q: [total_q,Hq,D] u16; pools: [NB,bs,Hkv,D] u16 -> [total_q,Hq,D] f64."""
    args = _attn_args(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale)
    out = np.empty(args[0].shape, dtype=np.float64)
    rc = _load().oracle_attn_mixed_batch(*args, out)
    if rc:
        raise ValueError("oracle_attn_mixed_batch: invalid problem (%d)" % rc)
    return out


def attn_rows(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale, rows):
    """Selected rows; rows: [n,3] = (segment, new-token index, query head) -> [n,D] f64."""
    args = _attn_args(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale)
    rows = _c32(rows).reshape(-1, 3)
    out = np.empty((rows.shape[0], args[0].shape[2]), dtype=np.float64)
    rc = _load().oracle_attn_rows(*args, rows.shape[0], rows, out)
    if rc:
        raise ValueError("oracle_attn_rows: invalid problem (%d)" % rc)
    return out


def attn_row_weights(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale, i, j, h):
    """Softmax weights and output of one row -> (weights[p+1], out[D])."""
    args = _attn_args(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale)
    w = np.zeros(int(args[6][i]), dtype=np.float64)
    o = np.empty(args[0].shape[2], dtype=np.float64)
    n = _load().oracle_attn_row_weights(*args, int(i), int(j), int(h), w, o)
    if n < 0:
        raise ValueError("oracle_attn_row_weights: invalid problem (%d)" % n)
    return w[:n], o


def _pool_args(k_pool, v_pool):
    """Pools are [L,NB,bs,Hkv,D] u16, C-contiguous, modified in place by unpack."""
    assert k_pool.dtype == np.uint16 and v_pool.dtype == np.uint16
    assert k_pool.flags.c_contiguous and v_pool.flags.c_contiguous
    assert k_pool.ndim == 5 and k_pool.shape == v_pool.shape
    L, NB, bs, Hkv, D = k_pool.shape
    return L, NB * bs * Hkv * D, bs, Hkv, D


def _chunk_args(chunks):
    """chunks: iterable of (seq, token_begin, num_tokens, chunk_offset_elements)."""
    ch = np.asarray(list(chunks), dtype=np.int64).reshape(-1, 4)
    return (ch.shape[0], _c32(ch[:, 0]), _c32(ch[:, 1]), _c32(ch[:, 2]),
            np.ascontiguousarray(ch[:, 3], dtype=np.int64))


def kv_pack_chunks(k_pool, v_pool, block_tables, chunks, chunk_buf):
    L, stride, bs, Hkv, D = _pool_args(k_pool, v_pool)
    bt = _c32(block_tables)
    n, seq, tb, nt, off = _chunk_args(chunks)
    assert chunk_buf.dtype == np.uint16 and chunk_buf.flags.c_contiguous
    rc = _load().oracle_kv_pack_chunks(k_pool.reshape(-1), v_pool.reshape(-1), stride, L, bs, Hkv,
                                       D, bt, bt.shape[1], bt.shape[0], n, seq, tb, nt, off,
                                       chunk_buf.reshape(-1))
    if rc:
        raise ValueError("oracle_kv_pack_chunks: invalid problem (%d)" % rc)
    return chunk_buf


def kv_unpack_chunks(chunk_buf, chunks, k_pool, v_pool, block_tables):
    L, stride, bs, Hkv, D = _pool_args(k_pool, v_pool)
    bt = _c32(block_tables)
    n, seq, tb, nt, off = _chunk_args(chunks)
    assert chunk_buf.dtype == np.uint16 and chunk_buf.flags.c_contiguous
    rc = _load().oracle_kv_unpack_chunks(chunk_buf.reshape(-1), n, seq, tb, nt, off,
                                         k_pool.reshape(-1), v_pool.reshape(-1), stride, L, bs,
                                         Hkv, D, bt, bt.shape[1], bt.shape[0])
    if rc:
        raise ValueError("oracle_kv_unpack_chunks: invalid problem (%d)" % rc)


def kv_append(k_new, v_new, k_pool, v_pool, block_tables, q_offsets, ctx_lens):
    """Writes the new tokens' K/V rows [total_q, Hkv, D] (bf16 bits) into the one-layer pool
    [NB, 16, Hkv, D] in place, at the positions [ctx_len - q_len, ctx_len) of each segment."""
    assert k_pool.ndim == 4 and k_pool.shape == v_pool.shape
    for a in (k_new, v_new, k_pool, v_pool):
        assert a.dtype == np.uint16 and a.flags.c_contiguous
    _, bs, Hkv, D = k_pool.shape
    assert k_new.shape == v_new.shape and k_new.shape[1:] == (Hkv, D)
    bt, qo, cl = _c32(block_tables), _c32(q_offsets), _c32(ctx_lens)
    assert k_new.shape[0] == int(qo[-1])
    rc = _load().oracle_kv_append(k_new.reshape(-1), v_new.reshape(-1), k_pool.reshape(-1),
                                  v_pool.reshape(-1), bs, Hkv, D, bt, bt.shape[1], bt.shape[0],
                                  qo, cl)
    if rc:
        raise ValueError("oracle_kv_append: invalid problem (%d)" % rc)
    return k_pool, v_pool
