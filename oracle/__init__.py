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
_SRCS = [_SRC, os.path.join(_HERE, "oracle_fp8.c")]
_LIB = os.path.join(_HERE, "liboracle.so")
_SAN_LIB = os.path.join(_HERE, "liboracle_san.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c and oracle_fp8.c with gcc (OpenMP) into liboracle.so next to them."""
    stale = (not os.path.exists(_LIB)) or any(
        os.path.getmtime(_LIB) < os.path.getmtime(src) for src in _SRCS)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", tmp] + _SRCS + ["-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized() -> str:
    """The same two sources with AddressSanitizer and UndefinedBehaviorSanitizer (host code only),
    into liboracle_san.so.  A process that loads it must have been started with the sanitizer
    runtime preloaded: ``tests/test_oracle_sanitized.py`` runs the pin tests that way, in a child
    process with ORACLE_LIB pointing here."""
    tmp = _SAN_LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(
        ["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
         "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
         "-o", tmp] + _SRCS + ["-lm"])
    os.replace(tmp, _SAN_LIB)
    return _SAN_LIB


_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
_u16p = np.ctypeslib.ndpointer(np.uint16, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")
_c = ctypes


def _load():
    global _lib
    with _lock:
        if _lib is None:
            # ORACLE_LIB: a library built elsewhere from the same sources (the sanitizer build)
            lib = ctypes.CDLL(os.environ.get("ORACLE_LIB") or build())
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
            lib.oracle_e4m3_decode.argtypes = [_u8p, _c.c_int64, _f64p]
            lib.oracle_e4m3_quantize.argtypes = [_u16p, _c.c_int64, _c.c_float, _u8p]
            lib.oracle_e4m3_from_float.argtypes = [_f32p, _c.c_int64, _u8p]
            lib.oracle_attn_rows_fp8kv.argtypes = [
                _u16p, _u8p, _u8p, _i32p, _c.c_int32, _i32p, _i32p, _c.c_int32, _c.c_int32,
                _c.c_int32, _c.c_int32, _c.c_int32, _c.c_double, _c.c_double, _c.c_double,
                _c.c_int32, _i32p, _f64p]
            lib.oracle_kv_append_fp8.argtypes = [
                _u16p, _u16p, _u8p, _u8p, _c.c_int32, _c.c_int32, _c.c_int32, _i32p, _c.c_int32,
                _c.c_int32, _i32p, _i32p, _c.c_float, _c.c_float]
            for f in (lib.oracle_e4m3_decode, lib.oracle_e4m3_quantize, lib.oracle_e4m3_from_float,
                      lib.oracle_attn_rows_fp8kv, lib.oracle_kv_append_fp8):
                f.restype = _c.c_int
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


# ---- 8-bit (E4M3) KV variant: oracle_fp8.c -------------------------------------------------

def e4m3_decode(codes):
    """Values of E4M3 codes (uint8, any shape) -> float64, NaN for 0x7f / 0xff."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape, dtype=np.float64)
    rc = _load().oracle_e4m3_decode(codes.reshape(-1), codes.size, out.reshape(-1))
    if rc:
        raise ValueError("oracle_e4m3_decode: invalid arguments (%d)" % rc)
    return out


def e4m3_quantize(x_bf16, scale):
    """Codes of bf16 inputs (uint16 bits, any shape): nearest E4M3 value of fp32(x)/scale."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    out = np.empty(x.shape, dtype=np.uint8)
    rc = _load().oracle_e4m3_quantize(x.reshape(-1), x.size, float(scale), out.reshape(-1))
    if rc:
        raise ValueError("oracle_e4m3_quantize: invalid arguments (%d)" % rc)
    return out


def e4m3_from_float(y):
    """Nearest E4M3 codes of fp32 values (the rounding rule alone, no scale)."""
    y = np.ascontiguousarray(y, dtype=np.float32)
    out = np.empty(y.shape, dtype=np.uint8)
    rc = _load().oracle_e4m3_from_float(y.reshape(-1), y.size, out.reshape(-1))
    if rc:
        raise ValueError("oracle_e4m3_from_float: invalid arguments (%d)" % rc)
    return out


def _attn8_args(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale, k_scale, v_scale):
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k_pool = np.ascontiguousarray(k_pool, dtype=np.uint8)
    v_pool = np.ascontiguousarray(v_pool, dtype=np.uint8)
    assert q.ndim == 3 and k_pool.ndim == 4 and k_pool.shape == v_pool.shape
    _, Hq, D = q.shape
    _, bs, Hkv, Dk = k_pool.shape
    assert D == Dk
    bt = _c32(block_tables)
    qo, cl = _c32(q_offsets), _c32(ctx_lens)
    S = cl.shape[0]
    assert bt.ndim == 2 and qo.shape[0] == S + 1 and bt.shape[0] == S and qo[-1] == q.shape[0]
    return (q, k_pool, v_pool, bt, bt.shape[1], qo, cl, S, Hq, Hkv, D, bs, float(scale),
            float(k_scale), float(v_scale))


def attn_rows_fp8kv(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale, k_scale, v_scale,
                    rows):
    """Selected rows on an E4M3 cache; rows: [n,3] = (segment, new-token index, head) -> [n,D]."""
    args = _attn8_args(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale, k_scale, v_scale)
    rows = _c32(rows).reshape(-1, 3)
    out = np.empty((rows.shape[0], args[0].shape[2]), dtype=np.float64)
    rc = _load().oracle_attn_rows_fp8kv(*args, rows.shape[0], rows, out)
    if rc:
        raise ValueError("oracle_attn_rows_fp8kv: invalid problem (%d)" % rc)
    return out


def attn_mixed_batch_fp8kv(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale, k_scale,
                           v_scale):
    """All rows on an E4M3 cache.  q: [total_q,Hq,D] u16; pools: [NB,bs,Hkv,D] u8 -> f64."""
    qo = _c32(q_offsets)
    Hq = q.shape[1]
    rows = [(i, j, h) for i in range(len(qo) - 1) for j in range(int(qo[i + 1] - qo[i]))
            for h in range(Hq)]
    out = attn_rows_fp8kv(q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, scale, k_scale,
                          v_scale, np.asarray(rows, dtype=np.int32).reshape(-1, 3))
    return out.reshape(q.shape[0], Hq, q.shape[2])


def kv_append_fp8(k_new, v_new, k_pool, v_pool, block_tables, q_offsets, ctx_lens, k_scale,
                  v_scale):
    """Quantises the new tokens' K/V rows [total_q, Hkv, D] (bf16 bits) and writes the codes into
    the one-layer uint8 pool [NB, 16, Hkv, D] in place."""
    assert k_pool.ndim == 4 and k_pool.shape == v_pool.shape
    for a in (k_new, v_new):
        assert a.dtype == np.uint16 and a.flags.c_contiguous
    for a in (k_pool, v_pool):
        assert a.dtype == np.uint8 and a.flags.c_contiguous
    _, bs, Hkv, D = k_pool.shape
    assert k_new.shape == v_new.shape and k_new.shape[1:] == (Hkv, D)
    bt, qo, cl = _c32(block_tables), _c32(q_offsets), _c32(ctx_lens)
    assert k_new.shape[0] == int(qo[-1])
    rc = _load().oracle_kv_append_fp8(k_new.reshape(-1), v_new.reshape(-1), k_pool.reshape(-1),
                                      v_pool.reshape(-1), bs, Hkv, D, bt, bt.shape[1],
                                      bt.shape[0], qo, cl, float(k_scale), float(v_scale))
    if rc:
        raise ValueError("oracle_kv_append_fp8: invalid problem (%d)" % rc)
    return k_pool, v_pool
