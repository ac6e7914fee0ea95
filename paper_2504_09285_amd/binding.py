"""ctypes binding of libdsv_attn.so: argument marshalling only.

torch is used for device memory and streams; tensors are passed to the library as raw device
pointers.  Function names and argument order follow ``include/dsv_attn.h``.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("DSV_ATTN_LIB") or os.path.join(_HERE, "libdsv_attn.so")
_lib = None

DSV_OUT_F32, DSV_OUT_BF16 = 0, 1
_ERRORS = {-1: "DSV_E_INVALID", -2: "DSV_E_UNSUPPORTED", -3: "DSV_E_WORKSPACE", -4: "DSV_E_LAUNCH"}


class DsvError(RuntimeError):
    def __init__(self, fn: str, code: int):
        super().__init__("%s failed: %s (%d)" % (fn, _ERRORS.get(code, "?"), code))
        self.code = code


class _Pool(C.Structure):
    _fields_ = [("k_base", C.c_void_p), ("v_base", C.c_void_p), ("layer_stride", C.c_int64),
                ("num_layers", C.c_int32), ("num_blocks", C.c_int32), ("block_size", C.c_int32),
                ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32)]


class _Plan(C.Structure):
    _fields_ = [("opaque", C.c_uint64 * 16)]


class AttnPlan:
    """Host-side record of ``attn_mixed_batch_plan`` (``dsv_attn_plan``), handed to the planned calls."""

    def __init__(self):
        self.c = _Plan()


CHUNK_DTYPE = np.dtype([("seq", "<i4"), ("token_begin", "<i4"), ("num_tokens", "<i4"),
                        ("reserved", "<i4"), ("chunk_offset", "<i8")])
assert CHUNK_DTYPE.itemsize == 24

EXPORTS = ("attn_mixed_batch_workspace_bytes", "attn_mixed_batch_plan_info", "attn_mixed_batch", "kv_pack_chunks",
           "kv_unpack_chunks", "kv_append", "attn_mixed_batch_fp8kv_workspace_bytes",
           "attn_mixed_batch_fp8kv", "kv_append_fp8", "kv_pack_chunks_fp8", "kv_unpack_chunks_fp8",
           "attn_mixed_batch_plan", "attn_mixed_batch_planned", "attn_mixed_batch_fp8kv_planned",
           "attn_mixed_batch_static", "attn_mixed_batch_static_max_bytes",
           "kv_unpack_chunks_ordered", "kv_unpack_chunks_ordered_workspace_bytes", "dsv_check_block_tables", "dsv_calib_hbm", "dsv_calib_mfma", "dsv_calib_mfma_data", "dsv_calib_paged_read", "dsv_profile_events", "dsv_build_info")
KERNEL_PLAN, KERNEL_ROWS, KERNEL_TILES, KERNEL_MERGE, KERNEL_MIXED, KERNEL_STAGE = 0, 1, 2, 3, 4, 5


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libdsv_attn.so (built in-tree by ``paper_2504_09285_amd.build``).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("libdsv_attn.so is not built: run `python -m paper_2504_09285_amd.build` "
                           "(there is no fallback path)")
    # torch ships a HIP runtime of its own (same soname as the system's, different file).  Tensors
    # and streams come from torch, so its runtime has to be the one this library binds to: loaded
    # first, it satisfies the library's dependency; loaded second, the process would hold two
    # runtimes that do not know each other's allocations, and every launch would fail.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(_LIB_PATH)
    i32p, vp = C.POINTER(C.c_int32), C.c_void_p
    lib.attn_mixed_batch_workspace_bytes.restype = C.c_size_t
    lib.attn_mixed_batch_workspace_bytes.argtypes = [C.c_int32, i32p, i32p, C.c_int32, C.c_int32, C.c_int32]
    lib.attn_mixed_batch_plan_info.restype = C.c_int
    lib.attn_mixed_batch_plan_info.argtypes = [C.c_int32, i32p, i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, i32p]
    lib.attn_mixed_batch.restype = C.c_int
    lib.attn_mixed_batch.argtypes = [vp, vp, C.POINTER(_Pool), C.c_int32, vp, C.c_int32, vp, vp,
                                     i32p, i32p, C.c_int32, C.c_int32, C.c_float, C.c_int32,
                                     vp, C.c_size_t, vp]
    lib.kv_append.restype = C.c_int
    lib.kv_append.argtypes = [vp, vp, C.POINTER(_Pool), C.c_int32, vp, C.c_int32, vp, vp, i32p, i32p,
                              C.c_int32, vp]
    lib.kv_pack_chunks.restype = C.c_int
    lib.kv_pack_chunks.argtypes = [C.POINTER(_Pool), vp, C.c_int32, vp, vp, C.c_int32, vp, vp]
    lib.kv_unpack_chunks.restype = C.c_int
    lib.kv_unpack_chunks.argtypes = [vp, vp, vp, C.c_int32, C.POINTER(_Pool), vp, C.c_int32, vp]
    lib.attn_mixed_batch_fp8kv_workspace_bytes.restype = C.c_size_t
    lib.attn_mixed_batch_fp8kv_workspace_bytes.argtypes = lib.attn_mixed_batch_workspace_bytes.argtypes
    lib.attn_mixed_batch_fp8kv.restype = C.c_int
    lib.attn_mixed_batch_fp8kv.argtypes = [vp, vp, C.POINTER(_Pool), C.c_int32, vp, C.c_int32, vp, vp,
                                           i32p, i32p, C.c_int32, C.c_int32, C.c_float, C.c_float,
                                           C.c_float, C.c_int32, vp, C.c_size_t, vp]
    lib.attn_mixed_batch_plan.restype = C.c_int
    lib.attn_mixed_batch_plan.argtypes = [C.POINTER(_Plan), vp, C.c_int32, vp, vp, i32p, i32p, C.c_int32,
                                          C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, C.c_size_t, vp]
    lib.attn_mixed_batch_planned.restype = C.c_int
    lib.attn_mixed_batch_planned.argtypes = [C.POINTER(_Plan)] + lib.attn_mixed_batch.argtypes
    lib.attn_mixed_batch_fp8kv_planned.restype = C.c_int
    lib.attn_mixed_batch_fp8kv_planned.argtypes = [C.POINTER(_Plan)] + lib.attn_mixed_batch_fp8kv.argtypes
    lib.kv_append_fp8.restype = C.c_int
    lib.kv_append_fp8.argtypes = [vp, vp, C.POINTER(_Pool), C.c_int32, vp, C.c_int32, vp, vp, i32p,
                                  i32p, C.c_int32, C.c_float, C.c_float, vp]
    lib.kv_pack_chunks_fp8.restype = C.c_int
    lib.kv_pack_chunks_fp8.argtypes = lib.kv_pack_chunks.argtypes
    lib.kv_unpack_chunks_fp8.restype = C.c_int
    lib.kv_unpack_chunks_fp8.argtypes = lib.kv_unpack_chunks.argtypes
    lib.attn_mixed_batch_static.restype = C.c_int
    lib.attn_mixed_batch_static.argtypes = [vp, vp, C.POINTER(_Pool), C.c_int32, vp, C.c_int32, vp, vp,
                                            i32p, i32p, C.c_int32, C.c_int32, C.c_float, C.c_int32, vp]
    lib.attn_mixed_batch_static_max_bytes.restype = C.c_size_t
    lib.attn_mixed_batch_static_max_bytes.argtypes = []
    lib.kv_unpack_chunks_ordered_workspace_bytes.restype = C.c_size_t
    lib.kv_unpack_chunks_ordered_workspace_bytes.argtypes = [C.c_int32]
    lib.kv_unpack_chunks_ordered.restype = C.c_int
    lib.kv_unpack_chunks_ordered.argtypes = [vp, vp, vp, C.c_int32, C.POINTER(_Pool), vp, C.c_int32, vp, C.c_size_t, vp]
    lib.dsv_check_block_tables.restype = C.c_int
    lib.dsv_check_block_tables.argtypes = [vp, C.c_int32, vp, C.c_int32, C.c_int32, vp, vp]
    lib.dsv_calib_hbm.restype = C.c_int
    lib.dsv_calib_hbm.argtypes = [C.c_int32, vp, vp, C.c_size_t, vp]
    lib.dsv_calib_mfma.restype = C.c_int
    lib.dsv_calib_mfma.argtypes = [C.c_int32, vp, C.POINTER(C.c_double), vp]
    lib.dsv_calib_mfma_data.restype = C.c_int
    lib.dsv_calib_mfma_data.argtypes = [C.c_int32, C.c_int32, vp, C.c_size_t, vp, C.POINTER(C.c_double), vp]
    lib.dsv_calib_paged_read.restype = C.c_int
    lib.dsv_calib_paged_read.argtypes = [vp, vp, C.c_size_t, vp, C.POINTER(C.c_double), vp]
    lib.dsv_profile_events.restype = C.c_int
    lib.dsv_profile_events.argtypes = [C.c_int32, vp, vp]
    lib.dsv_build_info.restype = C.c_char_p
    lib.dsv_build_info.argtypes = []
    _lib = lib
    return lib


def build_info() -> str:
    return load_library().dsv_build_info().decode()


def dsv_profile_events(kernel_id: int, start_event: Optional[int], stop_event: Optional[int]) -> None:
    """See ``dsv_profile_events`` in include/dsv_attn.h; events are raw hipEvent_t handles."""
    rc = load_library().dsv_profile_events(int(kernel_id), start_event, stop_event)
    if rc:
        raise DsvError("dsv_profile_events", rc)


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _i32_ptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


class KVPool:
    """A paged KV pool held in two torch tensors ``[L, num_blocks, 16, Hkv, D]`` on the device:
    2-byte elements (bf16) for the plain entry points, 1-byte elements (E4M3 codes, e.g. uint8)
    for the ``*_fp8`` / ``*_fp8kv`` ones."""

    def __init__(self, k, v):
        assert k.shape == v.shape and k.dim() == 5 and k.is_contiguous() and v.is_contiguous()
        assert k.element_size() == v.element_size() and k.element_size() in (1, 2)
        self.elem_bytes = k.element_size()
        self.k, self.v = k, v
        L, NB, bs, Hkv, D = k.shape
        self.L, self.NB, self.bs, self.Hkv, self.D = L, NB, bs, Hkv, D
        self._c = _Pool(k.data_ptr(), v.data_ptr(), NB * bs * Hkv * D, L, NB, bs, Hkv, D)

    @property
    def c(self):
        return C.byref(self._c)


class ChunkDescs:
    """Chunk descriptors: host array (numpy, CHUNK_DTYPE) plus its device copy."""

    def __init__(self, chunks, device="cuda"):
        import torch
        ch = np.asarray(chunks, dtype=np.int64).reshape(-1, 4)
        host = np.zeros(ch.shape[0], dtype=CHUNK_DTYPE)
        host["seq"], host["token_begin"], host["num_tokens"], host["chunk_offset"] = ch.T
        self.host = host
        self.n = int(ch.shape[0])
        raw = np.frombuffer(host.tobytes(), dtype=np.uint8).copy() if self.n else np.zeros(0, np.uint8)
        self.dev = torch.from_numpy(raw).to(device)


def _require(cond, what: str) -> None:
    if not cond:
        raise ValueError("dsv binding: " + what)


def _nbytes(t) -> int:
    return int(t.numel() * t.element_size())


def _batch_lists(q_offsets_host, ctx_lens_host, block_tables, q_offsets, ctx_lens):
    """Host lists as int32 arrays, checked against each other and against the device arrays: the C
    ABI carries no lengths for these, so a mismatch would send a kernel outside a buffer."""
    import torch
    qo, cl = _host_i32(q_offsets_host), _host_i32(ctx_lens_host)
    _require(qo.ndim == 1 and cl.ndim == 1 and qo.shape[0] == cl.shape[0] + 1,
             "q_offsets_host needs one entry more than ctx_lens_host")
    _require(block_tables.dtype == torch.int32 and block_tables.dim() == 2 and block_tables.is_contiguous(),
             "block_tables must be a contiguous int32 [num_seqs, max_blocks] tensor")
    _require(block_tables.shape[0] >= cl.shape[0], "block_tables has fewer rows than the batch has segments")
    _require(q_offsets.dtype == torch.int32 and q_offsets.is_contiguous() and q_offsets.numel() >= qo.shape[0],
             "q_offsets (device) must be int32 with num_seqs + 1 entries")
    _require(ctx_lens.dtype == torch.int32 and ctx_lens.is_contiguous() and ctx_lens.numel() >= cl.shape[0],
             "ctx_lens (device) must be int32 with num_seqs entries")
    return qo, cl


def _attn_tensors(q, out, pool: "KVPool", num_q_heads, qo, elem_bytes):
    import torch
    _require(pool.elem_bytes == elem_bytes, "the pool's element size does not fit this entry point")
    _require(out.dtype in (torch.float32, torch.bfloat16), "out must be float32 or bfloat16")
    _require(q.is_contiguous() and out.is_contiguous() and q.element_size() == 2, "q must be contiguous bf16")
    total_q = int(qo[-1]) - int(qo[0])               # (offsets that do not start at 0: the library refuses them)
    want = (total_q, int(num_q_heads), pool.D)
    _require(tuple(q.shape) == want, "q must have shape [total_q, num_q_heads, head_dim] = %r" % (want,))
    _require(tuple(out.shape) == want, "out must have the shape of q")
    return DSV_OUT_F32 if out.dtype == torch.float32 else DSV_OUT_BF16


def _new_kv_tensors(k_new, v_new, pool: "KVPool", qo, elem_bytes):
    _require(pool.elem_bytes == elem_bytes, "the pool's element size does not fit this entry point")
    _require(k_new.is_contiguous() and v_new.is_contiguous() and k_new.element_size() == 2 and
             v_new.element_size() == 2, "k_new / v_new must be contiguous bf16")
    want = (int(qo[-1]) - int(qo[0]), pool.Hkv, pool.D)
    _require(tuple(k_new.shape) == want and tuple(v_new.shape) == want,
             "k_new / v_new must have shape [total_q, num_kv_heads, head_dim] = %r" % (want,))


def _copy_tensors(pool: "KVPool", block_tables, descs: "ChunkDescs", chunk_buf, elem_bytes):
    """Hand-off arguments: the table's dtype and row count, and that every chunk lies inside
    chunk_buf (the C ABI has no buffer length)."""
    import torch
    _require(pool.elem_bytes == elem_bytes, "the pool's element size does not fit this entry point")
    _require(block_tables.dtype == torch.int32 and block_tables.dim() == 2 and block_tables.is_contiguous(),
             "block_tables must be a contiguous int32 [rows, max_blocks] tensor")
    _require(chunk_buf.is_contiguous(), "chunk_buf must be contiguous")
    if descs.n:
        h = descs.host
        _require(int(h["seq"].min()) >= 0 and int(h["seq"].max()) < block_tables.shape[0],
                 "a chunk names a row the block table does not have")
        per_tok = 2 * pool.L * pool.Hkv * pool.D                       # elements per token of a chunk
        end = (h["chunk_offset"] + h["num_tokens"].astype(np.int64) * per_tok) * elem_bytes
        _require(int(h["chunk_offset"].min()) >= 0 and int(end.max()) <= _nbytes(chunk_buf),
                 "a chunk reaches past the end of chunk_buf")
        _require(_nbytes(descs.dev) >= descs.n * CHUNK_DTYPE.itemsize, "device copy of the descriptors too short")


def attn_mixed_batch_workspace_bytes(q_offsets_host, ctx_lens_host, num_q_heads, num_kv_heads,
                                     head_dim) -> int:
    qo, cl = _host_i32(q_offsets_host), _host_i32(ctx_lens_host)
    _require(qo.shape[0] == cl.shape[0] + 1, "q_offsets_host needs one entry more than ctx_lens_host")
    return int(load_library().attn_mixed_batch_workspace_bytes(
        cl.shape[0], _i32_ptr(qo), _i32_ptr(cl), num_q_heads, num_kv_heads, head_dim))


PLAN_INFO_FIELDS = ("row_streams", "part_tokens", "rows", "row_items", "tile_items", "tile_part_tiles",
                    "one_launch", "tile_tokens")


def attn_mixed_batch_plan_info(q_offsets_host, ctx_lens_host, num_q_heads, num_kv_heads, head_dim,
                               kv_elem_bytes=2) -> dict:
    """See ``attn_mixed_batch_plan_info`` in include/dsv_attn.h; the eight integers by name."""
    qo, cl = _host_i32(q_offsets_host), _host_i32(ctx_lens_host)
    _require(qo.shape[0] == cl.shape[0] + 1, "q_offsets_host needs one entry more than ctx_lens_host")
    info = np.zeros(8, np.int32)
    rc = load_library().attn_mixed_batch_plan_info(cl.shape[0], _i32_ptr(qo), _i32_ptr(cl), int(num_q_heads),
                                                   int(num_kv_heads), int(head_dim), int(kv_elem_bytes), _i32_ptr(info))
    if rc:
        raise DsvError("attn_mixed_batch_plan_info", rc)
    return dict(zip(PLAN_INFO_FIELDS, (int(x) for x in info)))


def attn_mixed_batch(q, out, pool: KVPool, layer, block_tables, q_offsets, ctx_lens,
                     q_offsets_host, ctx_lens_host, num_q_heads, softmax_scale, workspace,
                     stream=None) -> None:
    """See ``attn_mixed_batch`` in include/dsv_attn.h.  ``out`` dtype selects fp32 or bf16."""
    qo, cl = _batch_lists(q_offsets_host, ctx_lens_host, block_tables, q_offsets, ctx_lens)
    out_dtype = _attn_tensors(q, out, pool, num_q_heads, qo, 2)
    rc = load_library().attn_mixed_batch(
        q.data_ptr(), out.data_ptr(), pool.c, int(layer), block_tables.data_ptr(),
        int(block_tables.shape[1]), q_offsets.data_ptr(), ctx_lens.data_ptr(), _i32_ptr(qo), _i32_ptr(cl),
        int(cl.shape[0]), int(num_q_heads), float(softmax_scale), out_dtype,
        workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream))
    if rc:
        raise DsvError("attn_mixed_batch", rc)


def attn_mixed_batch_static_max_bytes() -> int:
    return int(load_library().attn_mixed_batch_static_max_bytes())


def attn_mixed_batch_static(q, out, pool: KVPool, layer, block_tables, q_offsets, ctx_lens,
                            q_offsets_host, ctx_lens_host, num_q_heads, softmax_scale, stream=None) -> None:
    """See ``attn_mixed_batch_static`` in include/dsv_attn.h: no workspace argument, nothing allocated."""
    qo, cl = _batch_lists(q_offsets_host, ctx_lens_host, block_tables, q_offsets, ctx_lens)
    out_dtype = _attn_tensors(q, out, pool, num_q_heads, qo, 2)
    rc = load_library().attn_mixed_batch_static(
        q.data_ptr(), out.data_ptr(), pool.c, int(layer), block_tables.data_ptr(),
        int(block_tables.shape[1]), q_offsets.data_ptr(), ctx_lens.data_ptr(), _i32_ptr(qo), _i32_ptr(cl),
        int(cl.shape[0]), int(num_q_heads), float(softmax_scale), out_dtype, _stream_ptr(stream))
    if rc:
        raise DsvError("attn_mixed_batch_static", rc)


def attn_mixed_batch_plan(block_tables, q_offsets, ctx_lens, q_offsets_host, ctx_lens_host,
                          num_q_heads, num_kv_heads, head_dim, workspace, kv_elem_bytes=2,
                          stream=None) -> AttnPlan:
    """See ``attn_mixed_batch_plan`` in include/dsv_attn.h: the work lists of a batch, built once
    into ``workspace`` for the planned calls of every layer."""
    qo, cl = _batch_lists(q_offsets_host, ctx_lens_host, block_tables, q_offsets, ctx_lens)
    plan = AttnPlan()
    rc = load_library().attn_mixed_batch_plan(
        C.byref(plan.c), block_tables.data_ptr(), int(block_tables.shape[1]), q_offsets.data_ptr(),
        ctx_lens.data_ptr(), _i32_ptr(qo), _i32_ptr(cl), int(cl.shape[0]), int(num_q_heads),
        int(num_kv_heads), int(head_dim), int(kv_elem_bytes), workspace.data_ptr(),
        _nbytes(workspace), _stream_ptr(stream))
    if rc:
        raise DsvError("attn_mixed_batch_plan", rc)
    return plan


def attn_mixed_batch_planned(plan: AttnPlan, q, out, pool: KVPool, layer, block_tables, q_offsets,
                             ctx_lens, q_offsets_host, ctx_lens_host, num_q_heads, softmax_scale,
                             workspace, stream=None) -> None:
    """See ``attn_mixed_batch_planned`` in include/dsv_attn.h."""
    qo, cl = _batch_lists(q_offsets_host, ctx_lens_host, block_tables, q_offsets, ctx_lens)
    out_dtype = _attn_tensors(q, out, pool, num_q_heads, qo, 2)
    rc = load_library().attn_mixed_batch_planned(
        C.byref(plan.c), q.data_ptr(), out.data_ptr(), pool.c, int(layer), block_tables.data_ptr(),
        int(block_tables.shape[1]), q_offsets.data_ptr(), ctx_lens.data_ptr(), _i32_ptr(qo), _i32_ptr(cl),
        int(cl.shape[0]), int(num_q_heads), float(softmax_scale), out_dtype,
        workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream))
    if rc:
        raise DsvError("attn_mixed_batch_planned", rc)


def attn_mixed_batch_fp8kv_planned(plan: AttnPlan, q, out, pool: KVPool, layer, block_tables,
                                   q_offsets, ctx_lens, q_offsets_host, ctx_lens_host, num_q_heads,
                                   softmax_scale, k_scale, v_scale, workspace, stream=None) -> None:
    """See ``attn_mixed_batch_fp8kv_planned`` in include/dsv_attn.h; ``pool`` holds 1-byte elements."""
    qo, cl = _batch_lists(q_offsets_host, ctx_lens_host, block_tables, q_offsets, ctx_lens)
    out_dtype = _attn_tensors(q, out, pool, num_q_heads, qo, 1)
    rc = load_library().attn_mixed_batch_fp8kv_planned(
        C.byref(plan.c), q.data_ptr(), out.data_ptr(), pool.c, int(layer), block_tables.data_ptr(),
        int(block_tables.shape[1]), q_offsets.data_ptr(), ctx_lens.data_ptr(), _i32_ptr(qo), _i32_ptr(cl),
        int(cl.shape[0]), int(num_q_heads), float(softmax_scale), float(k_scale), float(v_scale),
        out_dtype, workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream))
    if rc:
        raise DsvError("attn_mixed_batch_fp8kv_planned", rc)


def kv_append(k_new, v_new, pool: KVPool, layer, block_tables, q_offsets, ctx_lens, q_offsets_host,
              ctx_lens_host, stream=None) -> None:
    """See ``kv_append`` in include/dsv_attn.h."""
    qo, cl = _batch_lists(q_offsets_host, ctx_lens_host, block_tables, q_offsets, ctx_lens)
    _new_kv_tensors(k_new, v_new, pool, qo, 2)
    rc = load_library().kv_append(
        k_new.data_ptr(), v_new.data_ptr(), pool.c, int(layer), block_tables.data_ptr(),
        int(block_tables.shape[1]), q_offsets.data_ptr(), ctx_lens.data_ptr(), _i32_ptr(qo), _i32_ptr(cl),
        int(cl.shape[0]), _stream_ptr(stream))
    if rc:
        raise DsvError("kv_append", rc)


def kv_pack_chunks(src: KVPool, block_tables, descs: ChunkDescs, chunk_buf, stream=None) -> None:
    """See ``kv_pack_chunks`` in include/dsv_attn.h."""
    _copy_tensors(src, block_tables, descs, chunk_buf, 2)
    rc = load_library().kv_pack_chunks(
        src.c, block_tables.data_ptr(), int(block_tables.shape[1]), descs.dev.data_ptr(),
        descs.host.ctypes.data, descs.n, chunk_buf.data_ptr(), _stream_ptr(stream))
    if rc:
        raise DsvError("kv_pack_chunks", rc)


def kv_unpack_chunks(chunk_buf, descs: ChunkDescs, dst: KVPool, dst_block_tables, stream=None) -> None:
    """See ``kv_unpack_chunks`` in include/dsv_attn.h."""
    _copy_tensors(dst, dst_block_tables, descs, chunk_buf, 2)
    rc = load_library().kv_unpack_chunks(
        chunk_buf.data_ptr(), descs.dev.data_ptr(), descs.host.ctypes.data, descs.n, dst.c,
        dst_block_tables.data_ptr(), int(dst_block_tables.shape[1]), _stream_ptr(stream))
    if rc:
        raise DsvError("kv_unpack_chunks", rc)


def kv_unpack_chunks_ordered_workspace_bytes(num_blocks: int) -> int:
    return int(load_library().kv_unpack_chunks_ordered_workspace_bytes(int(num_blocks)))


def kv_unpack_chunks_ordered(chunk_buf, descs: ChunkDescs, dst: KVPool, dst_block_tables, workspace,
                             stream=None) -> None:
    """See ``kv_unpack_chunks_ordered`` in include/dsv_attn.h."""
    _copy_tensors(dst, dst_block_tables, descs, chunk_buf, 2)
    rc = load_library().kv_unpack_chunks_ordered(
        chunk_buf.data_ptr(), descs.dev.data_ptr(), descs.host.ctypes.data, descs.n, dst.c,
        dst_block_tables.data_ptr(), int(dst_block_tables.shape[1]), workspace.data_ptr(), _nbytes(workspace),
        _stream_ptr(stream))
    if rc:
        raise DsvError("kv_unpack_chunks_ordered", rc)


def dsv_check_block_tables(block_tables, tokens_per_seq, num_blocks, result, stream=None) -> None:
    """See ``dsv_check_block_tables`` in include/dsv_attn.h.  ``result``: int32 device tensor of two
    entries, written by the call; read it after synchronising with the stream."""
    import torch
    _require(block_tables.dtype == torch.int32 and block_tables.dim() == 2 and block_tables.is_contiguous(),
             "block_tables must be a contiguous int32 [num_seqs, max_blocks] tensor")
    _require(tokens_per_seq.dtype == torch.int32 and tokens_per_seq.is_contiguous() and
             tokens_per_seq.numel() == block_tables.shape[0], "tokens_per_seq must be int32 [num_seqs]")
    _require(result.dtype == torch.int32 and result.is_contiguous() and result.numel() >= 2,
             "result must be an int32 tensor of two entries")
    rc = load_library().dsv_check_block_tables(
        block_tables.data_ptr(), int(block_tables.shape[1]), tokens_per_seq.data_ptr(),
        int(block_tables.shape[0]), int(num_blocks), result.data_ptr(), _stream_ptr(stream))
    if rc:
        raise DsvError("dsv_check_block_tables", rc)


def dsv_calib_hbm(mode: int, dst, src, nbytes: int, stream=None) -> None:
    """See ``dsv_calib_hbm`` in include/dsv_attn.h (0 read, 1 write, 2 copy)."""
    _require(_nbytes(dst) >= (nbytes if mode else 16) and (mode == 1 or _nbytes(src) >= nbytes),
             "calibration buffers shorter than the byte count")
    rc = load_library().dsv_calib_hbm(int(mode), dst.data_ptr(), 0 if mode == 1 else src.data_ptr(),
                                      int(nbytes), _stream_ptr(stream))
    if rc:
        raise DsvError("dsv_calib_hbm", rc)


def dsv_calib_mfma(iters: int, sink, stream=None) -> float:
    """See ``dsv_calib_mfma`` in include/dsv_attn.h; returns the flops of the launch."""
    flops = C.c_double()
    rc = load_library().dsv_calib_mfma(int(iters), sink.data_ptr(), C.byref(flops), _stream_ptr(stream))
    if rc:
        raise DsvError("dsv_calib_mfma", rc)
    return float(flops.value)


def dsv_calib_mfma_data(iters: int, operands, sink, shape: int = 1, stream=None) -> float:
    """See ``dsv_calib_mfma_data`` in include/dsv_attn.h (shape 0: 32x32x16 MFMAs, 1: 16x16x32);
    returns the flops of the launch."""
    _require(operands.is_contiguous(), "operands must be contiguous")
    flops = C.c_double()
    rc = load_library().dsv_calib_mfma_data(int(shape), int(iters), operands.data_ptr(), _nbytes(operands), sink.data_ptr(),
                                            C.byref(flops), _stream_ptr(stream))
    if rc:
        raise DsvError("dsv_calib_mfma_data", rc)
    return float(flops.value)


def dsv_calib_paged_read(k, v, sink, stream=None) -> float:
    """See ``dsv_calib_paged_read`` in include/dsv_attn.h; returns the bytes the launch reads."""
    _require(k.is_contiguous() and v.is_contiguous(), "k and v must be contiguous")
    _require(k.numel() * k.element_size() == v.numel() * v.element_size(), "k and v must have the same size")
    nbytes = C.c_double()
    rc = load_library().dsv_calib_paged_read(k.data_ptr(), v.data_ptr(), k.numel() * k.element_size(),
                                             sink.data_ptr(), C.byref(nbytes), _stream_ptr(stream))
    if rc:
        raise DsvError("dsv_calib_paged_read", rc)
    return float(nbytes.value)


# ---- 8-bit KV cache variant ------------------------------------------------------------------

def attn_mixed_batch_fp8kv_workspace_bytes(q_offsets_host, ctx_lens_host, num_q_heads, num_kv_heads,
                                           head_dim) -> int:
    qo, cl = _host_i32(q_offsets_host), _host_i32(ctx_lens_host)
    _require(qo.shape[0] == cl.shape[0] + 1, "q_offsets_host needs one entry more than ctx_lens_host")
    return int(load_library().attn_mixed_batch_fp8kv_workspace_bytes(
        cl.shape[0], _i32_ptr(qo), _i32_ptr(cl), num_q_heads, num_kv_heads, head_dim))


def attn_mixed_batch_fp8kv(q, out, pool: KVPool, layer, block_tables, q_offsets, ctx_lens,
                           q_offsets_host, ctx_lens_host, num_q_heads, softmax_scale, k_scale,
                           v_scale, workspace, stream=None) -> None:
    """See ``attn_mixed_batch_fp8kv`` in include/dsv_attn.h; ``pool`` holds 1-byte elements."""
    qo, cl = _batch_lists(q_offsets_host, ctx_lens_host, block_tables, q_offsets, ctx_lens)
    out_dtype = _attn_tensors(q, out, pool, num_q_heads, qo, 1)
    rc = load_library().attn_mixed_batch_fp8kv(
        q.data_ptr(), out.data_ptr(), pool.c, int(layer), block_tables.data_ptr(),
        int(block_tables.shape[1]), q_offsets.data_ptr(), ctx_lens.data_ptr(), _i32_ptr(qo), _i32_ptr(cl),
        int(cl.shape[0]), int(num_q_heads), float(softmax_scale), float(k_scale), float(v_scale),
        out_dtype, workspace.data_ptr(), _nbytes(workspace), _stream_ptr(stream))
    if rc:
        raise DsvError("attn_mixed_batch_fp8kv", rc)


def kv_append_fp8(k_new, v_new, pool: KVPool, layer, block_tables, q_offsets, ctx_lens,
                  q_offsets_host, ctx_lens_host, k_scale, v_scale, stream=None) -> None:
    """See ``kv_append_fp8`` in include/dsv_attn.h: bf16 rows in, E4M3 codes stored."""
    qo, cl = _batch_lists(q_offsets_host, ctx_lens_host, block_tables, q_offsets, ctx_lens)
    _new_kv_tensors(k_new, v_new, pool, qo, 1)
    rc = load_library().kv_append_fp8(
        k_new.data_ptr(), v_new.data_ptr(), pool.c, int(layer), block_tables.data_ptr(),
        int(block_tables.shape[1]), q_offsets.data_ptr(), ctx_lens.data_ptr(), _i32_ptr(qo), _i32_ptr(cl),
        int(cl.shape[0]), float(k_scale), float(v_scale), _stream_ptr(stream))
    if rc:
        raise DsvError("kv_append_fp8", rc)


def kv_pack_chunks_fp8(src: KVPool, block_tables, descs: ChunkDescs, chunk_buf, stream=None) -> None:
    """See ``kv_pack_chunks_fp8`` in include/dsv_attn.h."""
    _copy_tensors(src, block_tables, descs, chunk_buf, 1)
    rc = load_library().kv_pack_chunks_fp8(
        src.c, block_tables.data_ptr(), int(block_tables.shape[1]), descs.dev.data_ptr(),
        descs.host.ctypes.data, descs.n, chunk_buf.data_ptr(), _stream_ptr(stream))
    if rc:
        raise DsvError("kv_pack_chunks_fp8", rc)


def kv_unpack_chunks_fp8(chunk_buf, descs: ChunkDescs, dst: KVPool, dst_block_tables, stream=None) -> None:
    """See ``kv_unpack_chunks_fp8`` in include/dsv_attn.h."""
    _copy_tensors(dst, dst_block_tables, descs, chunk_buf, 1)
    rc = load_library().kv_unpack_chunks_fp8(
        chunk_buf.data_ptr(), descs.dev.data_ptr(), descs.host.ctypes.data, descs.n, dst.c,
        dst_block_tables.data_ptr(), int(dst_block_tables.shape[1]), _stream_ptr(stream))
    if rc:
        raise DsvError("kv_unpack_chunks_fp8", rc)
