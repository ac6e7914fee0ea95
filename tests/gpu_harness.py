"""Helpers for the GPU parity tests: upload a seeded workload, call the C ABI through the thin
binding, bring results back as numpy.  torch is used only for device memory."""
import numpy as np
import torch

import paper_2504_09285_amd as dsv


def dev_bf16(u16: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)


def host_u16(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


class DeviceBatch:
    """Device copy of a workloads.AttnBatch (single-layer pool)."""

    def __init__(self, b, k_pool=None, v_pool=None, block_tables=None):
        self.b = b
        self.q = dev_bf16(b.q)
        self.pool = dsv.KVPool(dev_bf16((b.k_pool if k_pool is None else k_pool)[None]),
                               dev_bf16((b.v_pool if v_pool is None else v_pool)[None]))
        bt = b.block_tables if block_tables is None else block_tables
        self.block_tables = torch.from_numpy(np.ascontiguousarray(bt, dtype=np.int32)).cuda()
        self.q_offsets = torch.from_numpy(b.q_offsets).cuda()
        self.ctx_lens = torch.from_numpy(b.ctx_lens).cuda()
        nbytes = dsv.attn_mixed_batch_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
        assert nbytes > 0
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")

    def run(self, out_dtype=torch.float32, stream=None, fill=None):
        b = self.b
        out = torch.empty(self.q.shape, dtype=out_dtype, device="cuda")
        if fill is not None:
            out.fill_(fill)
        dsv.attn_mixed_batch(self.q, out, self.pool, 0, self.block_tables, self.q_offsets,
                             self.ctx_lens, b.q_offsets, b.ctx_lens, b.Hq, b.scale, self.workspace,
                             stream=stream)
        return out


def run_attention(b, out_dtype=torch.float32, **over) -> np.ndarray:
    out = DeviceBatch(b, **over).run(out_dtype, fill=float("nan"))
    torch.cuda.synchronize()
    if out_dtype == torch.bfloat16:
        return host_u16(out)
    return out.cpu().numpy()


class DeviceHandoff:
    """Device copy of a workloads.Handoff."""

    def __init__(self, h):
        self.h = h
        self.src = dsv.KVPool(dev_bf16(h.src_k), dev_bf16(h.src_v))
        self.dst = dsv.KVPool(dev_bf16(h.dst_k), dev_bf16(h.dst_v))
        self.src_tables = torch.from_numpy(h.src_tables).cuda()
        self.dst_tables = torch.from_numpy(h.dst_tables).cuda()
        self.descs = dsv.ChunkDescs(h.chunks)
        self.chunk_buf = torch.full((max(h.chunk_elems, 8),), -21555, dtype=torch.int16,
                                    device="cuda").view(torch.bfloat16)

    def pack(self, stream=None):
        dsv.kv_pack_chunks(self.src, self.src_tables, self.descs, self.chunk_buf, stream=stream)

    def unpack(self, stream=None):
        dsv.kv_unpack_chunks(self.chunk_buf, self.descs, self.dst, self.dst_tables, stream=stream)


def dev_u8(u8: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(u8, dtype=np.uint8)).cuda()


class DeviceBatchFp8:
    """Device copy of a workloads.AttnBatch whose single-layer pools hold E4M3 codes (uint8)."""

    def __init__(self, b, k_pool=None, v_pool=None):
        self.b = b
        self.q = dev_bf16(b.q)
        self.pool = dsv.KVPool(dev_u8((b.k_pool if k_pool is None else k_pool)[None]),
                               dev_u8((b.v_pool if v_pool is None else v_pool)[None]))
        self.block_tables = torch.from_numpy(np.ascontiguousarray(b.block_tables, dtype=np.int32)).cuda()
        self.q_offsets = torch.from_numpy(b.q_offsets).cuda()
        self.ctx_lens = torch.from_numpy(b.ctx_lens).cuda()
        nbytes = dsv.attn_mixed_batch_fp8kv_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
        assert nbytes > 0
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")

    def run(self, out_dtype=torch.float32, stream=None, fill=None, k_scale=None, v_scale=None):
        b = self.b
        out = torch.empty(self.q.shape, dtype=out_dtype, device="cuda")
        if fill is not None:
            out.fill_(fill)
        dsv.attn_mixed_batch_fp8kv(self.q, out, self.pool, 0, self.block_tables, self.q_offsets,
                                   self.ctx_lens, b.q_offsets, b.ctx_lens, b.Hq, b.scale,
                                   b.meta["k_scale"] if k_scale is None else k_scale,
                                   b.meta["v_scale"] if v_scale is None else v_scale,
                                   self.workspace, stream=stream)
        return out


def run_attention_fp8kv(b, out_dtype=torch.float32, **over) -> np.ndarray:
    out = DeviceBatchFp8(b, **over).run(out_dtype, fill=float("nan"))
    torch.cuda.synchronize()
    if out_dtype == torch.bfloat16:
        return host_u16(out)
    return out.cpu().numpy()


def loaded_hip_runtime():
    """The HIP runtime already in this process (torch's), for tests that call it directly."""
    import ctypes
    for line in open("/proc/self/maps"):
        if "libamdhip64" in line:
            return ctypes.CDLL(line.split()[-1])
    raise RuntimeError("no HIP runtime loaded")
