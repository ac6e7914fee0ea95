"""Chunk-pipelined hand-off (paper section 4.3): the sending instance processes a prompt in
equal-sized chunks and ships the KV of chunk k while it computes chunk k+1; completed KV is
append-only, so the transfer needs no coherence with the running computation.

One GPU stands in for both servers: the compute stream appends each chunk's K/V to the source
pool and runs its attention, layer by layer; the transfer stream, chained to it by one event per
chunk, packs the finished chunk (all layers), copies the chunk buffer to a receive buffer (a
device-to-device copy in place of the wire) and unpacks it into the destination pool through
the receiver's block table.  Orchestration only: every step is a call into the C ABI.
"""
from __future__ import annotations

import time
from typing import Dict

import numpy as np


class ChunkedPrefill:
    """A prompt of ``total`` tokens (one request) cut into chunks of ``chunk`` tokens, ``layers``
    layers deep; synthetic Q/K/V.  ``run(pipelined)`` executes compute and transfer."""

    def __init__(self, total: int, chunk: int, layers: int, num_q_heads: int = 32, num_kv_heads: int = 8,
                 head_dim: int = 128, seed: int = 92859, k_new=None, v_new=None, q=None,
                 src_table=None, dst_table=None, dst_fill: int = 0):
        import torch

        from . import binding as dsv
        self.dsv, self.torch = dsv, torch
        assert total % chunk == 0 and chunk % 16 == 0
        self.total, self.chunk, self.L = total, chunk, layers
        self.Hq, self.Hkv, self.D = num_q_heads, num_kv_heads, head_dim
        self.n_chunks = total // chunk
        nb = total // 16
        rng = np.random.default_rng(seed)
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        shape_new = (layers, total, num_kv_heads, head_dim)
        rnd = lambda shape: torch.randn(shape, generator=g, device="cuda").to(torch.bfloat16)
        self.k_new = rnd(shape_new) if k_new is None else k_new      # what each layer's forward pass produced
        self.v_new = rnd(shape_new) if v_new is None else v_new
        self.q = rnd((layers, total, num_q_heads, head_dim)) if q is None else q
        st = rng.permutation(nb).astype(np.int32)[None] if src_table is None else src_table
        dt = rng.permutation(nb).astype(np.int32)[None] if dst_table is None else dst_table
        self.src_table_host, self.dst_table_host = st, dt
        self.src_table, self.dst_table = torch.from_numpy(st).cuda(), torch.from_numpy(dt).cuda()
        pool_shape = (layers, nb, 16, num_kv_heads, head_dim)
        self.src = dsv.KVPool(torch.zeros(pool_shape, dtype=torch.bfloat16, device="cuda"),
                              torch.zeros(pool_shape, dtype=torch.bfloat16, device="cuda"))
        self.dst = dsv.KVPool(torch.full(pool_shape, dst_fill, dtype=torch.int16, device="cuda").view(torch.bfloat16),
                              torch.full(pool_shape, dst_fill, dtype=torch.int16, device="cuda").view(torch.bfloat16))
        self.out = torch.empty((layers, total, num_q_heads, head_dim), dtype=torch.float32, device="cuda")
        self.chunk_elems = layers * 2 * chunk * num_kv_heads * head_dim
        self.send_buf = torch.empty(self.n_chunks * self.chunk_elems, dtype=torch.bfloat16, device="cuda")
        self.recv_buf = torch.empty_like(self.send_buf)
        # Per-chunk descriptors and batch descriptions, made once.
        self.descs = [dsv.ChunkDescs([[0, k * chunk, chunk, k * self.chunk_elems]]) for k in range(self.n_chunks)]
        self.q_off_host = np.array([0, chunk], np.int32)
        self.q_off = torch.from_numpy(self.q_off_host).cuda()
        self.ctx_host = [np.array([(k + 1) * chunk], np.int32) for k in range(self.n_chunks)]
        self.ctx = [torch.from_numpy(c).cuda() for c in self.ctx_host]
        ws = max(dsv.attn_mixed_batch_workspace_bytes(self.q_off_host, c, num_q_heads, num_kv_heads, head_dim)
                 for c in self.ctx_host)
        self.workspace = torch.empty(ws, dtype=torch.uint8, device="cuda")
        self.scale = 1.0 / float(np.sqrt(head_dim))
        self.s_compute, self.s_transfer = torch.cuda.Stream(), torch.cuda.Stream()
        self.payload_bytes = layers * 2 * total * num_kv_heads * head_dim * 2
        self.graphs = None

    def capture_graphs(self) -> None:
        """Records each chunk's computation (append + attention of every layer: 2-4 kernels per
        layer) into a HIP graph of its own, replayed by ``compute_chunk`` from then on with one
        host call per chunk, so that the compute stream is kept busy by the GPU's work and not
        by the host's enqueue rate.  The library's calls allocate nothing and record kernel
        launches only; one eager pass must have run before (first-call set-up)."""
        torch = self.torch
        torch.cuda.synchronize()
        graphs = []
        for k in range(self.n_chunks):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=self.s_compute):
                self._compute_chunk_eager(k)
            graphs.append(g)
        torch.cuda.synchronize()
        self.graphs = graphs

    def compute_chunk(self, k: int) -> None:
        if self.graphs is not None:
            with self.torch.cuda.stream(self.s_compute):
                self.graphs[k].replay()
            return
        self._compute_chunk_eager(k)

    def _compute_chunk_eager(self, k: int) -> None:
        dsv, c = self.dsv, self.chunk
        for l in range(self.L):
            dsv.kv_append(self.k_new[l, k * c:(k + 1) * c], self.v_new[l, k * c:(k + 1) * c], self.src, l,
                          self.src_table, self.q_off, self.ctx[k], self.q_off_host, self.ctx_host[k],
                          stream=self.s_compute)
            dsv.attn_mixed_batch(self.q[l, k * c:(k + 1) * c], self.out[l, k * c:(k + 1) * c], self.src, l,
                                 self.src_table, self.q_off, self.ctx[k], self.q_off_host, self.ctx_host[k],
                                 self.Hq, self.scale, self.workspace, stream=self.s_compute)

    def transfer_chunk(self, k: int) -> None:
        dsv, torch = self.dsv, self.torch
        dsv.kv_pack_chunks(self.src, self.src_table, self.descs[k], self.send_buf, stream=self.s_transfer)
        a, b = k * self.chunk_elems, (k + 1) * self.chunk_elems
        with torch.cuda.stream(self.s_transfer):
            self.recv_buf[a:b].copy_(self.send_buf[a:b], non_blocking=True)      # the wire
        dsv.kv_unpack_chunks(self.recv_buf, self.descs[k], self.dst, self.dst_table, stream=self.s_transfer)

    def run(self, pipelined: bool) -> dict:
        """Enqueues the whole prefill with its hand-off and waits for it.  Returns wall time and,
        from events on the two streams, the GPU time from the end of the last chunk's computation
        to the end of the last transfer: the transfer time that computation did not hide."""
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        compute_end = torch.cuda.Event(enable_timing=True)
        transfer_end = torch.cuda.Event(enable_timing=True)
        if pipelined:
            for k in range(self.n_chunks):
                self.compute_chunk(k)
                ev = torch.cuda.Event()
                ev.record(self.s_compute)
                self.s_transfer.wait_event(ev)          # chunk k's KV is complete and immutable from here on
                self.transfer_chunk(k)
            compute_end.record(self.s_compute)
        else:
            for k in range(self.n_chunks):
                self.compute_chunk(k)
            compute_end.record(self.s_compute)
            self.s_transfer.wait_event(compute_end)
            for k in range(self.n_chunks):
                self.transfer_chunk(k)
        transfer_end.record(self.s_transfer)
        self.s_compute.synchronize()
        self.s_transfer.synchronize()
        wall = time.perf_counter() - t0
        return {"wall_s": wall, "non_overlapped_transfer_ms": max(compute_end.elapsed_time(transfer_end), 0.0)}

    def run_compute_only(self) -> float:
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(self.n_chunks):
            self.compute_chunk(k)
        self.s_compute.synchronize()
        return time.perf_counter() - t0

    def run_transfer_only(self) -> float:
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(self.n_chunks):
            self.transfer_chunk(k)
        self.s_transfer.synchronize()
        return time.perf_counter() - t0


def measure(total: int = 8192, chunk: int = 512, layers: int = 8, rounds: int = 3, graphs: bool = True,
            **kw) -> Dict[str, float]:
    """Compute alone, transfer alone, transfer after all computation, and pipelined.  The paper's
    figure of merit is the transfer time that is not hidden behind computation, read on the
    GPU's own clock (events).  With ``graphs`` each chunk's computation is one graph launch, so
    the compute stream runs at the GPU's pace (enqueued call by call, the host's 20-40 us per
    call leave the GPU idle between kernels, and any transfer hides in the gaps)."""
    p = ChunkedPrefill(total, chunk, layers, **kw)
    p.run(True)                                             # warm-up (also fills the source pool)
    if graphs:
        p.capture_graphs()
        p.run(True)
    tc = min(p.run_compute_only() for _ in range(rounds))
    tt = min(p.run_transfer_only() for _ in range(rounds))
    seq = [p.run(False) for _ in range(rounds)]
    pipe = [p.run(True) for _ in range(rounds)]
    exposed_seq = float(np.median([r["non_overlapped_transfer_ms"] for r in seq]))
    exposed_pipe = float(np.median([r["non_overlapped_transfer_ms"] for r in pipe]))
    return {"prompt_tokens": total, "chunk_tokens": chunk, "chunks": p.n_chunks, "layers": layers,
            "compute_enqueued_as": "one HIP graph per chunk" if graphs else "one call per kernel group",
            "payload_bytes": p.payload_bytes, "compute_alone_wall_ms": tc * 1e3, "transfer_alone_wall_ms": tt * 1e3,
            "sequential_wall_ms": min(r["wall_s"] for r in seq) * 1e3,
            "pipelined_wall_ms": min(r["wall_s"] for r in pipe) * 1e3,
            "non_overlapped_transfer_sequential_ms": exposed_seq,
            "non_overlapped_transfer_pipelined_ms": exposed_pipe,
            "non_overlapped_transfer_reduction": (1.0 - exposed_pipe / exposed_seq) if exposed_seq > 0 else 0.0}
