#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5|lp] [--no-extras]
                    [--no-cpu-baseline]

A step is one attn_mixed_batch call (plan + attention kernels + merge) over one seeded synthetic
batch that is already resident in HBM.  The headline workload is the decode-heavy batch
(256 decodes, 32/8 heads, D=128, lognormal contexts); `value` is query tokens per second.  The
same JSON line carries the roofline of the dominant kernel (HIP events recorded around that
kernel on its own stream) and the fp64 CPU oracle timed on this machine's host cores.  Short extra
measurements of the other workloads (prefill-heavy, micro-request, hand-off copy) are attached
under "extras".
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "mixed-batch attention tokens/s; decode HBM GB/s & prefill MFMA util vs peak"
# HBM bytes per rows_kernel launch from rocprofv3 FETCH_SIZE + WRITE_SIZE, each scaled by what the
# counter reads for a plain 1 GiB copy (profiles/rows_kernel_c2_decode_heavy.md).
MEASURED_TRAFFIC_BYTES = {"c2_decode_heavy": 1.495e9}
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


# ---------------------------------------------------------------------------- HIP events
class HipEvents:
    """hipEvent_t pairs created straight on the HIP runtime (the library records them itself)."""

    def __init__(self):
        self.hip = None
        for line in open("/proc/self/maps"):
            if "libamdhip64" in line:
                self.hip = C.CDLL(line.split()[-1])
                break
        if self.hip is None:
            self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def create(self):
        ev = C.c_void_p()
        rc = self.hip.hipEventCreate(C.byref(ev))
        assert rc == 0 and ev.value
        return ev.value

    def record(self, ev, stream_ptr):
        assert self.hip.hipEventRecord(ev, stream_ptr) == 0

    def elapsed_ms(self, a, b) -> float:
        ms = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(ms), a, b)
        if rc != 0:
            self.hip.hipGetLastError()        # events never recorded: clear the sticky error
            raise AssertionError("hipEventElapsedTime rc=%d" % rc)
        return float(ms.value)

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)


# ---------------------------------------------------------------------------- algorithmic work
def decode_bytes(b, out_elem_bytes: int) -> int:
    """KV bytes of the decode rows (ctx tokens, not padded blocks) + Q + O + block-table entries."""
    dec = b.q_lens == 1
    ctx = b.ctx_lens[dec].astype(np.int64)
    kv = int(ctx.sum()) * 2 * b.Hkv * b.D * 2
    nq = int(dec.sum())
    return kv + nq * b.Hq * b.D * (2 + out_elem_bytes) + 4 * int(((ctx + 15) // 16).sum())


def prefill_flops(b) -> int:
    """4*D*Hq per causal (q,k) pair of the prefill spans; masked halves and padding not counted."""
    pre = b.q_lens > 1
    ql = b.q_lens[pre].astype(np.int64)
    prefix = b.ctx_lens[pre].astype(np.int64) - ql
    pairs = int((ql * prefix + ql * (ql + 1) // 2).sum())
    return 4 * b.D * b.Hq * pairs


# ---------------------------------------------------------------------------- device side
def upload(b):
    import torch
    import paper_2504_09285_amd as dsv

    def dev_bf16(u16):
        return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)

    d = argparse.Namespace()
    d.b = b
    d.q = dev_bf16(b.q)
    d.pool = dsv.KVPool(dev_bf16(b.k_pool[None]), dev_bf16(b.v_pool[None]))
    d.block_tables = torch.from_numpy(b.block_tables).cuda()
    d.q_offsets = torch.from_numpy(b.q_offsets).cuda()
    d.ctx_lens = torch.from_numpy(b.ctx_lens).cuda()
    nbytes = dsv.attn_mixed_batch_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
    d.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    d.out = torch.empty(d.q.shape, dtype=torch.bfloat16, device="cuda")
    return d


def attn_step(d):
    import paper_2504_09285_amd as dsv
    if getattr(d, "step", None) is not None:
        return d.step()
    b = d.b
    dsv.attn_mixed_batch(d.q, d.out, d.pool, 0, d.block_tables, d.q_offsets, d.ctx_lens,
                         b.q_offsets, b.ctx_lens, b.Hq, b.scale, d.workspace)


def time_attention(d, steps, warmup, kernel_ids, hev):
    """Wall time of `steps` calls between device synchronisations, plus per-kernel event times."""
    import torch
    import paper_2504_09285_amd as dsv
    for _ in range(warmup):
        attn_step(d)
    torch.cuda.synchronize()
    evs = {k: [(hev.create(), hev.create()) for _ in range(steps)] for k in kernel_ids}
    t0 = time.perf_counter()
    for s in range(steps):
        for k in kernel_ids:
            dsv.dsv_profile_events(k, *evs[k][s])
        attn_step(d)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for k in kernel_ids:
        dsv.dsv_profile_events(k, None, None)
    per_kernel = {}
    for k in kernel_ids:
        try:
            ms = [hev.elapsed_ms(a, b) for a, b in evs[k]]
            per_kernel[k] = float(np.mean(ms))
        except AssertionError:
            per_kernel[k] = None          # kernel not launched for this batch
        for a, b in evs[k]:
            hev.destroy(a)
            hev.destroy(b)
    return (t1 - t0) / steps, per_kernel


def timed_step(d, steps, warmup, hev, ids=None):
    """Seconds per step with events around the dominant kernel only, and every kernel's time:
    the dominant one from the timed steps, the others from a short pass before."""
    import paper_2504_09285_amd as dsv
    if ids is None:
        ids = [dsv.KERNEL_ROWS, dsv.KERNEL_TILES, dsv.KERNEL_MERGE, dsv.KERNEL_PLAN, dsv.KERNEL_MIXED,
               dsv.KERNEL_STAGE]
    _, probe = time_attention(d, max(min(steps, 5), 2), warmup, ids, hev)
    dominant = max((k for k in ids if probe[k] is not None), key=lambda k: probe[k])
    sec, main = time_attention(d, steps, 2, [dominant], hev)
    per_kernel = dict(probe)
    per_kernel[dominant] = main[dominant]
    return sec, per_kernel


def bench_attention(b, steps, warmup, hev):
    """The step is timed as the library runs it (a batch holding prefill tiles and row items runs
    them in one launch).  Recording events around every kernel costs about 20 us per step, so the
    timed steps carry the events of the dominant kernel only (the one the roofline is about);
    which kernel that is, and the times of the others, come from a short pass before.  The
    per-kernel times that feed the roofline fractions of a mixed batch come from a further pass with
    the two kernels launched apart (DSV_MIXED_LAUNCH=0), where each can be timed."""
    import paper_2504_09285_amd as dsv
    d = upload(b)
    ids = [dsv.KERNEL_ROWS, dsv.KERNEL_TILES, dsv.KERNEL_MERGE, dsv.KERNEL_PLAN, dsv.KERNEL_MIXED]
    sec, per_kernel = timed_step(d, steps, warmup, hev, ids)
    res = {"workload": b.name, "ms_per_step": sec * 1e3, "tokens_per_s": b.total_q / sec,
           "total_q": b.total_q, "num_seqs": b.num_seqs}
    if per_kernel[dsv.KERNEL_MIXED] is not None:
        res["mixed_launch_ms"] = per_kernel[dsv.KERNEL_MIXED]
        os.environ["DSV_MIXED_LAUNCH"] = "0"
        try:
            sec_apart, per_kernel = time_attention(d, max(steps // 2, 3), 2, ids, hev)
        finally:
            del os.environ["DSV_MIXED_LAUNCH"]
        res["ms_per_step_kernels_apart"] = sec_apart * 1e3
    rows_ms, tiles_ms = per_kernel[dsv.KERNEL_ROWS], per_kernel[dsv.KERNEL_TILES]
    res["kernel_ms"] = {"rows": rows_ms, "tiles": tiles_ms, "merge": per_kernel[dsv.KERNEL_MERGE],
                        "plan": per_kernel[dsv.KERNEL_PLAN]}
    nbytes = decode_bytes(b, 2)
    flops = prefill_flops(b)
    if rows_ms and nbytes:
        gbs = nbytes / (rows_ms * 1e-3) / 1e9
        res["decode"] = {"algorithmic_bytes": nbytes, "GB/s": gbs, "frac_hbm_peak": gbs / HBM_PEAK_GBS}
    if tiles_ms and flops:
        tf = flops / (tiles_ms * 1e-3) / 1e12
        res["prefill"] = {"algorithmic_flops": flops, "TFLOP/s": tf, "frac_mfma_peak": tf / MFMA_BF16_PEAK_TFLOPS}
    return res, d


def bench_shared_plan(d, layers, iterations, warmup):
    """A serving iteration runs one batch through every layer: one attn_mixed_batch_plan, then one
    planned call per layer (the same single-layer pool stands in for every layer: the KV does not
    fit any cache, so each call streams it from HBM).  Wall time per layer call, plan included."""
    import torch
    import paper_2504_09285_amd as dsv
    b = d.b

    def iteration():
        plan = dsv.attn_mixed_batch_plan(d.block_tables, d.q_offsets, d.ctx_lens, b.q_offsets, b.ctx_lens,
                                         b.Hq, b.Hkv, b.D, d.workspace)
        for _ in range(layers):
            dsv.attn_mixed_batch_planned(plan, d.q, d.out, d.pool, 0, d.block_tables, d.q_offsets, d.ctx_lens,
                                         b.q_offsets, b.ctx_lens, b.Hq, b.scale, d.workspace)
    for _ in range(warmup):
        iteration()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iterations):
        iteration()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / (iterations * layers)
    return {"workload": b.name, "layers_per_plan": layers, "ms_per_layer_call": sec * 1e3,
            "tokens_per_s": b.total_q / sec}


def settle_runtime():
    """The HIP runtime stalls the host once per process, for about 70 ms, somewhere around its
    thousandth kernel launch (measured on this image: 18 us per call before and after, 714 us per
    call over one block of 100 calls).  Long steps hide it behind queued work; short ones (config
    1, the profile table) would carry it into whichever timed region it falls.  A few hundred
    untimed calls on a tiny batch take the process past it before anything is timed."""
    import torch
    from workloads import gen
    d = upload(gen.make_batch("settle", 1, 8, 2, 64, [(1, 40), (20, 30), (1, 300)]))
    for _ in range(500):
        attn_step(d)
    torch.cuda.synchronize()


def bench_append(b, steps, warmup, hev):
    """kv_append of the batch's new tokens (the step before attention): read once, written once."""
    import torch
    import paper_2504_09285_amd as dsv

    def dev_bf16(u16):
        return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)

    pool = dsv.KVPool(dev_bf16(b.k_pool[None]), dev_bf16(b.v_pool[None]))
    bt = torch.from_numpy(np.ascontiguousarray(b.block_tables, dtype=np.int32)).cuda()
    qo, cl = torch.from_numpy(b.q_offsets).cuda(), torch.from_numpy(b.ctx_lens).cuda()
    k_new = torch.randn((b.total_q, b.Hkv, b.D), device="cuda").to(torch.bfloat16)
    v_new = torch.randn((b.total_q, b.Hkv, b.D), device="cuda").to(torch.bfloat16)
    stream = torch.cuda.current_stream().cuda_stream or None
    fn = lambda: dsv.kv_append(k_new, v_new, pool, 0, bt, qo, cl, b.q_offsets, b.ctx_lens)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    evs = [(hev.create(), hev.create()) for _ in range(steps)]
    for e0, e1 in evs:
        hev.record(e0, stream)
        fn()
        hev.record(e1, stream)
    torch.cuda.synchronize()
    ms = float(np.median([hev.elapsed_ms(e0, e1) for e0, e1 in evs]))
    nbytes = 2 * 2 * b.total_q * b.Hkv * b.D * 2          # K and V, read + written
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"workload": b.name, "new_tokens": int(b.total_q), "ms": ms, "bytes": nbytes, "GB/s": gbs,
            "frac_hbm_peak": gbs / HBM_PEAK_GBS}


def bench_handoff(h, steps, warmup, hev):
    import torch
    import paper_2504_09285_amd as dsv

    def dev_bf16(u16):
        return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)

    src = dsv.KVPool(dev_bf16(h.src_k), dev_bf16(h.src_v))
    dst = dsv.KVPool(dev_bf16(h.dst_k), dev_bf16(h.dst_v))
    st, dt = torch.from_numpy(h.src_tables).cuda(), torch.from_numpy(h.dst_tables).cuda()
    descs = dsv.ChunkDescs(h.chunks)
    buf = torch.empty(h.chunk_elems, dtype=torch.bfloat16, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream or None
    out = {}
    for name, fn in (("pack", lambda: dsv.kv_pack_chunks(src, st, descs, buf)),
                     ("unpack", lambda: dsv.kv_unpack_chunks(buf, descs, dst, dt))):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        evs = [(hev.create(), hev.create()) for _ in range(steps)]
        for a, b in evs:
            hev.record(a, stream)
            fn()
            hev.record(b, stream)
        torch.cuda.synchronize()
        ms = float(np.mean([hev.elapsed_ms(a, b) for a, b in evs]))
        gbs = 2 * h.payload_bytes / (ms * 1e-3) / 1e9
        out[name] = {"ms": ms, "GB/s": gbs, "frac_hbm_peak": gbs / HBM_PEAK_GBS}
    out["payload_bytes"] = h.payload_bytes
    out["workload"] = h.name
    return out


def bench_fp8kv(steps, warmup, hev):
    """Second workload: the same shapes on a cache of 8-bit (E4M3) codes.  Decode streams half
    the bytes per token, so tokens/s should double at the same GB/s; prefill spans pay for a bf16
    copy of their contexts (the "stage" kernel); chunks are half the size."""
    import torch
    import paper_2504_09285_amd as dsv
    from workloads import gen
    out = {}
    ids = [dsv.KERNEL_ROWS, dsv.KERNEL_TILES, dsv.KERNEL_MERGE, dsv.KERNEL_PLAN, dsv.KERNEL_STAGE]
    for b in (gen.config2_fp8kv(), gen.config3_fp8kv()):
        d = argparse.Namespace()
        d.b = b
        d.q = torch.from_numpy(np.ascontiguousarray(b.q).view(np.int16)).cuda().view(torch.bfloat16)
        d.pool = dsv.KVPool(torch.from_numpy(b.k_pool[None]).cuda(), torch.from_numpy(b.v_pool[None]).cuda())
        d.block_tables = torch.from_numpy(b.block_tables).cuda()
        d.q_offsets, d.ctx_lens = torch.from_numpy(b.q_offsets).cuda(), torch.from_numpy(b.ctx_lens).cuda()
        nbytes = dsv.attn_mixed_batch_fp8kv_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
        d.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        d.out = torch.empty(d.q.shape, dtype=torch.bfloat16, device="cuda")
        d.step = lambda d=d, b=b: dsv.attn_mixed_batch_fp8kv(
            d.q, d.out, d.pool, 0, d.block_tables, d.q_offsets, d.ctx_lens, b.q_offsets, b.ctx_lens, b.Hq,
            b.scale, b.meta["k_scale"], b.meta["v_scale"], d.workspace)
        sec, pk = timed_step(d, steps, warmup, hev, ids)
        r = {"ms_per_step": sec * 1e3, "tokens_per_s": b.total_q / sec, "workspace_bytes": int(nbytes),
             "kernel_ms": {"rows": pk[dsv.KERNEL_ROWS], "tiles": pk[dsv.KERNEL_TILES], "merge": pk[dsv.KERNEL_MERGE],
                           "plan": pk[dsv.KERNEL_PLAN], "stage": pk[dsv.KERNEL_STAGE]}}
        dec = b.q_lens == 1
        ctx = b.ctx_lens[dec].astype(np.int64)
        kv_bytes = int(ctx.sum()) * 2 * b.Hkv * b.D + int(dec.sum()) * b.Hq * b.D * 4 + 4 * int(((ctx + 15) // 16).sum())
        if pk[dsv.KERNEL_ROWS]:
            gbs = kv_bytes / (pk[dsv.KERNEL_ROWS] * 1e-3) / 1e9
            r["decode"] = {"algorithmic_bytes": kv_bytes, "GB/s": gbs, "frac_hbm_peak": gbs / HBM_PEAK_GBS}
        if pk[dsv.KERNEL_TILES]:
            tf = prefill_flops(b) / (pk[dsv.KERNEL_TILES] * 1e-3) / 1e12
            r["prefill"] = {"TFLOP/s": tf, "frac_mfma_peak": tf / MFMA_BF16_PEAK_TFLOPS}
        out[b.name] = r
        del d
    h = gen.config5_handoff_fp8kv(layers=4)
    src = dsv.KVPool(torch.from_numpy(h.src_k).cuda(), torch.from_numpy(h.src_v).cuda())
    dst = dsv.KVPool(torch.from_numpy(h.dst_k).cuda(), torch.from_numpy(h.dst_v).cuda())
    st, dt = torch.from_numpy(h.src_tables).cuda(), torch.from_numpy(h.dst_tables).cuda()
    descs = dsv.ChunkDescs(h.chunks)
    buf = torch.empty(h.chunk_elems, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream or None
    ho = {"payload_bytes": h.payload_bytes}
    for name, fn in (("pack", lambda: dsv.kv_pack_chunks_fp8(src, st, descs, buf)),
                     ("unpack", lambda: dsv.kv_unpack_chunks_fp8(buf, descs, dst, dt))):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        evs = [(hev.create(), hev.create()) for _ in range(10)]
        for a, e in evs:
            hev.record(a, stream)
            fn()
            hev.record(e, stream)
        torch.cuda.synchronize()
        ms = float(np.mean([hev.elapsed_ms(a, e) for a, e in evs]))
        gbs = 2 * h.payload_bytes / (ms * 1e-3) / 1e9
        ho[name] = {"ms": ms, "GB/s": gbs, "frac_hbm_peak": gbs / HBM_PEAK_GBS}
    out["handoff_c5_4layers_fp8kv"] = ho
    return out


def bench_config4(threads, steps, warmup, hev):
    """Config 4: the split prompt's prefix reaches its second span through GPU pack/unpack, then
    one mixed batch (two prefill spans + 128 decodes).  Reports the hand-off time and the step."""
    import torch
    import paper_2504_09285_amd as dsv
    from workloads import gen
    b, sp = gen.config4(threads=threads)
    t = np.arange(sp.k, sp.total)
    for pool in (b.k_pool, b.v_pool):
        pool[b.block_tables[1, t // 16], t % 16] = pool[b.block_tables[0, t // 16], t % 16]
    d = upload(b)
    descs = dsv.ChunkDescs(sp.chunks)
    buf = torch.zeros(sp.chunk_elems, dtype=torch.bfloat16, device="cuda")
    src_tbl, dst_tbl = d.block_tables[0:1].contiguous(), d.block_tables[1:2].contiguous()
    stream = torch.cuda.current_stream().cuda_stream or None
    e0, e1 = hev.create(), hev.create()
    torch.cuda.synchronize()
    hev.record(e0, stream)
    dsv.kv_pack_chunks(d.pool, src_tbl, descs, buf)
    dsv.kv_unpack_chunks(buf, descs, d.pool, dst_tbl)
    hev.record(e1, stream)
    torch.cuda.synchronize()
    handoff_ms = hev.elapsed_ms(e0, e1)
    ids = [dsv.KERNEL_ROWS, dsv.KERNEL_TILES, dsv.KERNEL_MERGE, dsv.KERNEL_PLAN, dsv.KERNEL_MIXED]
    sec, pk = timed_step(d, steps, warmup, hev, ids)                   # as the library runs it: one mixed launch
    mixed_ms = pk[dsv.KERNEL_MIXED]
    os.environ["DSV_MIXED_LAUNCH"] = "0"                               # the two kernels apart, to time each
    try:
        sec_apart, pk = time_attention(d, steps, warmup, ids, hev)
    finally:
        del os.environ["DSV_MIXED_LAUNCH"]
    nbytes, flops = decode_bytes(b, 2), prefill_flops(b)
    t_mem, t_mfma = nbytes / (HBM_PEAK_GBS * 1e9), flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    rows_ms, tiles_ms = pk[dsv.KERNEL_ROWS], pk[dsv.KERNEL_TILES]
    return {"workload": b.name, "split_k": sp.k, "ms_per_step": sec * 1e3, "tokens_per_s": b.total_q / sec,
            "mixed_launch_ms": mixed_ms, "ms_per_step_kernels_apart": sec_apart * 1e3,
            "kernel_ms": {"rows": rows_ms, "tiles": tiles_ms, "merge": pk[dsv.KERNEL_MERGE], "plan": pk[dsv.KERNEL_PLAN]},
            "handoff_pack_unpack_ms": handoff_ms, "handoff_chunks": int(len(sp.chunks)),
            "decode": {"GB/s": nbytes / (rows_ms * 1e-3) / 1e9, "frac_hbm_peak": nbytes / (rows_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "prefill": {"TFLOP/s": flops / (tiles_ms * 1e-3) / 1e12, "frac_mfma_peak": flops / (tiles_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
            "bound_ms": {"hbm": t_mem * 1e3, "mfma": t_mfma * 1e3},
            "frac_of_overlap_bound": max(t_mem, t_mfma) / sec}


def bench_concurrent(b, h, rounds, hev):
    """Attention on one stream, pack+unpack on a second one (config 5): each alone, then together."""
    import torch
    import paper_2504_09285_amd as dsv
    d = upload(b)

    def dev_bf16(u16):
        return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)

    src = dsv.KVPool(dev_bf16(h.src_k), dev_bf16(h.src_v))
    dst = dsv.KVPool(dev_bf16(h.dst_k), dev_bf16(h.dst_v))
    st, dt = torch.from_numpy(h.src_tables).cuda(), torch.from_numpy(h.dst_tables).cuda()
    descs = dsv.ChunkDescs(h.chunks)
    buf = torch.empty(h.chunk_elems, dtype=torch.bfloat16, device="cuda")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()

    def attn():
        bb = d.b
        dsv.attn_mixed_batch(d.q, d.out, d.pool, 0, d.block_tables, d.q_offsets, d.ctx_lens, bb.q_offsets,
                             bb.ctx_lens, bb.Hq, bb.scale, d.workspace, stream=s1)

    def copy():
        dsv.kv_pack_chunks(src, st, descs, buf, stream=s2)
        dsv.kv_unpack_chunks(buf, descs, dst, dt, stream=s2)

    def timed(fns):
        for f in fns:
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(rounds):
            for f in fns:
                f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / rounds

    ta, tc, tb = timed([attn]), timed([copy]), timed([attn, copy])
    ab, cb = decode_bytes(b, 2), 4 * h.payload_bytes
    return {"attention": b.name, "handoff": h.name, "handoff_layers": h.L,
            "attn_alone_ms": ta * 1e3, "handoff_alone_ms": tc * 1e3, "together_ms": tb * 1e3,
            "attn_alone_GB/s": ab / ta / 1e9, "handoff_alone_GB/s": cb / tc / 1e9,
            "together_GB/s": (ab + cb) / tb / 1e9, "together_frac_hbm_peak": (ab + cb) / tb / 1e9 / HBM_PEAK_GBS,
            "overlap_gain": (ta + tc) / tb}


# ---------------------------------------------------------------------------- CPU baseline
def cpu_baseline(b, target_seconds=12.0):
    """The fp64 oracle as it stands, on this machine's host cores, on a bounded sample of the batch:
    eighths of the batch (whole sequences, all heads) are processed in turn, wrapping around,
    until about target_seconds of CPU work has been done."""
    import oracle
    oracle.build()
    n = b.num_seqs
    done_tokens, elapsed, used = 0, 0.0, 0
    step = max(1, n // 8)
    while elapsed < target_seconds and used < 40 * n:
        idx = (np.arange(used, used + step)) % n
        qo = np.zeros(len(idx) + 1, np.int32)
        np.cumsum(b.q_lens[idx], out=qo[1:])
        q = np.concatenate([b.q[b.q_offsets[i]:b.q_offsets[i + 1]] for i in idx])
        t0 = time.perf_counter()
        oracle.attn_mixed_batch(q, b.k_pool, b.v_pool, b.block_tables[idx], qo, b.ctx_lens[idx], b.scale)
        elapsed += time.perf_counter() - t0
        done_tokens += int(qo[-1])
        used += len(idx)
    return {"value": done_tokens / elapsed, "unit": "tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": elapsed,
            "sample": "%d sequences (%.1f passes over the %d of %s; %d query tokens), all heads"
                      % (used, used / n, n, b.name, done_tokens)}


# ---------------------------------------------------------------------------- main
def make_workload(name, threads):
    from workloads import gen
    if name == "c2":
        return gen.config2(threads=threads)
    if name == "c3":
        return gen.config3(threads=threads)
    if name == "c4":
        return gen.config4(threads=threads)[0]
    if name == "c5":
        return gen.config5_attention(threads=threads)
    if name == "lp":
        return gen.long_prefix_chunk(threads=threads)
    raise SystemExit("unknown workload " + name)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "c5", "lp"])
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--full-extras", action="store_true", help="config 5 at full context lengths (16 GB of KV)")
    ap.add_argument("--fp8kv-only", action="store_true",
                    help="run only the second workload (8-bit KV cache) and print its results")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB device copy, 10 times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on one GPU only (no sharding, no collectives); "
                         "use --gpus 1")
    import torch
    import paper_2504_09285_amd as dsv
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "copies": 10}))
        return
    dsv.load_library()
    threads = min(16, os.cpu_count() or 8)
    hev = HipEvents()
    settle_runtime()
    if args.fp8kv_only:
        print(json.dumps({"fp8kv": bench_fp8kv(args.steps, args.warmup, hev)}))
        return

    b = make_workload(args.workload, threads)
    res, d = bench_attention(b, args.steps, args.warmup, hev)
    line = {
        "metric": METRIC, "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": b.name, "num_seqs": b.num_seqs, "total_q": b.total_q,
                   "q_heads": b.Hq, "kv_heads": b.Hkv, "head_dim": b.D, "block_size": 16,
                   "kv_tokens": int(b.ctx_lens.sum()), "out_dtype": "bf16"},
        "kernel_ms": res["kernel_ms"],
    }
    if "prefill" in res and (args.workload in ("c3", "lp")):
        p = res["prefill"]
        line["roofline"] = {"bound": "mfma", "achieved": p["TFLOP/s"], "peak": MFMA_BF16_PEAK_TFLOPS,
                            "unit": "TFLOP/s", "frac": p["frac_mfma_peak"], "traffic": None,
                            "kernel": "prefill_tiles_kernel"}
    elif "decode" in res:
        p = res["decode"]
        line["roofline"] = {"bound": "hbm", "achieved": p["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": p["frac_hbm_peak"], "traffic": MEASURED_TRAFFIC_BYTES.get(b.name),
                            "kernel": "rows_kernel",
                            "algorithmic_bytes": p["algorithmic_bytes"]}
    if "prefill" in res:
        line["prefill"] = res["prefill"]
    if "decode" in res:
        line["decode"] = res["decode"]

    if not args.no_extras:
        from workloads import gen
        extras = {}
        if args.workload == "c2":
            # the same batch with the work lists built once per 32 layer calls
            extras["c2_one_plan_per_32_layers"] = bench_shared_plan(d, 32, 6, 1)
        h = gen.config5_handoff(layers=4, threads=threads)     # 8 x 8192 tokens, 256-token chunks, 4 of 32 layers
        extras["handoff_c5_4layers"] = bench_handoff(h, 10, 2, hev)
        del h
        if args.workload != "c3":
            r3, d3 = bench_attention(gen.config3(threads=threads), 40, 5, hev)
            extras["c3_prefill_heavy"] = {k: r3[k] for k in ("ms_per_step", "tokens_per_s", "mixed_launch_ms", "ms_per_step_kernels_apart", "kernel_ms", "prefill", "decode") if k in r3}
            del d3
        keys = ("ms_per_step", "tokens_per_s", "mixed_launch_ms", "ms_per_step_kernels_apart", "kernel_ms", "prefill", "decode")
        # config 3's segments with the head counts of the models the paper serves (Qwen-2.5-14B/32B:
        # 40 query heads on 8 KV heads, five per KV head)
        rq, dq = bench_attention(gen.config3_heads(40, 8, threads=threads), 30, 5, hev)
        extras["c3_segments_40q_8kv_heads"] = {k: rq[k] for k in keys if k in rq}
        del dq
        r1, d1 = bench_attention(gen.config1()[0], 20, 3, hev)          # the tiny case: launch-bound
        extras["c1_tiny"] = {k: r1[k] for k in keys if k in r1}
        del d1
        if args.workload != "c5":
            r5, d5 = bench_attention(gen.config5_attention(threads=threads), 20, 3, hev)   # full contexts, one layer
            extras["c5_long_context"] = {k: r5[k] for k in keys if k in r5}
            del d5
        extras["kv_append_c3"] = bench_append(gen.config3(threads=threads), 20, 3, hev)
        extras["c4_micro_request"] = bench_config4(threads, 40, 5, hev)
        extras["fp8kv"] = bench_fp8kv(20, 3, hev)
        # A 512-token chunk on a 130,560-token prefix: eight query tiles, cut along the context.
        rl, dl = bench_attention(gen.long_prefix_chunk(threads=threads), 30, 5, hev)
        extras["long_prefix_chunk"] = {k: rl[k] for k in ("ms_per_step", "tokens_per_s", "kernel_ms", "prefill") if k in rl}
        del dl
        # Chunk-pipelined hand-off (paper section 4.3): transfer of chunk k next to computation of k+1.
        from paper_2504_09285_amd.chunk_pipeline import measure as measure_chunk_pipeline
        extras["chunk_pipelined_handoff"] = measure_chunk_pipeline(8192, 512, 8)
        # The local scheduler's profile table (paper section 4.2) on the grid of the paper's
        # batch-latency figure: prefill length x decode context x number of decodes -> step ms.
        from paper_2504_09285_amd.local_scheduler import ProfileTable, sweep
        tbl = sweep(ProfileTable(plen_step=512), plens=(0, 512, 1024), ctxs=(128, 1024), dnums=(8, 32, 64), steps=5)
        extras["profile_table_ms"] = {"plen=%d,ctx=%d,dnum=%d" % k: round(v, 4) for k, v in sorted(tbl.entries().items())}
        extras["max_prefill_allowed"] = {"target_ms=0.1,ctx=1024,dnum=32": tbl.max_prefill_allowed(0.1, 1024, 32),
                                         "target_ms=0.2,ctx=1024,dnum=32": tbl.max_prefill_allowed(0.2, 1024, 32)}
        if args.full_extras:
            extras["c5_two_streams"] = bench_concurrent(gen.config5_attention(threads=threads),
                                                        gen.config5_handoff(layers=8, threads=threads), 5, hev)
        else:
            extras["c5_two_streams_quarter_contexts"] = bench_concurrent(
                gen.config5_attention(shrink=4, threads=threads), gen.config5_handoff(layers=4, threads=threads), 5, hev)
        line["extras"] = extras
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(b)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
