#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c3h|c4|c5|lp] [--no-extras]
                    [--no-cpu-baseline] [--handoff-only] [--fp8kv-only] [--calibrate-copy]

A step is one attn_mixed_batch call (plan + attention kernels + merge) over one seeded synthetic
batch that is already resident in HBM.  The headline workload is the largest of the five
configurations: config 5's attention, 64 decodes on contexts of 16K-128K tokens, 14.6 GB of KV
streamed per step (32/8 heads, D=128); `value` is query tokens per second.  The same JSON line
carries
  roofline      the dominant kernel of the headline step (HIP events recorded around that kernel
                on its own stream, over the timed steps),
  rooflines     one entry per target kernel and workload: the row kernel on configs 2 and 5, the
                MFMA kernel on config 3 (and with 40/8 heads), the mixed launch on config 4 against
                its overlap bound, pack / unpack / append, the 8-bit cache,
  ceilings      what this GPU delivers on plain streaming and MFMA loops (the library's
                calibration kernels), next to the nominal peaks the fractions are taken against,
  cpu_baseline  the fp64 oracle timed on this machine's host cores on a bounded sample of the headline
                workload; cpu_baselines: the same for the other configurations and the hand-off,
  extras        further short measurements (two streams at config 5's full size, shared plan,
                chunk-pipelined hand-off, profile table, ...).
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
PROFILES = os.path.join(ROOT, "profiles")


def profile_traffic(kernel: str, workload: str):
    """HBM bytes per launch of a kernel on a workload as measured with rocprofv3 counters (two
    --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size): NOT measured in
    this run, read from the committed summary profiles/<kernel>_<workload>.md, from its line
    `traffic_bytes_per_launch: N`.  (None, None) if the summary has no such line."""
    import re
    path = os.path.join(PROFILES, "%s_%s.md" % (kernel, workload))
    try:
        m = re.search(r"^traffic_bytes_per_launch\s*[:=]\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    except OSError:
        return None, None
    return (float(m.group(1)), "profiles/%s (rocprofv3 --pmc, separate run)" % os.path.basename(path)) if m else (None, None)


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


def size_workspace(d):
    """(Re)allocates the workspace for the batch under the knobs in force now: what a call needs
    depends on how the planner cuts the batch, which the environment knobs can change."""
    import torch
    import paper_2504_09285_amd as dsv
    b = d.b
    nbytes = dsv.attn_mixed_batch_workspace_bytes(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
    if getattr(d, "workspace", None) is None or d.workspace.numel() < nbytes:
        d.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")


def attn_step(d):
    import paper_2504_09285_amd as dsv
    if getattr(d, "step", None) is not None:
        return d.step()
    b = d.b
    dsv.attn_mixed_batch(d.q, d.out, d.pool, 0, d.block_tables, d.q_offsets, d.ctx_lens,
                         b.q_offsets, b.ctx_lens, b.Hq, b.scale, d.workspace)


def time_attention(d, steps, warmup, kernel_ids, hev, min_warm_ms=0.0):
    """Wall time of `steps` calls between device synchronisations, plus per-kernel event times."""
    import torch
    import paper_2504_09285_amd as dsv
    for _ in range(warmup):
        attn_step(d)
    torch.cuda.synchronize()
    if min_warm_ms:
        # Short steps: the untimed calls go on until the GPU has been busy for a while, so that its
        # clocks have left their idle state before anything is timed.
        t_w = time.perf_counter()
        while (time.perf_counter() - t_w) * 1e3 < min_warm_ms:
            for _ in range(10):
                attn_step(d)
            torch.cuda.synchronize()
    evs = {k: [(hev.create(), hev.create()) for _ in range(steps)] for k in kernel_ids}
    t0 = time.perf_counter()
    for s in range(steps):
        for k in kernel_ids:
            dsv.dsv_profile_events(k, *evs[k][s])
        attn_step(d)
    t_enqueued = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for k in kernel_ids:
        dsv.dsv_profile_events(k, None, None)
    # Host time per call (validation, plan choice, launches, binding), the GPU still working on
    # earlier calls: what the host adds to a step only where the GPU would otherwise run dry.
    per_kernel = {"host_enqueue_us": (t_enqueued - t0) / steps * 1e6}
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
    _, probe = time_attention(d, max(min(steps, 5), 2), warmup, ids, hev, min_warm_ms=20.0)
    dominant = max((k for k in ids if probe[k] is not None), key=lambda k: probe[k])
    sec, main = time_attention(d, steps, 2, [dominant], hev)
    per_kernel = dict(probe)
    per_kernel[dominant] = main[dominant]
    per_kernel["host_enqueue_us"] = main["host_enqueue_us"]
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
           "total_q": b.total_q, "num_seqs": b.num_seqs,
           "host_enqueue_us_per_call": per_kernel["host_enqueue_us"]}
    # Which kernels those were: the library says how it cuts the batch under the knobs in force.
    info = dsv.attn_mixed_batch_plan_info(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
    res["plan"] = info
    res["rows_kernel"] = "rows_stream_kernel" if info["row_streams"] else "rows_kernel"
    if per_kernel[dsv.KERNEL_MIXED] is not None:
        res["mixed_launch_ms"] = per_kernel[dsv.KERNEL_MIXED]
        res["mixed_kernel"] = "mixed_stream_kernel" if info["row_streams"] else "mixed_kernel"
        os.environ["DSV_MIXED_LAUNCH"] = "0"
        try:
            size_workspace(d)
            apart = dsv.attn_mixed_batch_plan_info(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
            res["rows_kernel"] = "rows_stream_kernel" if apart["row_streams"] else "rows_kernel"
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


def bench_block_placement(d, res, hev):
    """The row kernel on the same batch and pool with each sequence's blocks at ascending
    addresses instead of the seeded permutation: what the scattered 32 KiB blocks cost."""
    import torch
    import paper_2504_09285_amd as dsv
    b = d.b
    nblk = (b.ctx_lens.astype(np.int64) + 15) // 16
    table = np.zeros_like(b.block_tables)
    first = 0
    for i, n in enumerate(nblk):
        table[i, :n] = np.arange(first, first + n, dtype=np.int32)
        first += int(n)
    permuted = d.block_tables
    d.block_tables = torch.from_numpy(table).cuda()
    try:
        _, per_kernel = timed_step(d, 20, 3, hev, [dsv.KERNEL_ROWS])
    finally:
        d.block_tables = permuted
    nbytes = decode_bytes(b, 2)
    ms = per_kernel[dsv.KERNEL_ROWS]
    return {"seeded_permutation": {"rows_ms": res["kernel_ms"]["rows"], "GB/s": res["decode"]["GB/s"]},
            "ascending_blocks": {"rows_ms": ms, "GB/s": nbytes / (ms * 1e-3) / 1e9}}


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
    ows = torch.empty(dsv.kv_unpack_chunks_ordered_workspace_bytes(dst.NB), dtype=torch.uint8, device="cuda")
    for name, fn in (("pack", lambda: dsv.kv_pack_chunks(src, st, descs, buf)),
                     ("unpack", lambda: dsv.kv_unpack_chunks(buf, descs, dst, dt)),
                     ("unpack_ordered", lambda: dsv.kv_unpack_chunks_ordered(buf, descs, dst, dt, ows))):
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


def bench_tiles_cu_sweep(threads, hev):
    """Config 3's four prefill spans alone (no decodes: the MFMA kernel's own launch, persistent
    workgroups), with the grid held to 256, 128 and 64 workgroups (DSV_TILES_WGS): kernel time and
    TFLOP/s per compute unit in use."""
    import paper_2504_09285_amd as dsv
    from workloads import gen
    full = gen.config3(threads=threads)
    n = 4
    b = gen.AttnBatch("c3_spans_only", full.Hq, full.Hkv, full.D, full.scale, full.q[:full.q_offsets[n]], full.k_pool,
                      full.v_pool, full.block_tables[:n], full.q_offsets[:n + 1], full.ctx_lens[:n])
    d = upload(b)
    flops = prefill_flops(b)
    out = {}
    for wgs in (256, 128, 64):
        os.environ["DSV_TILES_WGS"] = str(wgs)
        try:
            _, pk = time_attention(d, 20, 3, [dsv.KERNEL_TILES], hev, min_warm_ms=30.0)
        finally:
            del os.environ["DSV_TILES_WGS"]
        ms = pk[dsv.KERNEL_TILES]
        out["%d_workgroups" % wgs] = {"ms": ms, "TFLOP/s": flops / (ms * 1e-3) / 1e12,
                                      "TFLOP/s_per_compute_unit": flops / (ms * 1e-3) / 1e12 / wgs}
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
    plan = dsv.attn_mixed_batch_plan_info(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
    os.environ["DSV_MIXED_LAUNCH"] = "0"                               # the two kernels apart, to time each
    try:
        size_workspace(d)
        apart = dsv.attn_mixed_batch_plan_info(b.q_offsets, b.ctx_lens, b.Hq, b.Hkv, b.D)
        sec_apart, pk = time_attention(d, steps, warmup, ids, hev)
    finally:
        del os.environ["DSV_MIXED_LAUNCH"]
    nbytes, flops = decode_bytes(b, 2), prefill_flops(b)
    t_mem, t_mfma = nbytes / (HBM_PEAK_GBS * 1e9), flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    rows_ms, tiles_ms = pk[dsv.KERNEL_ROWS], pk[dsv.KERNEL_TILES]
    return {"workload": b.name, "split_k": sp.k, "ms_per_step": sec * 1e3, "tokens_per_s": b.total_q / sec,
            "plan": plan, "mixed_kernel": "mixed_stream_kernel" if plan["row_streams"] else "mixed_kernel",
            "rows_kernel": "rows_stream_kernel" if apart["row_streams"] else "rows_kernel",
            "mixed_launch_ms": mixed_ms, "ms_per_step_kernels_apart": sec_apart * 1e3,
            "kernel_ms": {"rows": rows_ms, "tiles": tiles_ms, "merge": pk[dsv.KERNEL_MERGE], "plan": pk[dsv.KERNEL_PLAN]},
            "handoff_pack_unpack_ms": handoff_ms, "handoff_chunks": int(len(sp.chunks)),
            "decode": {"GB/s": nbytes / (rows_ms * 1e-3) / 1e9, "frac_hbm_peak": nbytes / (rows_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "prefill": {"TFLOP/s": flops / (tiles_ms * 1e-3) / 1e12, "frac_mfma_peak": flops / (tiles_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
            "bound_ms": {"hbm": t_mem * 1e3, "mfma": t_mfma * 1e3}, "decode_bytes": nbytes, "prefill_flops": flops,
            "frac_of_overlap_bound": max(t_mem, t_mfma) / sec}


def device_handoff(h):
    """Device side of a hand-off whose pools are not generated on the host (gen ... pools=False):
    the pools are filled with seeded N(0,1) on the device."""
    import torch
    import paper_2504_09285_amd as dsv
    g = torch.Generator(device="cuda")
    g.manual_seed(92855)

    def pool(shape):
        t = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
        for l in range(shape[0]):                              # layer by layer: no fp32 copy of the whole pool
            t[l] = torch.randn(shape[1:], generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        return t
    d = argparse.Namespace()
    d.h = h
    d.src = dsv.KVPool(pool(h.src_k), pool(h.src_v))
    d.dst = dsv.KVPool(pool(h.dst_k), pool(h.dst_v))
    d.st, d.dt = torch.from_numpy(h.src_tables).cuda(), torch.from_numpy(h.dst_tables).cuda()
    d.descs = dsv.ChunkDescs(h.chunks)
    d.buf = torch.empty(h.chunk_elems, dtype=torch.bfloat16, device="cuda")
    return d


def bench_concurrent(b, h, rounds, hev):
    """Config 5 as stated: attention on one stream while the hand-off (pack + unpack of every
    layer) runs on a second one.  Each alone, then together: wall time of the whole, and the
    attention step's own latency (events on its stream) alone and under the concurrent hand-off,
    for the full-rate copy and for copies held to a share of the compute units
    (DSV_COPY_MAX_WGS: resident workgroups of the copy kernel)."""
    import torch
    import paper_2504_09285_amd as dsv
    d = upload(b)
    c = device_handoff(h)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    p1, p2 = s1.cuda_stream, s2.cuda_stream

    def attn():
        bb = d.b
        dsv.attn_mixed_batch(d.q, d.out, d.pool, 0, d.block_tables, d.q_offsets, d.ctx_lens, bb.q_offsets,
                             bb.ctx_lens, bb.Hq, bb.scale, d.workspace, stream=s1)

    def copy():
        dsv.kv_pack_chunks(c.src, c.st, c.descs, c.buf, stream=s2)
        dsv.kv_unpack_chunks(c.buf, c.descs, c.dst, c.dt, stream=s2)

    def wall(fns, n):
        for f in fns:
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            for f in fns:
                f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    def attn_latency(with_copy, steps):
        """Mean GPU time of an attention step (events around each call on its stream), with the
        hand-off looping on the other stream or not."""
        torch.cuda.synchronize()
        evs = [(hev.create(), hev.create()) for _ in range(steps)]
        if with_copy:
            copy()                                           # in flight before the first step starts
        for k, (e0, e1) in enumerate(evs):
            hev.record(e0, p1)
            attn()
            hev.record(e1, p1)
            if with_copy and k % 2 == 1:
                copy()                                       # keep the second stream busy throughout
        torch.cuda.synchronize()
        ms = [hev.elapsed_ms(e0, e1) for e0, e1 in evs]
        for e0, e1 in evs:
            hev.destroy(e0)
            hev.destroy(e1)
        return float(np.mean(ms[1:])), float(np.max(ms[1:]))

    ta, tc = wall([attn], rounds), wall([copy], max(rounds // 2, 2))
    # together: one hand-off next to as many attention steps as fit its length
    k = max(1, int(round(tc / ta)))
    tb = wall([copy] + [attn] * k, max(rounds // 2, 2))
    ab, cb = decode_bytes(b, 2), 4 * h.payload_bytes
    out = {"attention": b.name, "handoff": h.name, "handoff_layers": h.L, "handoff_payload_bytes": h.payload_bytes,
           "attn_alone_ms": ta * 1e3, "handoff_alone_ms": tc * 1e3, "attn_steps_per_handoff": k,
           "together_ms": tb * 1e3, "sum_alone_ms": (k * ta + tc) * 1e3,
           "attn_alone_GB/s": ab / ta / 1e9, "handoff_alone_GB/s": cb / tc / 1e9,
           "together_GB/s": (k * ab + cb) / tb / 1e9, "together_frac_hbm_peak": (k * ab + cb) / tb / 1e9 / HBM_PEAK_GBS,
           "overlap_gain": (k * ta + tc) / tb}
    lat = {}
    lat["alone"] = dict(zip(("mean_ms", "max_ms"), attn_latency(False, 12)))
    for share in (0, 128, 64, 32):                            # 0: the copy takes what it can get
        if share:
            os.environ["DSV_COPY_MAX_WGS"] = str(share * 8)  # workgroups of the copy kernel in flight
        try:
            mean, worst = attn_latency(True, 12)
            t_copy = wall([copy], 2)
        finally:
            os.environ.pop("DSV_COPY_MAX_WGS", None)
        lat["copy_unlimited" if not share else "copy_max_%d_workgroups" % (share * 8)] = {
            "attn_mean_ms": mean, "attn_max_ms": worst, "handoff_alone_ms": t_copy * 1e3,
            "handoff_alone_GB/s": cb / t_copy / 1e9}
    out["attn_step_latency"] = lat
    return out


# ---------------------------------------------------------------------------- board power
class BoardSensors:
    """The card's power sensor and shader-clock state as the amdgpu driver shows them in sysfs
    (readable without privileges); every reading is None where the files are absent."""

    def __init__(self):
        import glob
        self.power = (glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") +
                      glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average") + [None])[0]
        self.sclk = (glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk") + [None])[0]
        cap = self.power and os.path.join(os.path.dirname(self.power), "power1_cap")
        self.cap_W = self._read_uW(cap)

    @staticmethod
    def _read_uW(path):
        try:
            return int(open(path).read()) / 1e6
        except (OSError, ValueError, TypeError):
            return None

    def watts(self):
        return self._read_uW(self.power)

    def mhz(self):
        try:
            for ln in open(self.sclk).read().splitlines():
                if "*" in ln:
                    return float(ln.split(":")[1].strip().lower().split("mhz")[0])
        except (OSError, ValueError, TypeError, IndexError):
            pass
        return None


def power_under(fn, sensors, seconds=2.0, batch=20):
    """Loops fn for `seconds` while a thread samples the board sensors every 50 ms; the first third
    of the samples (clock and power still settling) is dropped."""
    import threading
    import torch
    fn()
    torch.cuda.synchronize()
    watts, mhz, stop = [], [], [False]

    def sampler():
        while not stop[0]:
            watts.append(sensors.watts())
            mhz.append(sensors.mhz())
            time.sleep(0.05)
    th = threading.Thread(target=sampler)
    th.start()
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(batch):
            fn()
        torch.cuda.synchronize()
        n += batch
    dt = time.perf_counter() - t0
    stop[0] = True
    th.join()

    def mean(xs):
        xs = [x for x in xs[len(xs) // 3:] if x is not None]
        return float(np.mean(xs)) if xs else None
    w = mean(watts)
    return {"ms_per_call": dt / n * 1e3, "board_W": w, "sclk_MHz": mean(mhz),
            "mJ_per_call": None if w is None else w * dt / n * 1e3}


def bench_power(threads, hev):
    """Board power and shader clock under each kind of work, looped for two seconds each: the
    calibration loops, config 4's decodes alone, its prefill spans alone, and the mixed batch.
    With every loop at the board's power limit, the time of a step is its energy over that limit,
    and two kinds of work that each fill the limit cannot overlap for free."""
    import torch
    import paper_2504_09285_amd as dsv
    from workloads import gen
    sensors = BoardSensors()
    out = {"power_cap_W": sensors.cap_W}
    if sensors.power is None:
        out["note"] = "no power sensor readable on this box"
        return out
    torch.cuda.synchronize()
    time.sleep(1.0)
    out["W_after_1s_idle"] = sensors.watts()
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")
    n = 1 << 30
    src = torch.full((n,), 1, dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(92856)
    operands = torch.randn(1 << 20, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    flops = [0.0]

    def mfma_fixed():
        flops[0] = dsv.dsv_calib_mfma(4000, sink)

    def mfma_data():
        flops[0] = dsv.dsv_calib_mfma_data(4000, operands, sink, shape=1)

    def mfma_data32():
        flops[0] = dsv.dsv_calib_mfma_data(4000, operands, sink, shape=0)
    r = power_under(mfma_fixed, sensors, batch=4)
    r["TFLOP/s"] = flops[0] / (r["ms_per_call"] * 1e-3) / 1e12
    out["mfma_loop_fixed_operands"] = r
    r = power_under(mfma_data, sensors, batch=4)
    r["TFLOP/s"] = flops[0] / (r["ms_per_call"] * 1e-3) / 1e12
    out["mfma_loop_random_operands"] = r
    r = power_under(mfma_data32, sensors, batch=4)
    r["TFLOP/s"] = flops[0] / (r["ms_per_call"] * 1e-3) / 1e12
    out["mfma_loop_32x32x16_random_operands"] = r
    r = power_under(lambda: dsv.dsv_calib_hbm(0, sink, src, n), sensors)
    r["GB/s"] = n / (r["ms_per_call"] * 1e-3) / 1e9
    out["hbm_read_loop"] = r
    del src
    b4, _ = gen.config4(threads=threads)
    segs = list(zip(np.diff(b4.q_offsets).tolist(), b4.ctx_lens.tolist()))
    parts = {"c4_decodes_alone": [sg for sg in segs if sg[0] == 1], "c4_prefill_spans_alone": [sg for sg in segs if sg[0] > 1]}
    d4 = upload(b4)
    out["c4_mixed_batch"] = power_under(lambda: attn_step(d4), sensors)
    del d4
    for name, sub in parts.items():
        dd = upload(gen.make_batch(name, 92857, b4.Hq, b4.Hkv, b4.D, sub, threads=threads))
        out[name] = power_under(lambda: attn_step(dd), sensors)
        del dd
    return out


# ---------------------------------------------------------------------------- ceilings
def measure_ceilings(hev):
    """What this GPU delivers on the plainest loops, through the library's calibration kernels:
    HBM read / write / copy over 2 GiB with kv_copy_kernel's launch shape and hints, a read of
    2 x 2 GiB in the row kernel's access shape with no arithmetic, and a register-resident bf16
    MFMA loop at the prefill kernel's occupancy."""
    import torch
    import paper_2504_09285_amd as dsv
    n = 2 << 30
    src = torch.full((n,), 1, dtype=torch.uint8, device="cuda")
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream or None

    def timed(fn, reps=5):
        fn()
        fn()
        torch.cuda.synchronize()
        e0, e1 = hev.create(), hev.create()
        best = 1e30
        for _ in range(3):
            hev.record(e0, stream)
            for _ in range(reps):
                fn()
            hev.record(e1, stream)
            torch.cuda.synchronize()
            best = min(best, hev.elapsed_ms(e0, e1) / reps)
        hev.destroy(e0)
        hev.destroy(e1)
        return best
    out = {"nominal": {"hbm_GB/s": HBM_PEAK_GBS, "mfma_bf16_TFLOP/s": MFMA_BF16_PEAK_TFLOPS}, "bytes": n}
    for name, mode, moved in (("read", 0, n), ("write", 1, n), ("copy", 2, 2 * n)):
        ms = timed(lambda: dsv.dsv_calib_hbm(mode, dst, src, n))
        out["hbm_%s_GB/s" % name] = moved / (ms * 1e-3) / 1e9
    # the row kernel's access shape (scattered 32 KiB blocks, one head's pieces per wave, through LDS)
    moved = [0.0]

    def paged():
        moved[0] = dsv.dsv_calib_paged_read(src, dst, sink)
    ms = timed(paged)
    out["hbm_read_paged_rows_GB/s"] = moved[0] / (ms * 1e-3) / 1e9
    flops = [0.0]

    def mfma():
        flops[0] = dsv.dsv_calib_mfma(4000, sink)
    ms = timed(mfma, reps=2)
    out["mfma_bf16_TFLOP/s"] = flops[0] / (ms * 1e-3) / 1e12
    # the same loop on N(0,1) operands that change from MFMA to MFMA: what the board's power limit
    # leaves of the matrix cores' rate on data like the attention kernel's
    g = torch.Generator(device="cuda")
    g.manual_seed(92856)
    operands = torch.randn(1 << 20, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)

    # (16x16x32 is the MFMA the head_dim-128 prefill kernels are built on; 32x32x16 for comparison)
    for key, shape in (("mfma_bf16_random_operands_TFLOP/s", 1), ("mfma_bf16_32x32x16_random_operands_TFLOP/s", 0)):
        def mfma_data():
            flops[0] = dsv.dsv_calib_mfma_data(4000, operands, sink, shape=shape)
        for _ in range(20):                   # the clock settles under the load before anything is timed
            mfma_data()
        ms = timed(mfma_data, reps=4)
        out[key] = flops[0] / (ms * 1e-3) / 1e12
    del src, dst
    return out


def against_measured_ceilings(entries, ceilings):
    """Adds to every roofline entry what the same box delivered on the matching calibration loop
    in this run (a kernel that only reads: the sequential read; the copies: the plain copy;
    MFMA-bound: the register-resident MFMA loop) and the kernel's fraction of that; the row
    kernels also against the paged read in their own access shape."""
    for e in entries:
        kernel = e.get("kernel", "")
        if e.get("bound") == "mfma":
            top = ceilings["mfma_bf16_TFLOP/s"]
        elif e.get("bound") == "hbm":
            top = ceilings["hbm_copy_GB/s"] if kernel.startswith(("kv_copy", "kv_append")) else ceilings["hbm_read_GB/s"]
        else:
            continue
        e["measured_ceiling"] = top
        e["frac_of_measured_ceiling"] = e["achieved"] / top
        if e.get("bound") == "mfma" and "mfma_bf16_random_operands_TFLOP/s" in ceilings:
            e["frac_of_mfma_on_random_operands"] = e["achieved"] / ceilings["mfma_bf16_random_operands_TFLOP/s"]
        if kernel.startswith("rows_") and "hbm_read_paged_rows_GB/s" in ceilings:
            e["frac_of_paged_read"] = e["achieved"] / ceilings["hbm_read_paged_rows_GB/s"]


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
            "kind": "oracle", "seconds": elapsed, "workload": b.name,
            "sample": "%d sequences (%.1f passes over the %d of %s; %d query tokens), all heads"
                      % (used, used / n, n, b.name, done_tokens)}


def cpu_baseline_handoff(threads):
    """The oracle's pack + unpack (memcpy per token row) on config 5's hand-off geometry with two
    of the 32 layers: 8 x 8,192 tokens in 256-token chunks, 0.54 GB of payload."""
    import oracle
    from workloads import gen
    oracle.build()
    h = gen.config5_handoff(layers=2, threads=threads)
    buf = np.zeros(h.chunk_elems, np.uint16)
    dk, dv = h.dst_k, h.dst_v
    t0 = time.perf_counter()
    oracle.kv_pack_chunks(h.src_k, h.src_v, h.src_tables, h.chunks, buf)
    oracle.kv_unpack_chunks(buf, h.chunks, dk, dv, h.dst_tables)
    sec = time.perf_counter() - t0
    tok_layers = int(h.chunks[:, 2].sum()) * h.L
    return {"value": 4 * h.payload_bytes / sec / 1e9, "unit": "GB/s (pack + unpack, bytes read + written)",
            "kv_token_layers_per_s": 2 * tok_layers / sec, "cores": oracle.num_threads(), "kind": "oracle",
            "seconds": sec, "workload": h.name,
            "sample": "pack + unpack of 8 x 8192 tokens x 2 of 32 layers (%d bytes of payload)" % h.payload_bytes}


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
    if name == "c3h":
        return gen.config3_heads(40, 8, threads=threads)
    raise SystemExit("unknown workload " + name)


def roofline_entry(kernel, workload, bound, achieved, unit, ms, algorithmic, note=None):
    peak = HBM_PEAK_GBS if bound == "hbm" else MFMA_BF16_PEAK_TFLOPS
    traffic, source = profile_traffic(kernel, workload)
    e = {"kernel": kernel, "workload": workload, "bound": bound, "achieved": achieved, "peak": peak,
         "unit": unit, "frac": achieved / peak, "ms": ms,
         ("algorithmic_bytes" if bound == "hbm" else "algorithmic_flops"): algorithmic,
         "traffic": traffic}
    if source:
        e["traffic_source"] = source
    if note:
        e["note"] = note
    return e


def prefill_kernel_name(head_dim):
    """The kernel that runs prefill spans in a launch of their own: built on the 16x16x32 MFMA for
    head_dim 128, on the 32x32x16 one for head_dim 64."""
    return "prefill_tiles_persistent16_kernel" if head_dim == 128 else "prefill_tiles_persistent_kernel"


def attention_rooflines(res, b):
    out = []
    k = res["kernel_ms"]
    if "decode" in res:
        p = res["decode"]
        out.append(roofline_entry(res.get("rows_kernel", "rows_kernel"), b.name, "hbm", p["GB/s"], "GB/s", k["rows"],
                                  p["algorithmic_bytes"]))
    if "prefill" in res:
        p = res["prefill"]
        out.append(roofline_entry(prefill_kernel_name(b.D), b.name, "mfma", p["TFLOP/s"], "TFLOP/s", k["tiles"],
                                  p["algorithmic_flops"], note="the spans' MFMA kernel in a launch of its own"))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5", choices=["c2", "c3", "c4", "c5", "lp", "c3h"])
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fp8kv-only", action="store_true",
                    help="run only the second workload (8-bit KV cache) and print its results")
    ap.add_argument("--handoff-only", action="store_true",
                    help="run only pack / unpack / ordered unpack on config 5's hand-off geometry (4 of 32 layers)")
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
    from workloads import gen
    if args.handoff_only:
        print(json.dumps({"handoff_c5_4layers": bench_handoff(gen.config5_handoff(layers=4, threads=threads),
                                                              max(args.steps, 1), args.warmup, hev)}))
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
        "kernel_ms": res["kernel_ms"], "host_enqueue_us_per_call": res["host_enqueue_us_per_call"],
    }
    own = attention_rooflines(res, b)
    prefer = "prefill_tiles" if args.workload in ("c3", "c3h", "lp") else "rows_"
    main_rf = next((e for e in own if e["kernel"].startswith(prefer)), own[0] if own else None)
    if main_rf:
        line["roofline"] = {k: main_rf[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel")}
        for k in ("traffic_source", "algorithmic_bytes", "algorithmic_flops"):
            if k in main_rf:
                line["roofline"][k] = main_rf[k]
    rooflines = list(own)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(b, 10.0)
    if args.workload == "c2" and not args.no_extras:
        shared = bench_shared_plan(d, 32, 6, 1)
    placement = None
    if args.workload == "c5" and not args.no_extras:
        placement = bench_block_placement(d, res, hev)
    del d, b

    if not args.no_extras:
        extras = {}
        cpu = []
        if placement:
            extras["c5_rows_kernel_vs_block_placement"] = placement
        line["ceilings"] = measure_ceilings(hev)
        keys = ("ms_per_step", "tokens_per_s", "host_enqueue_us_per_call", "plan", "rows_kernel", "mixed_kernel", "mixed_launch_ms",
                "ms_per_step_kernels_apart", "kernel_ms", "prefill", "decode")

        def other(name, bb, steps, cpu_seconds=0.0, shared_plan=False):
            r, dd = bench_attention(bb, steps, 5, hev)
            extras[name] = {k: r[k] for k in keys if k in r}
            if bb.total_q >= 64:                     # a launch-bound toy batch has no roofline to speak of
                rooflines.extend(attention_rooflines(r, bb))
            if shared_plan:
                extras[name + "_one_plan_per_32_layers"] = bench_shared_plan(dd, 32, 6, 1)
            if cpu_seconds and not args.no_cpu_baseline:
                cpu.append(cpu_baseline(bb, cpu_seconds))
            del dd
        if args.workload != "c2":
            other("c2_decode_heavy", gen.config2(threads=threads), 100, 3.0, shared_plan=True)
        else:
            extras["c2_decode_heavy_one_plan_per_32_layers"] = shared
        if args.workload != "c3":
            other("c3_prefill_heavy", gen.config3(threads=threads), 40, 4.0)
        if args.workload != "c5":
            other("c5_long_context", gen.config5_attention(threads=threads), 20, 3.0)
        # config 3's segments with the head counts of the models the paper serves (Qwen-2.5-14B/32B:
        # 40 query heads on 8 KV heads, five per KV head)
        other("c3_segments_40q_8kv_heads", gen.config3_heads(40, 8, threads=threads), 30)
        other("c1_tiny", gen.config1()[0], 20, 1.0)              # the tiny case: launch-bound
        # A 512-token chunk on a 130,560-token prefix: eight query tiles, cut along the context.
        other("long_prefix_chunk", gen.long_prefix_chunk(threads=threads), 30)
        # Config 4: the mixed batch against its overlap bound, and the two kernels apart.
        c4 = bench_config4(threads, 40, 5, hev)
        extras["c4_micro_request"] = c4
        extras["board_power"] = bench_power(threads, hev)
        rooflines.append({"kernel": c4["mixed_kernel"], "workload": c4["workload"], "bound": "max(hbm, mfma): perfect overlap",
                          "t_hbm_ms": c4["bound_ms"]["hbm"], "t_mfma_ms": c4["bound_ms"]["mfma"], "ms": c4["ms_per_step"],
                          "frac": c4["frac_of_overlap_bound"], "unit": "fraction of the step's overlap bound",
                          "achieved": c4["frac_of_overlap_bound"], "peak": 1.0, "traffic": None})
        rooflines.append(roofline_entry(c4["rows_kernel"], c4["workload"], "hbm", c4["decode"]["GB/s"], "GB/s",
                                        c4["kernel_ms"]["rows"], c4["decode_bytes"], note="launched apart from the tiles"))
        rooflines.append(roofline_entry(prefill_kernel_name(128), c4["workload"], "mfma", c4["prefill"]["TFLOP/s"], "TFLOP/s",
                                        c4["kernel_ms"]["tiles"], c4["prefill_flops"], note="launched apart from the rows"))
        if not args.no_cpu_baseline:
            cpu.append(cpu_baseline(gen.config4(threads=threads)[0], 3.0))
        # Hand-off with config 5's geometry, 4 of the 32 layers (2.15 GB moved per direction).
        h = gen.config5_handoff(layers=4, threads=threads)
        ho = bench_handoff(h, 10, 2, hev)
        extras["handoff_c5_4layers"] = ho
        for name in ("pack", "unpack", "unpack_ordered"):
            rooflines.append(roofline_entry("kv_copy_kernel_" + name, "c5_handoff", "hbm", ho[name]["GB/s"], "GB/s",
                                            ho[name]["ms"], 2 * h.payload_bytes, note="4 of 32 layers"))
        del h
        ap3 = bench_append(gen.config3(threads=threads), 20, 3, hev)
        extras["kv_append_c3"] = ap3
        rooflines.append(roofline_entry("kv_append_kernel", "c3_prefill_heavy", "hbm", ap3["GB/s"], "GB/s", ap3["ms"], ap3["bytes"]))
        f8 = bench_fp8kv(20, 3, hev)
        extras["fp8kv"] = f8
        r8 = f8["c2_decode_heavy_fp8kv"]
        rooflines.append(roofline_entry("rows_stream_kernel_fp8kv", "c2_decode_heavy", "hbm", r8["decode"]["GB/s"], "GB/s",
                                        r8["kernel_ms"]["rows"], r8["decode"]["algorithmic_bytes"]))
        if not args.no_cpu_baseline:
            cpu.append(cpu_baseline_handoff(threads))
        # Config 5 as stated: attention at full context lengths next to the 32-layer hand-off.
        extras["c5_two_streams"] = bench_concurrent(gen.config5_attention(threads=threads),
                                                    gen.config5_handoff(threads=threads, pools=False), 6, hev)
        # The MFMA kernel on fewer compute units (config 3's spans alone): what a compute unit
        # delivers when fewer of them run, i.e. how far the whole chip holds the kernel back.
        extras["prefill_tiles_vs_compute_units"] = bench_tiles_cu_sweep(threads, hev)
        # Chunk-pipelined hand-off (paper section 4.3): transfer of chunk k next to computation of k+1.
        from paper_2504_09285_amd.chunk_pipeline import measure as measure_chunk_pipeline
        extras["chunk_pipelined_handoff"] = measure_chunk_pipeline(8192, 512, 8)
        # The local scheduler's profile table (paper section 4.2): prefill length x decode context x
        # number of decodes -> step ms, and the prefill budget it gives under latency targets.
        from paper_2504_09285_amd.local_scheduler import ProfileTable, sweep
        tbl = sweep(ProfileTable(plen_step=512), plens=(0, 512, 1024, 2048, 4096), ctxs=(1024, 4096), dnums=(32, 128), steps=5)
        extras["profile_table_ms"] = {"plen=%d,ctx=%d,dnum=%d" % k: round(v, 4) for k, v in sorted(tbl.entries().items())}
        extras["max_prefill_allowed"] = {"target_ms=%.2f,ctx=%d,dnum=%d" % (t, c, n): tbl.max_prefill_allowed(t, c, n)
                                         for t in (0.1, 0.2, 0.4) for c, n in ((1024, 32), (4096, 128))}
        against_measured_ceilings(rooflines, line["ceilings"])
        if "roofline" in line:
            against_measured_ceilings([line["roofline"]], line["ceilings"])
        line["rooflines"] = rooflines
        if cpu:
            line["cpu_baselines"] = cpu
        line["extras"] = extras
    else:
        line["rooflines"] = rooflines
    print(json.dumps(line))


if __name__ == "__main__":
    main()
