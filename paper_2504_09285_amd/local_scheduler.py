"""Batch composition of the local scheduler (paper section 4.2, Algorithm 2) around the
attention step of this library: a profile table of measured step latencies keyed by the batch
composition (prefill length ``plen``, decode context length ``ctx``, number of decodes
``dnum``), the prefill budget it implies under a latency target, and the greedy composer that
fills that budget from the prefill queue in arrival order.

Host-side logic; the only GPU work is ``sweep()``, which fills a table by timing
``attn_mixed_batch`` on synthetic batches of each composition (the paper fills it from the
batches it has run: ``record()`` is that same update).

Where the paper is silent (the table's resolution, what to do between or outside recorded
points) this module takes these readings:
  * keys are bucketed: plen up to a multiple of ``plen_step`` tokens, ctx up to a power of two,
    dnum up to a power of two (0 stays 0); a bucket keeps the running mean of its records;
  * a prediction for a composition uses the bucket it falls in; if that bucket is empty, the
    nearest recorded bucket that is at least as large in every coordinate (never an
    optimistic guess); if there is none, the composition is treated as not affordable;
  * MaxPrefillAllowed is the largest recorded plen bucket whose predicted latency is within
    the target, 0 if even plen = 0 is not (decodes are scheduled regardless: Algorithm 2 puts
    every decode into the batch before it asks for the budget).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple


def _pow2_at_least(x: int) -> int:
    return 0 if x <= 0 else 1 << (int(x) - 1).bit_length()


class ProfileTable:
    """Algorithm 2's profile table T."""

    def __init__(self, plen_step: int = 256):
        assert plen_step >= 1
        self.plen_step = int(plen_step)
        self._sum: Dict[Tuple[int, int, int], float] = {}
        self._cnt: Dict[Tuple[int, int, int], int] = {}

    def key(self, plen: int, ctx: int, dnum: int) -> Tuple[int, int, int]:
        p = -(-max(int(plen), 0) // self.plen_step) * self.plen_step
        return p, _pow2_at_least(ctx if dnum > 0 else 0), _pow2_at_least(dnum)

    def record(self, plen: int, ctx: int, dnum: int, time_ms: float) -> None:
        """Algorithm 2, first line: the previous batch's composition and measured latency."""
        k = self.key(plen, ctx, dnum)
        self._sum[k] = self._sum.get(k, 0.0) + float(time_ms)
        self._cnt[k] = self._cnt.get(k, 0) + 1

    def __len__(self) -> int:
        return len(self._cnt)

    def entries(self) -> Dict[Tuple[int, int, int], float]:
        return {k: self._sum[k] / self._cnt[k] for k in self._cnt}

    def predict(self, plen: int, ctx: int, dnum: int) -> Optional[float]:
        """Latency of a batch of this composition, or None if nothing recorded covers it."""
        k = self.key(plen, ctx, dnum)
        if k in self._cnt:
            return self._sum[k] / self._cnt[k]
        best = None
        for (p, c, d) in self._cnt:
            if p >= k[0] and c >= k[1] and d >= k[2]:
                dist = (p - k[0]) / self.plen_step + (c.bit_length() - k[1].bit_length()) + (d.bit_length() - k[2].bit_length())
                if best is None or dist < best[0] or (dist == best[0] and (p, c, d) < best[1]):
                    best = (dist, (p, c, d))
        return None if best is None else self._sum[best[1]] / self._cnt[best[1]]

    def max_prefill_allowed(self, slo_ms: float, ctx: int, dnum: int) -> int:
        """The prefill token budget M of Algorithm 2 for the decodes already in the batch."""
        plens = sorted({p for (p, _, _) in self._cnt})
        allowed = 0
        for p in plens:
            t = self.predict(p, ctx, dnum)
            if t is not None and t <= slo_ms:
                allowed = max(allowed, p)
        return allowed


@dataclass
class PrefillRequest:
    rid: int
    tokens: int            # prompt tokens not yet prefilled


@dataclass
class Batch:
    decodes: List[int] = field(default_factory=list)               # request ids, one token each
    prefills: List[Tuple[int, int]] = field(default_factory=list)  # (request id, tokens scheduled)
    ctx: int = 0           # mean context length of the decodes (0 if none)
    dnum: int = 0
    plen: int = 0          # prefill tokens in the batch
    budget: int = 0        # M as returned by the table


def compose_batch(prefill_queue: Sequence[PrefillRequest], decode_queue: Sequence[Tuple[int, int]],
                  slo_ms: float, table: ProfileTable) -> Batch:
    """Batch composition of section 4.2, Alg. 2.  ``decode_queue`` holds (request id, context
    length).  Every decode joins the batch; the table then gives the prefill token budget for
    those decodes under the latency target, and the prefill queue is cut at that budget in
    arrival order: a request gets whatever of the budget the requests ahead of it have left, at
    most its own remaining tokens.  The caller feeds the previous batch's measured latency to
    ``table.record`` before composing the next one.  The queues are not modified."""
    import numpy as np
    dnum = len(decode_queue)
    ctx = int(round(sum(c for _, c in decode_queue) / dnum)) if dnum else 0
    budget = table.max_prefill_allowed(slo_ms, ctx, dnum)
    want = np.maximum(np.asarray([r.tokens for r in prefill_queue], dtype=np.int64), 0)
    ahead = np.cumsum(want) - want                       # tokens asked for by the requests in front
    grant = np.clip(budget - ahead, 0, want)
    picks = [(prefill_queue[i].rid, int(grant[i])) for i in np.flatnonzero(grant > 0)]
    return Batch(decodes=[rid for rid, _ in decode_queue], prefills=picks, ctx=ctx, dnum=dnum,
                 plen=int(grant.sum()), budget=budget)


def sweep(table: ProfileTable, plens: Sequence[int], ctxs: Sequence[int], dnums: Sequence[int],
          num_q_heads: int = 32, num_kv_heads: int = 8, head_dim: int = 128, steps: int = 5,
          seed: int = 92858) -> ProfileTable:
    """Fills ``table`` by timing ``attn_mixed_batch`` on the GPU for every (plen, ctx, dnum) of the
    grid: one prefill span of plen tokens on an empty prefix plus dnum decodes of context ctx,
    synthetic N(0,1) data.  The latency recorded is the GPU time per call of ``steps`` calls queued
    back to back (events on the stream), median of three repetitions."""
    import numpy as np
    import torch

    from . import binding as dsv

    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    Hq, Hkv, D = num_q_heads, num_kv_heads, head_dim
    for ctx in ctxs:
        for dnum in dnums:
            for plen in plens:
                if plen == 0 and dnum == 0:
                    continue
                segs = ([(plen, plen)] if plen else []) + [(1, ctx)] * dnum
                q_lens = np.array([s[0] for s in segs], np.int32)
                ctx_lens = np.array([s[1] for s in segs], np.int32)
                q_off = np.zeros(len(segs) + 1, np.int32)
                np.cumsum(q_lens, out=q_off[1:])
                nblk = (ctx_lens + 15) // 16
                nb = int(nblk.sum())
                tables = np.zeros((len(segs), int(nblk.max())), np.int32)
                perm = np.random.default_rng(seed).permutation(nb).astype(np.int32)
                o = 0
                for i, n in enumerate(nblk):
                    tables[i, :n] = perm[o:o + n]
                    o += n
                k = torch.randn((1, nb, 16, Hkv, D), generator=g, device="cuda").to(torch.bfloat16)
                v = torch.randn((1, nb, 16, Hkv, D), generator=g, device="cuda").to(torch.bfloat16)
                q = torch.randn((int(q_off[-1]), Hq, D), generator=g, device="cuda").to(torch.bfloat16)
                out = torch.empty_like(q)
                pool = dsv.KVPool(k, v)
                bt = torch.from_numpy(tables).cuda()
                qo, cl = torch.from_numpy(q_off).cuda(), torch.from_numpy(ctx_lens).cuda()
                ws = torch.empty(dsv.attn_mixed_batch_workspace_bytes(q_off, ctx_lens, Hq, Hkv, D),
                                 dtype=torch.uint8, device="cuda")
                call = lambda: dsv.attn_mixed_batch(q, out, pool, 0, bt, qo, cl, q_off, ctx_lens, Hq,
                                                    1.0 / float(np.sqrt(D)), ws)
                call()
                call()
                torch.cuda.synchronize()
                # GPU time of a step, read on the device's own clock: `steps` calls queued back to
                # back between two events.  (Host wall time around a synchronised call sits on a
                # floor of tens of microseconds that hides the differences between small batches.)
                reps = []
                for _ in range(3):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(steps):
                        call()
                    e1.record()
                    torch.cuda.synchronize()
                    reps.append(e0.elapsed_time(e1) / steps)
                table.record(plen, ctx, dnum, float(np.median(reps)))
    return table
