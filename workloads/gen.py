"""Seeded synthetic inputs for the five workloads.

This module only draws random numbers and lays out index tables.  It holds none
of the attention or hand-off arithmetic and imports neither the CPU oracle nor
the HIP library; both are fed from here so that they see identical bits.

Everything is numpy.  bf16 tensors are ``uint16`` bit patterns produced by
rounding fp32 N(0,1) draws to nearest-even.  Random numbers come from Philox
streams keyed by ``(seed, tensor_id)`` and drawn in fixed-size pieces, so a
tensor's contents depend on nothing but its seed, id and length.

The shapes stand in for the serving traces the paper replays (section 6.1): the
traces only supply length skew, which the lognormal / log-uniform context draws
reproduce; head geometry (8 KV heads, head_dim 128, GQA) is that of the model
families the paper serves.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

SEED_BASE = 92850
BLOCK_SIZE = 16
_PIECE = 1 << 22          # elements per Philox piece (fixed: part of the recipe)

# tensor ids (sub-streams of one workload seed)
TID_Q, TID_K, TID_V, TID_LENS, TID_PERM, TID_SPLIT = 1, 2, 3, 4, 5, 6
TID_SRC_K, TID_SRC_V, TID_DST_K, TID_DST_V, TID_SRC_PERM, TID_DST_PERM = 11, 12, 13, 14, 15, 16


def seed_for(config: int) -> int:
    return SEED_BASE + int(config)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit pattern (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, tensor_id: int, piece: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tensor_id)],
                                                counter=[0, 0, int(piece), 0]))


def normal_bf16(seed: int, tensor_id: int, shape, threads: int = 8) -> np.ndarray:
    """bf16 bits of N(0,1) draws, shape ``shape``."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    pieces = range((n + _PIECE - 1) // _PIECE)

    def fill(p):
        lo = p * _PIECE
        hi = min(n, lo + _PIECE)
        out[lo:hi] = f32_to_bf16_bits(_rng(seed, tensor_id, p).standard_normal(hi - lo, dtype=np.float32))

    if len(pieces) <= 1 or threads <= 1:
        for p in pieces:
            fill(p)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, pieces))
    return out.reshape(shape)


def lognormal_lengths(seed: int, n: int, median: float, sigma: float, lo: int, hi: int) -> np.ndarray:
    z = _rng(seed, TID_LENS).standard_normal(n)
    v = np.rint(np.exp(math.log(median) + sigma * z))
    return np.clip(v, lo, hi).astype(np.int32)


def loguniform_lengths(seed: int, n: int, lo: int, hi: int) -> np.ndarray:
    u = _rng(seed, TID_LENS).random(n)
    v = np.rint(np.exp(math.log(lo) + u * (math.log(hi) - math.log(lo))))
    return np.clip(v, lo, hi).astype(np.int32)


def blocks_for(tokens) -> np.ndarray:
    return (np.asarray(tokens, dtype=np.int64) + BLOCK_SIZE - 1) // BLOCK_SIZE


def build_block_tables(seed: int, tensor_id: int, tokens_per_seq: Sequence[int],
                       free_frac: float = 0.10, min_blocks: int = 0,
                       pad_value: int = 0) -> Tuple[np.ndarray, int]:
    """Assign pool blocks to sequences from one seeded permutation.

    The pool has ceil((1+free_frac) * sum(blocks needed)) blocks (at least
    ``min_blocks``); sequence i takes the next ceil(tokens_i/16) entries of a
    seeded shuffle of all block ids; the remainder stays free.  Table rows are
    padded with ``pad_value`` (never dereferenced by a correct reader).
    """
    need = blocks_for(tokens_per_seq)
    total = int(need.sum())
    nb = max(int(math.ceil((1.0 + free_frac) * total)), int(min_blocks), 1)
    perm = _rng(seed, tensor_id).permutation(nb).astype(np.int32)
    max_blocks = max(int(need.max()) if len(need) else 1, 1)
    tables = np.full((len(need), max_blocks), pad_value, dtype=np.int32)
    pos = 0
    for i, nblk in enumerate(need):
        tables[i, :nblk] = perm[pos:pos + int(nblk)]
        pos += int(nblk)
    return tables, nb


@dataclass
class AttnBatch:
    """One mixed batch over a single-layer paged pool."""
    name: str
    Hq: int
    Hkv: int
    D: int
    scale: float
    q: np.ndarray              # [total_q, Hq, D] u16
    k_pool: np.ndarray         # [NB, 16, Hkv, D] u16
    v_pool: np.ndarray
    block_tables: np.ndarray   # [S, max_blocks] i32
    q_offsets: np.ndarray      # [S+1] i32
    ctx_lens: np.ndarray       # [S] i32
    meta: dict = field(default_factory=dict)

    @property
    def num_seqs(self) -> int:
        return int(self.ctx_lens.shape[0])

    @property
    def total_q(self) -> int:
        return int(self.q_offsets[-1])

    @property
    def q_lens(self) -> np.ndarray:
        return np.diff(self.q_offsets)


def make_batch(name: str, seed: int, Hq: int, Hkv: int, D: int,
               segments: Sequence[Tuple[int, int]], free_frac: float = 0.10,
               min_blocks: int = 0, table_tokens: Optional[Sequence[int]] = None,
               threads: int = 8, meta: Optional[dict] = None) -> AttnBatch:
    """segments: (q_len, ctx_len) per sequence, ctx_len includes the q_len new tokens.

    The whole pool (owned or not) is filled with N(0,1): a serving pool is never
    zeroed, and a sequence's logical K/V is whatever its table points at.
    ``table_tokens`` lets a row own more blocks than ctx_len needs.
    """
    q_lens = np.asarray([s[0] for s in segments], dtype=np.int32)
    ctx_lens = np.asarray([s[1] for s in segments], dtype=np.int32)
    assert (q_lens >= 1).all() and (ctx_lens >= q_lens).all()
    q_offsets = np.zeros(len(segments) + 1, dtype=np.int32)
    np.cumsum(q_lens, out=q_offsets[1:])
    own = ctx_lens if table_tokens is None else np.asarray(table_tokens, dtype=np.int32)
    tables, nb = build_block_tables(seed, TID_PERM, own, free_frac, min_blocks)
    q = normal_bf16(seed, TID_Q, (int(q_offsets[-1]), Hq, D), threads)
    k_pool = normal_bf16(seed, TID_K, (nb, BLOCK_SIZE, Hkv, D), threads)
    v_pool = normal_bf16(seed, TID_V, (nb, BLOCK_SIZE, Hkv, D), threads)
    return AttnBatch(name, Hq, Hkv, D, 1.0 / math.sqrt(D), q, k_pool, v_pool, tables,
                     q_offsets, ctx_lens, dict(meta or {}))


# ---- 8-bit KV variant --------------------------------------------------------------------
# Exponent field of a drawn E4M3 code, indexed by four random bits: mostly around 1.0, a few
# small and subnormal magnitudes, nothing above 7.5, never the NaN code.
_E4M3_EXP_OF_NIBBLE = np.asarray([0, 1, 4, 5, 5, 6, 6, 6, 7, 7, 7, 7, 8, 8, 8, 9], dtype=np.uint8)
TID_K8, TID_V8 = 21, 22


def e4m3_codes(seed: int, tensor_id: int, shape) -> np.ndarray:
    """Random E4M3 codes (uint8): sign and mantissa bits uniform, exponent field drawn from the
    table above.  A pure bit recipe: no rounding or scaling of real values is involved."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint8)
    for p in range((n + _PIECE - 1) // _PIECE):
        lo, hi = p * _PIECE, min(n, (p + 1) * _PIECE)
        u = _rng(seed, tensor_id, p).integers(0, 256, size=hi - lo, dtype=np.uint8)
        out[lo:hi] = (u & np.uint8(0x87)) | (_E4M3_EXP_OF_NIBBLE[(u >> np.uint8(3)) & np.uint8(15)] << np.uint8(3))
    return out.reshape(shape)


def make_batch_fp8kv(name: str, seed: int, Hq: int, Hkv: int, D: int,
                     segments: Sequence[Tuple[int, int]], k_scale: float = 0.5,
                     v_scale: float = 0.5, free_frac: float = 0.10, min_blocks: int = 0,
                     meta: Optional[dict] = None) -> AttnBatch:
    """As make_batch, with the pools holding E4M3 codes (uint8) drawn by e4m3_codes; the two
    dequantisation scales travel in ``meta``.  With the default scales the cached values have a
    root mean square near 1 and magnitudes up to 3.75."""
    q_lens = np.asarray([s[0] for s in segments], dtype=np.int32)
    ctx_lens = np.asarray([s[1] for s in segments], dtype=np.int32)
    assert (q_lens >= 1).all() and (ctx_lens >= q_lens).all()
    q_offsets = np.zeros(len(segments) + 1, dtype=np.int32)
    np.cumsum(q_lens, out=q_offsets[1:])
    tables, nb = build_block_tables(seed, TID_PERM, ctx_lens, free_frac, min_blocks)
    q = normal_bf16(seed, TID_Q, (int(q_offsets[-1]), Hq, D))
    k_pool = e4m3_codes(seed, TID_K8, (nb, BLOCK_SIZE, Hkv, D))
    v_pool = e4m3_codes(seed, TID_V8, (nb, BLOCK_SIZE, Hkv, D))
    m = dict(meta or {})
    m.update(k_scale=float(k_scale), v_scale=float(v_scale))
    return AttnBatch(name, Hq, Hkv, D, 1.0 / math.sqrt(D), q, k_pool, v_pool, tables,
                     q_offsets, ctx_lens, m)


@dataclass
class Handoff:
    """Chunked KV hand-off: source pool/table -> chunks -> destination pool/table."""
    name: str
    L: int
    Hkv: int
    D: int
    src_k: np.ndarray          # [L, NB_src, 16, Hkv, D] u16
    src_v: np.ndarray
    src_tables: np.ndarray     # [R, max_blocks] i32
    dst_k: np.ndarray          # [L, NB_dst, 16, Hkv, D] u16 (pre-filled; untouched slots must survive)
    dst_v: np.ndarray
    dst_tables: np.ndarray
    chunks: np.ndarray         # [C, 4] i64: seq, token_begin, num_tokens, chunk_offset (elements)
    chunk_elems: int           # total elements of the chunk buffer
    elem_bytes: int = 2        # 2: bf16 bits (uint16 arrays); 1: E4M3 codes (uint8 arrays)

    @property
    def payload_bytes(self) -> int:
        return int(self.chunks[:, 2].sum()) * 2 * self.L * self.Hkv * self.D * self.elem_bytes


def make_chunks(ranges: Sequence[Tuple[int, int, int]], chunk_tokens: int, L: int, Hkv: int,
                D: int) -> Tuple[np.ndarray, int]:
    """ranges: (seq, token_begin, token_end).  Equal-sized chunks, the last of a range may be
    short and is stored short.  Chunk c occupies 2*L*num_tokens*Hkv*D elements, back to back."""
    out, off = [], 0
    for seq, tb, te in ranges:
        t = tb
        while t < te:
            n = min(chunk_tokens, te - t)
            out.append((seq, t, n, off))
            off += 2 * L * n * Hkv * D
            t += n
    return np.asarray(out, dtype=np.int64).reshape(-1, 4), off


def make_handoff(name: str, seed: int, L: int, Hkv: int, D: int, req_tokens: Sequence[int],
                 ranges: Sequence[Tuple[int, int, int]], chunk_tokens: int,
                 free_frac: float = 0.10, threads: int = 8, pools: bool = True) -> Handoff:
    """``pools=False``: tables and chunk descriptors only; the four pool fields then hold the pools'
    shapes (tuples) instead of arrays, for a caller that fills the pools on the device."""
    src_tables, nb_s = build_block_tables(seed, TID_SRC_PERM, req_tokens, free_frac)
    dst_tables, nb_d = build_block_tables(seed, TID_DST_PERM, req_tokens, free_frac)
    shp_s = (L, nb_s, BLOCK_SIZE, Hkv, D)
    shp_d = (L, nb_d, BLOCK_SIZE, Hkv, D)
    chunks, n_el = make_chunks(ranges, chunk_tokens, L, Hkv, D)
    if not pools:
        return Handoff(name, L, Hkv, D, shp_s, shp_s, src_tables, shp_d, shp_d, dst_tables, chunks, n_el)
    return Handoff(name, L, Hkv, D,
                   normal_bf16(seed, TID_SRC_K, shp_s, threads), normal_bf16(seed, TID_SRC_V, shp_s, threads),
                   src_tables,
                   normal_bf16(seed, TID_DST_K, shp_d, threads), normal_bf16(seed, TID_DST_V, shp_d, threads),
                   dst_tables, chunks, n_el)


# --------------------------------------------------------------------------------------
# The five workloads.  ``shrink`` divides context lengths / counts for CPU-sized variants;
# shrink=1 is the full size.
# --------------------------------------------------------------------------------------

def config1() -> Tuple[AttnBatch, Handoff]:
    """Tiny mixed batch: 4 q heads, 1 KV head, D=64; prefill 48 on 32 + decodes 70/129/200 in a
    256-block pool; hand-off of tokens [32,96) of the 129-token request as two 32-token chunks."""
    seed = seed_for(1)
    batch = make_batch("c1_tiny", seed, 4, 1, 64, [(48, 80), (1, 70), (1, 129), (1, 200)],
                       min_blocks=256)
    # The hand-off source is the batch's own pool (one layer) and table.
    dst_tables, nb_d = build_block_tables(seed, TID_DST_PERM, batch.ctx_lens, 0.10, 256)
    chunks, n_el = make_chunks([(2, 32, 96)], 32, 1, 1, 64)
    shp_d = (1, nb_d, BLOCK_SIZE, 1, 64)
    h = Handoff("c1_handoff", 1, 1, 64, batch.k_pool[None], batch.v_pool[None], batch.block_tables,
                normal_bf16(seed, TID_DST_K, shp_d), normal_bf16(seed, TID_DST_V, shp_d),
                dst_tables, chunks, n_el)
    return batch, h


def config2(shrink: int = 1, threads: int = 8) -> AttnBatch:
    """Decode-heavy: 256 decodes, ctx ~ LogN(median 1024, sigma 0.8) clipped to [64, 8192]."""
    seed = seed_for(2)
    n = max(256 // shrink, 8)
    ctx = lognormal_lengths(seed, n, 1024.0 / shrink, 0.8, max(64 // shrink, 1), 8192 // shrink)
    return make_batch("c2_decode_heavy", seed, 32, 8, 128, [(1, int(c)) for c in ctx],
                      threads=threads, meta={"shrink": shrink})


def config3(shrink: int = 1, threads: int = 8) -> AttnBatch:
    """Prefill-heavy: 4 prefills of 2048 on prefixes 0/512/1024/4096 + 16 decodes,
    ctx ~ LogN(median 2048, sigma 0.8) clipped to [64, 16384]."""
    seed = seed_for(3)
    ql = 2048 // shrink
    segs = [(ql, ql + p // shrink) for p in (0, 512, 1024, 4096)]
    ctx = lognormal_lengths(seed, 16, 2048.0 / shrink, 0.8, max(64 // shrink, 1), 16384 // shrink)
    segs += [(1, int(c)) for c in ctx]
    return make_batch("c3_prefill_heavy", seed, 32, 8, 128, segs, threads=threads,
                      meta={"shrink": shrink})


def config3_heads(num_q_heads: int, num_kv_heads: int, threads: int = 8) -> AttnBatch:
    """Config 3's segments (same seed) with another head geometry, e.g. 40 query and 8 KV heads:
    Qwen-2.5-14B/32B, the models the paper serves, whose five query heads per KV head do not fill
    groups of four."""
    seed = seed_for(3)
    segs = [(2048, 2048 + p) for p in (0, 512, 1024, 4096)]
    ctx = lognormal_lengths(seed, 16, 2048.0, 0.8, 64, 16384)
    segs += [(1, int(c)) for c in ctx]
    return make_batch("c3_prefill_heavy_%dq_%dkv" % (num_q_heads, num_kv_heads), seed, num_q_heads,
                      num_kv_heads, 128, segs, threads=threads)


@dataclass
class SplitRequest:
    """Config 4's split prompt: request tokens live under table row 0 (segment A's table);
    row 1 is segment B's table on the receiving side."""
    total: int
    k: int
    chunks: np.ndarray         # hand-off of tokens [0,k) from row 0 to row 1, 64-token chunks
    chunk_elems: int


def config4(shrink: int = 1, threads: int = 8) -> Tuple[AttnBatch, SplitRequest]:
    """SLO-aware micro-request batch: a 4096-token prompt split at a seeded uniform boundary k
    into segment A (k tokens on nothing) and segment B (4096-k tokens on a k-token prefix that
    arrives by hand-off into a different table row), plus 128 decodes with
    ctx ~ LogN(median 4096, sigma 0.8) clipped to [32, 32768].  64 q heads, 8 KV heads.

    Both rows 0 and 1 own blocks for all 4096 tokens; the caller is expected to make row 1's
    tokens [k,4096) equal to row 0's and to bring [0,k) over by pack/unpack."""
    seed = seed_for(4)
    total = 4096 // shrink
    k = int(_rng(seed, TID_SPLIT).integers(1, total))          # 1..total-1: both spans non-empty
    nd = max(128 // shrink, 4)
    ctx = lognormal_lengths(seed, nd, 4096.0 / shrink, 0.8, max(32 // shrink, 1), 32768 // shrink)
    segs = [(k, k), (total - k, total)] + [(1, int(c)) for c in ctx]
    own = [total, total] + [int(c) for c in ctx]
    batch = make_batch("c4_micro_request", seed, 64, 8, 128, segs, table_tokens=own,
                       threads=threads, meta={"shrink": shrink, "split_k": k, "prompt": total})
    chunks, n_el = make_chunks([(0, 0, k)], 64, 1, 8, 128)
    return batch, SplitRequest(total, k, chunks, n_el)


def config5_attention(shrink: int = 1, threads: int = 8) -> AttnBatch:
    """Long-context skew: 64 decodes, ctx log-uniform in [16384, 131072]; one layer's pool."""
    seed = seed_for(5)
    n = max(64 // shrink, 4)
    ctx = loguniform_lengths(seed, n, 16384 // shrink, 131072 // shrink)
    return make_batch("c5_long_context", seed, 32, 8, 128, [(1, int(c)) for c in ctx],
                      threads=threads, meta={"shrink": shrink})


def config5_handoff(shrink: int = 1, layers: int = 32, threads: int = 8, pools: bool = True) -> Handoff:
    """8 requests x 8192 tokens x 32 layers, 256-token chunks, into a second pool whose block
    table comes from a different seeded permutation."""
    seed = seed_for(5)
    n_req = max(8 // shrink, 2)
    tok = 8192 // shrink
    return make_handoff("c5_handoff", seed, layers, 8, 128, [tok] * n_req,
                        [(r, 0, tok) for r in range(n_req)], 256, threads=threads, pools=pools)


# ---- the 8-bit KV variant of the same shapes (second workload) -----------------------------------

def config2_fp8kv(shrink: int = 1) -> AttnBatch:
    """Config 2's batch (same seed, same contexts) on a cache of E4M3 codes."""
    seed = seed_for(2)
    n = max(256 // shrink, 8)
    ctx = lognormal_lengths(seed, n, 1024.0 / shrink, 0.8, max(64 // shrink, 1), 8192 // shrink)
    return make_batch_fp8kv("c2_decode_heavy_fp8kv", seed, 32, 8, 128, [(1, int(c)) for c in ctx],
                            meta={"shrink": shrink})


def config3_fp8kv(shrink: int = 1) -> AttnBatch:
    """Config 3's batch (same seed, same segments) on a cache of E4M3 codes."""
    seed = seed_for(3)
    ql = 2048 // shrink
    segs = [(ql, ql + p // shrink) for p in (0, 512, 1024, 4096)]
    ctx = lognormal_lengths(seed, 16, 2048.0 / shrink, 0.8, max(64 // shrink, 1), 16384 // shrink)
    segs += [(1, int(c)) for c in ctx]
    return make_batch_fp8kv("c3_prefill_heavy_fp8kv", seed, 32, 8, 128, segs, meta={"shrink": shrink})


def config5_handoff_fp8kv(shrink: int = 1, layers: int = 32) -> Handoff:
    """Config 5's hand-off (8 requests x 8192 tokens, 256-token chunks) with 1-byte elements:
    half the payload.  Offsets in ``chunks`` count elements, i.e. bytes."""
    seed = seed_for(5)
    n_req = max(8 // shrink, 2)
    tok = 8192 // shrink
    req = [tok] * n_req
    src_tables, nb_s = build_block_tables(seed, TID_SRC_PERM, req, 0.10)
    dst_tables, nb_d = build_block_tables(seed, TID_DST_PERM, req, 0.10)
    shp_s, shp_d = (layers, nb_s, BLOCK_SIZE, 8, 128), (layers, nb_d, BLOCK_SIZE, 8, 128)
    chunks, n_el = make_chunks([(r, 0, tok) for r in range(n_req)], 256, layers, 8, 128)
    return Handoff("c5_handoff_fp8kv", layers, 8, 128, e4m3_codes(seed, 41, shp_s), e4m3_codes(seed, 42, shp_s),
                   src_tables, e4m3_codes(seed, 43, shp_d), e4m3_codes(seed, 44, shp_d), dst_tables,
                   chunks, n_el, elem_bytes=1)


def long_prefix_chunk(q_len: int = 512, prefix: int = 131072 - 512, threads: int = 8) -> AttnBatch:
    """One chunk of a chunked prefill late in a long prompt (or the second span of a micro-request
    split near the end): q_len new tokens on a long cached prefix, nothing else in the batch.
    Few query tiles, each with a very long context."""
    return make_batch("long_prefix_chunk", seed_for(6), 32, 8, 128, [(q_len, prefix + q_len)],
                      threads=threads, meta={"q_len": q_len, "prefix": prefix})
