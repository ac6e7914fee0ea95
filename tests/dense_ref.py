"""Brute-force dense attention used only to pin the oracle.

Structurally different from the oracle on purpose: contiguous K/V per sequence, the whole
[q, k] score matrix at once, an explicit boolean mask matrix, masked scores set to -inf, and a
matrix product for PV.  fp64 numpy.  It follows the scaled dot-product definition the paper
refers to in section 2.1 and the span semantics of section 3.1 (a span of q_len tokens
resuming on ctx_len - q_len cached tokens).
"""
import numpy as np


def bf16_to_f64(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def gather_sequence(pool_bits, table_row, ctx_len, bs=16):
    """[ctx_len, Hkv, D] f64: the logical K (or V) of one sequence."""
    t = np.arange(ctx_len)
    return bf16_to_f64(pool_bits[table_row[t // bs], t % bs])


def dense_attention(q_bits, k_seq, v_seq, q_len, scale):
    """q_bits: [q_len, Hq, D] u16; k_seq/v_seq: [ctx, Hkv, D] f64 -> [q_len, Hq, D] f64."""
    q = bf16_to_f64(q_bits)
    ctx, Hkv, D = k_seq.shape
    Hq = q.shape[1]
    G = Hq // Hkv
    prefix = ctx - q_len
    mask = np.arange(ctx)[None, :] <= (prefix + np.arange(q_len))[:, None]      # [q, k]
    out = np.empty_like(q)
    for h in range(Hq):
        g = h // G
        s = scale * (q[:, h, :] @ k_seq[:, g, :].T)                              # [q, k]
        s = np.where(mask, s, -np.inf)
        e = np.exp(s - s.max(axis=1, keepdims=True))
        p = e / e.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v_seq[:, g, :]
    return out


def dense_batch(batch):
    """Dense reference for a whole workloads.AttnBatch."""
    out = np.empty((batch.total_q, batch.Hq, batch.D))
    for i in range(batch.num_seqs):
        a, b = int(batch.q_offsets[i]), int(batch.q_offsets[i + 1])
        ctx = int(batch.ctx_lens[i])
        k = gather_sequence(batch.k_pool, batch.block_tables[i], ctx)
        v = gather_sequence(batch.v_pool, batch.block_tables[i], ctx)
        out[a:b] = dense_attention(batch.q[a:b], k, v, b - a, batch.scale)
    return out
