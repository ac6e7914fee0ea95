/*
 * fp64 CPU oracle for mixed-batch paged-KV attention and chunked KV hand-off.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP kernels are checked against.  It shares no code, header, table or helper
 * with the GPU library, and nothing on the product path may call it.
 *
 * What it computes, and where the paper fixes it:
 *   - Autoregressive attention with a KV cache (paper section 2.1, "LLM
 *     Inference"): a query token at absolute position p attends to the cached
 *     keys/values of tokens 0..p of its own request.  A decode step is one
 *     query token over the whole context; a prefill span is many query tokens,
 *     each with its own causal horizon.
 *   - Micro-requests (paper section 3.1): a request may be cut at any token
 *     boundary; the second span resumes on the first span's tokens as cached
 *     prefix.  Hence a segment is (q_len new tokens, ctx_len total tokens) and
 *     the j-th new token sits at position ctx_len - q_len + j.
 *   - One step executes a token-level batch mixing prefill spans and decode
 *     tokens (paper sections 3.1 "Unified execution instances", 4.2, Alg. 2).
 *   - KV lives in fixed-size blocks (paper sections 3.1, 4.3); which block a
 *     token occupies is given by a per-request block table.
 *   - Chunk-based KV transfer (paper section 4.3): the KV of a token range is
 *     shipped as equal-sized contiguous chunks, and the receiver places it
 *     into blocks of its own choosing.  pack = paged -> contiguous chunk,
 *     unpack = contiguous chunk -> paged (only the covered slots are written).
 *   - KV append (paper section 2.1): before a step's attention reads the cache,
 *     the keys/values of the step's new tokens are written into it.
 *
 * The paper gives no formula beyond citing the standard scaled dot-product
 * attention; the definition written out here is
 *     s_t = scale * <q, K[t]>,  t = 0..p
 *     w_t = exp(s_t - max_t s_t),  Z = sum_t w_t
 *     O   = sum_t (w_t / Z) * V[t]
 * with query head h reading KV head floor(h / (Hq/Hkv)).
 *
 * Inputs are bf16 bit patterns (uint16), widened exactly to double; all
 * arithmetic is double; exp is libm's.  No blocking, fusion or reordering:
 * three plain passes over t per output row.
 *
 * Pool layout (one layer): [num_blocks][block_size][num_kv_heads][head_dim].
 * Chunk layout: [layer][K=0|V=1][num_tokens][num_kv_heads][head_dim], tight.
 *
 * Every function here is pinned by tests that do not use this file's own
 * arithmetic (dense brute force, a library attention routine, closed forms,
 * hand-derived values, invariances); none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

typedef struct {
    const uint16_t *q;            /* [total_q][Hq][D] */
    const uint16_t *k_pool;       /* [NB][bs][Hkv][D], the layer attended */
    const uint16_t *v_pool;
    const int32_t *block_tables;  /* [num_seqs][max_blocks] */
    const int32_t *q_offsets;     /* [num_seqs+1] */
    const int32_t *ctx_lens;      /* [num_seqs] */
    int32_t max_blocks, num_seqs, Hq, Hkv, D, bs;
    double scale;
} attn_problem;

/* element offset of (token t of sequence i, kv head g, dim 0) in a pool */
static int64_t kv_slot_offset(const attn_problem *a, int i, int t, int g)
{
    int64_t b = a->block_tables[(int64_t)i * a->max_blocks + t / a->bs];
    int64_t s = t % a->bs;
    return ((b * a->bs + s) * a->Hkv + g) * (int64_t)a->D;
}

/*
 * One output row: segment i, new token j, query head h.
 * scores: scratch of at least ctx_len_i doubles.
 * If weights_out != NULL it receives the normalised softmax weights (p+1 of them).
 */
static void attn_one_row(const attn_problem *a, int i, int j, int h,
                         double *scores, double *out_row, double *weights_out)
{
    const int q_len = a->q_offsets[i + 1] - a->q_offsets[i];
    const int p = a->ctx_lens[i] - q_len + j;       /* absolute position of the query token */
    const int g = h / (a->Hq / a->Hkv);             /* KV head shared by consecutive query heads */
    const uint16_t *qrow = a->q + ((int64_t)(a->q_offsets[i] + j) * a->Hq + h) * a->D;

    double m = -INFINITY;
    for (int t = 0; t <= p; ++t) {
        const uint16_t *krow = a->k_pool + kv_slot_offset(a, i, t, g);
        double dot = 0.0;
        for (int d = 0; d < a->D; ++d)
            dot += bf16_bits_to_double(qrow[d]) * bf16_bits_to_double(krow[d]);
        scores[t] = a->scale * dot;
        if (scores[t] > m) m = scores[t];
    }
    double Z = 0.0;
    for (int t = 0; t <= p; ++t) {
        scores[t] = exp(scores[t] - m);
        Z += scores[t];
    }
    for (int d = 0; d < a->D; ++d) out_row[d] = 0.0;
    for (int t = 0; t <= p; ++t) {
        const double w = scores[t] / Z;
        if (weights_out) weights_out[t] = w;
        const uint16_t *vrow = a->v_pool + kv_slot_offset(a, i, t, g);
        for (int d = 0; d < a->D; ++d)
            out_row[d] += w * bf16_bits_to_double(vrow[d]);
    }
}

static int check_problem(const attn_problem *a)
{
    if (!a->q || !a->k_pool || !a->v_pool || !a->block_tables || !a->q_offsets || !a->ctx_lens)
        return -1;
    if (a->num_seqs < 0 || a->Hq < 1 || a->Hkv < 1 || a->Hq % a->Hkv || a->D < 1 || a->bs < 1)
        return -1;
    for (int i = 0; i < a->num_seqs; ++i) {
        int q_len = a->q_offsets[i + 1] - a->q_offsets[i];
        if (q_len < 1 || a->ctx_lens[i] < q_len) return -1;
        if ((a->ctx_lens[i] + a->bs - 1) / a->bs > a->max_blocks) return -1;
    }
    return 0;
}

/* All rows of the batch.  out: [total_q][Hq][D] doubles. */
int oracle_attn_mixed_batch(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                            const int32_t *block_tables, int32_t max_blocks,
                            const int32_t *q_offsets, const int32_t *ctx_lens,
                            int32_t num_seqs, int32_t Hq, int32_t Hkv, int32_t D, int32_t bs,
                            double scale, double *out)
{
    attn_problem a = {q, k_pool, v_pool, block_tables, q_offsets, ctx_lens,
                      max_blocks, num_seqs, Hq, Hkv, D, bs, scale};
    int rc = check_problem(&a);
    if (rc) return rc;
    if (!out) return -1;
    const int64_t total_q = q_offsets[num_seqs];
    int32_t *seg_of_token = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total_q > 0 ? total_q : 1));
    int max_ctx = 1;
    for (int i = 0; i < num_seqs; ++i) {
        for (int tq = q_offsets[i]; tq < q_offsets[i + 1]; ++tq) seg_of_token[tq] = i;
        if (ctx_lens[i] > max_ctx) max_ctx = ctx_lens[i];
    }
#pragma omp parallel
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)max_ctx);
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < total_q * Hq; ++r) {
            const int tq = (int)(r / Hq), h = (int)(r % Hq);
            const int i = seg_of_token[tq];
            attn_one_row(&a, i, tq - q_offsets[i], h, scores, out + r * D, NULL);
        }
        free(scores);
    }
    free(seg_of_token);
    return 0;
}

/*
 * Selected rows only (for spot checks at sizes where the whole batch would take
 * too long).  rows: [n_rows][3] = (segment, new-token index j, query head h).
 * out: [n_rows][D] doubles.
 */
int oracle_attn_rows(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                     const int32_t *block_tables, int32_t max_blocks,
                     const int32_t *q_offsets, const int32_t *ctx_lens,
                     int32_t num_seqs, int32_t Hq, int32_t Hkv, int32_t D, int32_t bs,
                     double scale, int32_t n_rows, const int32_t *rows, double *out)
{
    attn_problem a = {q, k_pool, v_pool, block_tables, q_offsets, ctx_lens,
                      max_blocks, num_seqs, Hq, Hkv, D, bs, scale};
    int rc = check_problem(&a);
    if (rc) return rc;
    if (n_rows < 0 || (n_rows && (!rows || !out))) return -1;
    for (int r = 0; r < n_rows; ++r) {
        int i = rows[3 * r], j = rows[3 * r + 1], h = rows[3 * r + 2];
        if (i < 0 || i >= num_seqs || h < 0 || h >= Hq) return -1;
        if (j < 0 || j >= q_offsets[i + 1] - q_offsets[i]) return -1;
    }
#pragma omp parallel
    {
        int max_ctx = 1;
        for (int i = 0; i < num_seqs; ++i)
            if (ctx_lens[i] > max_ctx) max_ctx = ctx_lens[i];
        double *scores = (double *)malloc(sizeof(double) * (size_t)max_ctx);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_rows; ++r)
            attn_one_row(&a, rows[3 * r], rows[3 * r + 1], rows[3 * r + 2], scores,
                         out + (int64_t)r * D, NULL);
        free(scores);
    }
    return 0;
}

/*
 * Softmax weights of one row (segment i, new token j, head h): weights[0..p],
 * p = ctx_len - q_len + j.  Returns p+1, or a negative code.
 */
int oracle_attn_row_weights(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                            const int32_t *block_tables, int32_t max_blocks,
                            const int32_t *q_offsets, const int32_t *ctx_lens,
                            int32_t num_seqs, int32_t Hq, int32_t Hkv, int32_t D, int32_t bs,
                            double scale, int32_t i, int32_t j, int32_t h,
                            double *weights, double *out_row)
{
    attn_problem a = {q, k_pool, v_pool, block_tables, q_offsets, ctx_lens,
                      max_blocks, num_seqs, Hq, Hkv, D, bs, scale};
    int rc = check_problem(&a);
    if (rc) return rc;
    if (i < 0 || i >= num_seqs || h < 0 || h >= Hq || !weights || !out_row) return -1;
    const int q_len = q_offsets[i + 1] - q_offsets[i];
    if (j < 0 || j >= q_len) return -1;
    double *scores = (double *)malloc(sizeof(double) * (size_t)ctx_lens[i]);
    attn_one_row(&a, i, j, h, scores, out_row, weights);
    free(scores);
    return ctx_lens[i] - q_len + j + 1;
}

/* ---- chunked KV hand-off -------------------------------------------------- */

static int check_chunks(int32_t num_chunks, const int32_t *seq, const int32_t *token_begin,
                        const int32_t *num_tokens, const int64_t *chunk_offset,
                        int32_t num_seqs, int32_t max_blocks, int32_t bs)
{
    if (num_chunks < 0) return -1;
    if (num_chunks && (!seq || !token_begin || !num_tokens || !chunk_offset)) return -1;
    for (int c = 0; c < num_chunks; ++c) {
        if (seq[c] < 0 || seq[c] >= num_seqs) return -1;
        if (token_begin[c] < 0 || num_tokens[c] < 1 || chunk_offset[c] < 0) return -1;
        if (((int64_t)token_begin[c] + num_tokens[c] + bs - 1) / bs > max_blocks) return -1;
    }
    return 0;
}

/*
 * pack: for chunk c, layer l, kv in {K,V}, u in [0,num_tokens):
 *   chunk_buf[chunk_offset_c + ((l*2+kv)*num_tokens + u)*Hkv*D + ...]
 *     = pool_kv[l*layer_stride + (table[seq][(tb+u)/bs]*bs + (tb+u)%bs)*Hkv*D + ...]
 * dir = 0: pool -> chunk (pack); dir = 1: chunk -> pool (unpack).
 */
static int copy_chunks(int dir, uint16_t *k_pool, uint16_t *v_pool, int64_t layer_stride,
                       int32_t num_layers, int32_t bs, int32_t Hkv, int32_t D,
                       const int32_t *block_tables, int32_t max_blocks, int32_t num_seqs,
                       int32_t num_chunks, const int32_t *seq, const int32_t *token_begin,
                       const int32_t *num_tokens, const int64_t *chunk_offset,
                       uint16_t *chunk_buf)
{
    if (!k_pool || !v_pool || !block_tables || (num_chunks && !chunk_buf)) return -1;
    if (num_layers < 1 || bs < 1 || Hkv < 1 || D < 1) return -1;
    int rc = check_chunks(num_chunks, seq, token_begin, num_tokens, chunk_offset,
                          num_seqs, max_blocks, bs);
    if (rc) return rc;
    const int64_t row = (int64_t)Hkv * D;   /* elements per token per K or V */
    for (int c = 0; c < num_chunks; ++c) {
        for (int l = 0; l < num_layers; ++l) {
            for (int kv = 0; kv < 2; ++kv) {
                uint16_t *pool = (kv == 0 ? k_pool : v_pool) + (int64_t)l * layer_stride;
                for (int u = 0; u < num_tokens[c]; ++u) {
                    const int t = token_begin[c] + u;
                    const int64_t b = block_tables[(int64_t)seq[c] * max_blocks + t / bs];
                    uint16_t *slot = pool + (b * bs + t % bs) * row;
                    uint16_t *dst = chunk_buf + chunk_offset[c] +
                                    (((int64_t)l * 2 + kv) * num_tokens[c] + u) * row;
                    if (dir == 0) memcpy(dst, slot, sizeof(uint16_t) * (size_t)row);
                    else          memcpy(slot, dst, sizeof(uint16_t) * (size_t)row);
                }
            }
        }
    }
    return 0;
}

int oracle_kv_pack_chunks(const uint16_t *k_pool, const uint16_t *v_pool, int64_t layer_stride,
                          int32_t num_layers, int32_t bs, int32_t Hkv, int32_t D,
                          const int32_t *block_tables, int32_t max_blocks, int32_t num_seqs,
                          int32_t num_chunks, const int32_t *seq, const int32_t *token_begin,
                          const int32_t *num_tokens, const int64_t *chunk_offset,
                          uint16_t *chunk_buf)
{
    return copy_chunks(0, (uint16_t *)k_pool, (uint16_t *)v_pool, layer_stride, num_layers, bs,
                       Hkv, D, block_tables, max_blocks, num_seqs, num_chunks, seq, token_begin,
                       num_tokens, chunk_offset, chunk_buf);
}

int oracle_kv_unpack_chunks(const uint16_t *chunk_buf, int32_t num_chunks, const int32_t *seq,
                            const int32_t *token_begin, const int32_t *num_tokens,
                            const int64_t *chunk_offset, uint16_t *k_pool, uint16_t *v_pool,
                            int64_t layer_stride, int32_t num_layers, int32_t bs, int32_t Hkv,
                            int32_t D, const int32_t *block_tables, int32_t max_blocks,
                            int32_t num_seqs)
{
    return copy_chunks(1, k_pool, v_pool, layer_stride, num_layers, bs, Hkv, D, block_tables,
                       max_blocks, num_seqs, num_chunks, seq, token_begin, num_tokens,
                       chunk_offset, (uint16_t *)chunk_buf);
}

/* ---- KV append --------------------------------------------------------------- */

/*
 * The step right before attention reads the cache (paper section 2.1: prefill populates the
 * KV cache, each decode step appends to it): the keys/values of the batch's new tokens,
 * k_new/v_new [total_q][Hkv][D], are written into one layer of the pool at the positions the
 * new tokens occupy, through the block table.  For segment i and its j-th new token:
 *   p = ctx_len_i - q_len_i + j
 *   pool_kv[(table[i][p/bs]*bs + p%bs)*Hkv*D + ...] = kv_new[(q_off_i + j)*Hkv*D + ...]
 * Every other element of the pool keeps its value.
 */
int oracle_kv_append(const uint16_t *k_new, const uint16_t *v_new, uint16_t *k_pool,
                     uint16_t *v_pool, int32_t bs, int32_t Hkv, int32_t D,
                     const int32_t *block_tables, int32_t max_blocks, int32_t num_seqs,
                     const int32_t *q_offsets, const int32_t *ctx_lens)
{
    if (!k_new || !v_new || !k_pool || !v_pool || !block_tables || !q_offsets || !ctx_lens)
        return -1;
    if (bs < 1 || Hkv < 1 || D < 1 || num_seqs < 1 || q_offsets[0] != 0) return -1;
    for (int i = 0; i < num_seqs; ++i) {
        const int64_t q_len = (int64_t)q_offsets[i + 1] - q_offsets[i];
        if (q_len < 1 || ctx_lens[i] < q_len) return -1;
        if (((int64_t)ctx_lens[i] + bs - 1) / bs > max_blocks) return -1;
    }
    const int64_t row = (int64_t)Hkv * D;
    for (int i = 0; i < num_seqs; ++i) {
        const int32_t q_len = q_offsets[i + 1] - q_offsets[i];
        for (int32_t j = 0; j < q_len; ++j) {
            const int64_t p = (int64_t)ctx_lens[i] - q_len + j;
            const int64_t b = block_tables[(int64_t)i * max_blocks + p / bs];
            const int64_t dst = (b * bs + p % bs) * row;
            const int64_t src = ((int64_t)q_offsets[i] + j) * row;
            memcpy(k_pool + dst, k_new + src, sizeof(uint16_t) * (size_t)row);
            memcpy(v_pool + dst, v_new + src, sizeof(uint16_t) * (size_t)row);
        }
    }
    return 0;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
