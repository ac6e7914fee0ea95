/*
 * fp64 CPU oracle, 8-bit KV variant: the same mixed-batch attention and KV append as
 * oracle.c, with the cache stored as 8-bit floating point codes.
 *
 * TEST INFRASTRUCTURE ONLY.  It shares no code, header, table or helper with the GPU
 * library, and nothing on the product path may call it.
 *
 * The paper (sections 2.1, 3.1, 4.3) treats the KV cache as an opaque per-token payload whose
 * size drives both decode bandwidth and hand-off volume; it says nothing about its number
 * format.  This variant halves that payload.  What it fixes, and from where:
 *   - The 8-bit format is the published OCP 8-bit floating point E4M3 encoding: 1 sign bit,
 *     4 exponent bits with bias 7, 3 mantissa bits; exponent field 0 holds subnormals
 *     m/8 * 2^-6; there are no infinities; exponent 15 with mantissa 7 is NaN; the largest
 *     finite magnitude is 448 (code 0x7e).
 *   - One positive fp32 scale per tensor (k_scale, v_scale):  value = scale * decode(code).
 *   - Quantisation of a bf16 input x:  y = fp32(x) / scale, one IEEE fp32 division (the
 *     precision in which the code is decided);  code = the finite E4M3 value nearest to y,
 *     ties to the code with even mantissa bit, magnitudes >= 448 (infinities included) give
 *     +-448, NaN gives 0x7f with the sign bit of y.  The sign of zero is kept.
 *   - Attention is the definition of oracle.c on the dequantised cache:
 *       s_t = softmax_scale * <q, k_scale * decode(K8[t])>
 *       O   = sum_t softmax(s)_t * v_scale * decode(V8[t])
 *
 * The nearest-value search below is a brute force over all 127 non-negative finite codes, in
 * double (both the fp32 quotient and every decoded value are exact in double): no bit tricks.
 *
 * Pins (tests/test_oracle_fp8.py): decoded values the format's definition fixes, round trips
 * of every code, midpoints and their neighbours, saturation; the attention against oracle.c
 * on a cache whose codes are widened exactly to bf16, and the two scale identities.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double e4m3_to_double(uint8_t c)
{
    const int e = (c >> 3) & 15, m = c & 7;
    double mag;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) mag = ldexp((double)m / 8.0, -6);
    else        mag = ldexp(1.0 + (double)m / 8.0, e - 7);
    return (c & 0x80) ? -mag : mag;
}

static float bf16_bits_to_float(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static uint8_t e4m3_nearest(float y)
{
    uint32_t bits;
    memcpy(&bits, &y, sizeof bits);
    const uint8_t sign = (uint8_t)((bits >> 31) << 7);
    if (isnan(y)) return (uint8_t)(sign | 0x7f);
    const double a = fabs((double)y);
    if (a >= 448.0) return (uint8_t)(sign | 0x7e);
    int best = 0;
    double best_d = a;                          /* distance to code 0 (value 0) */
    for (int c = 1; c <= 0x7e; ++c) {
        const double d = fabs(e4m3_to_double((uint8_t)c) - a);
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best = c;
            best_d = d;
        }
    }
    return (uint8_t)(sign | best);
}

/* out[i] = value of code[i] (NaN for 0x7f / 0xff). */
int oracle_e4m3_decode(const uint8_t *codes, int64_t n, double *out)
{
    if (n < 0 || (n && (!codes || !out))) return -1;
    for (int64_t i = 0; i < n; ++i) out[i] = e4m3_to_double(codes[i]);
    return 0;
}

/* codes[i] = quantise(bf16 x[i]) with the rule in the header. */
int oracle_e4m3_quantize(const uint16_t *x, int64_t n, float scale, uint8_t *codes)
{
    if (n < 0 || (n && (!x || !codes)) || !(scale > 0.0f) || isinf(scale)) return -1;
    for (int64_t i = 0; i < n; ++i) {
        const float y = bf16_bits_to_float(x[i]) / scale;
        codes[i] = e4m3_nearest(y);
    }
    return 0;
}

/* codes[i] = nearest E4M3 code of the fp32 value y[i] itself (no scale): the rounding rule alone. */
int oracle_e4m3_from_float(const float *y, int64_t n, uint8_t *codes)
{
    if (n < 0 || (n && (!y || !codes))) return -1;
    for (int64_t i = 0; i < n; ++i) codes[i] = e4m3_nearest(y[i]);
    return 0;
}

typedef struct {
    const uint16_t *q;            /* [total_q][Hq][D] bf16 bits */
    const uint8_t *k_pool;        /* [NB][bs][Hkv][D] codes, the layer attended */
    const uint8_t *v_pool;
    const int32_t *block_tables;  /* [num_seqs][max_blocks] */
    const int32_t *q_offsets;     /* [num_seqs+1] */
    const int32_t *ctx_lens;      /* [num_seqs] */
    int32_t max_blocks, num_seqs, Hq, Hkv, D, bs;
    double scale, k_scale, v_scale;
} attn8_problem;

static int64_t slot_offset(const attn8_problem *a, int i, int t, int g)
{
    const int64_t b = a->block_tables[(int64_t)i * a->max_blocks + t / a->bs];
    return ((b * a->bs + t % a->bs) * a->Hkv + g) * (int64_t)a->D;
}

/* One output row (segment i, new token j, query head h); scores: >= ctx_len_i doubles. */
static void attn8_one_row(const attn8_problem *a, int i, int j, int h, double *scores,
                          double *out_row)
{
    const int q_len = a->q_offsets[i + 1] - a->q_offsets[i];
    const int p = a->ctx_lens[i] - q_len + j;
    const int g = h / (a->Hq / a->Hkv);
    const uint16_t *qrow = a->q + ((int64_t)(a->q_offsets[i] + j) * a->Hq + h) * a->D;

    double m = -INFINITY;
    for (int t = 0; t <= p; ++t) {
        const uint8_t *krow = a->k_pool + slot_offset(a, i, t, g);
        double dot = 0.0;
        for (int d = 0; d < a->D; ++d)
            dot += (double)bf16_bits_to_float(qrow[d]) * (a->k_scale * e4m3_to_double(krow[d]));
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
        const uint8_t *vrow = a->v_pool + slot_offset(a, i, t, g);
        for (int d = 0; d < a->D; ++d)
            out_row[d] += w * (a->v_scale * e4m3_to_double(vrow[d]));
    }
}

static int check8(const attn8_problem *a)
{
    if (!a->q || !a->k_pool || !a->v_pool || !a->block_tables || !a->q_offsets || !a->ctx_lens)
        return -1;
    if (a->num_seqs < 0 || a->Hq < 1 || a->Hkv < 1 || a->Hq % a->Hkv || a->D < 1 || a->bs < 1)
        return -1;
    if (!(a->k_scale > 0.0) || !(a->v_scale > 0.0)) return -1;
    for (int i = 0; i < a->num_seqs; ++i) {
        const int q_len = a->q_offsets[i + 1] - a->q_offsets[i];
        if (q_len < 1 || a->ctx_lens[i] < q_len) return -1;
        if ((a->ctx_lens[i] + a->bs - 1) / a->bs > a->max_blocks) return -1;
    }
    return 0;
}

/*
 * Selected rows.  rows: [n_rows][3] = (segment, new-token index j, query head h).
 * out: [n_rows][D] doubles.
 */
int oracle_attn_rows_fp8kv(const uint16_t *q, const uint8_t *k_pool, const uint8_t *v_pool,
                           const int32_t *block_tables, int32_t max_blocks,
                           const int32_t *q_offsets, const int32_t *ctx_lens, int32_t num_seqs,
                           int32_t Hq, int32_t Hkv, int32_t D, int32_t bs, double scale,
                           double k_scale, double v_scale, int32_t n_rows, const int32_t *rows,
                           double *out)
{
    attn8_problem a = {q, k_pool, v_pool, block_tables, q_offsets, ctx_lens, max_blocks,
                       num_seqs, Hq, Hkv, D, bs, scale, k_scale, v_scale};
    int rc = check8(&a);
    if (rc) return rc;
    if (n_rows < 0 || (n_rows && (!rows || !out))) return -1;
    int max_ctx = 1;
    for (int i = 0; i < num_seqs; ++i)
        if (ctx_lens[i] > max_ctx) max_ctx = ctx_lens[i];
    for (int r = 0; r < n_rows; ++r) {
        const int i = rows[3 * r], j = rows[3 * r + 1], h = rows[3 * r + 2];
        if (i < 0 || i >= num_seqs || h < 0 || h >= Hq) return -1;
        if (j < 0 || j >= q_offsets[i + 1] - q_offsets[i]) return -1;
    }
#pragma omp parallel
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)max_ctx);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_rows; ++r)
            attn8_one_row(&a, rows[3 * r], rows[3 * r + 1], rows[3 * r + 2], scores,
                          out + (int64_t)r * D);
        free(scores);
    }
    return 0;
}

/*
 * KV append with quantisation: the new tokens' keys/values (bf16, [total_q][Hkv][D]) are
 * quantised with the rule in the header and written to the positions the new tokens occupy
 * (segment i, new token j -> position ctx_len_i - q_len_i + j of row i of the block table).
 * Every other byte of the pool keeps its value.
 */
int oracle_kv_append_fp8(const uint16_t *k_new, const uint16_t *v_new, uint8_t *k_pool,
                         uint8_t *v_pool, int32_t bs, int32_t Hkv, int32_t D,
                         const int32_t *block_tables, int32_t max_blocks, int32_t num_seqs,
                         const int32_t *q_offsets, const int32_t *ctx_lens, float k_scale,
                         float v_scale)
{
    if (!k_new || !v_new || !k_pool || !v_pool || !block_tables || !q_offsets || !ctx_lens)
        return -1;
    if (bs < 1 || Hkv < 1 || D < 1 || num_seqs < 1 || q_offsets[0] != 0) return -1;
    if (!(k_scale > 0.0f) || !(v_scale > 0.0f) || isinf(k_scale) || isinf(v_scale)) return -1;
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
            for (int64_t e = 0; e < row; ++e) {
                k_pool[dst + e] = e4m3_nearest(bf16_bits_to_float(k_new[src + e]) / k_scale);
                v_pool[dst + e] = e4m3_nearest(bf16_bits_to_float(v_new[src + e]) / v_scale);
            }
        }
    }
    return 0;
}
