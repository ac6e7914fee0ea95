// kv_append: the step right before attention reads the cache (paper section 2.1: prefill
// populates the KV cache, each decode step appends to it).  The keys/values of the batch's new
// tokens, [total_q][Hkv][D] bf16, are written into one layer of the paged pool at the positions
// the new tokens occupy, [ctx_len - q_len, ctx_len) of each segment, through the block table.
// Pure byte movement, bit-exact.
//
// Work decomposition: one workgroup per (run of consecutive new tokens worth about 16 KiB, K|V).
// The first lanes find each token's segment by binary search in q_offsets and its row in the
// pool through the block table, leave the row's base in LDS, and all threads then move 16-byte
// units, four loads in flight per lane.  Source rows are read once (nontemporal); the stores go
// through the cache as usual because the attention kernels read these rows next.
//
// kv_append_fp8 is the same step for a cache of 8-bit codes: each workgroup reads bf16 rows and
// stores their E4M3 codes.  The code of x is decided in fp32: y = x / scale (one IEEE division),
// rounded to the nearest E4M3 value with ties to the even mantissa, magnitudes of 448 and above
// saturating to +-448.  The rounding is done on the bits of y (below), not by a conversion
// instruction, so that every case (ties, subnormals, saturation, zero signs) is spelled out.
#include <math.h>

#include "dsv_common.h"

namespace dsv {
namespace {

constexpr int kAppendThreads = 256;
constexpr int kAppendUnits = kAppendThreads * 4;     // 16-byte units per workgroup
constexpr int kMaxTileTokens = 64;

typedef uint32_t unit_t __attribute__((ext_vector_type(4)));

struct AppendParams {
  const unit_t* k_new;
  const unit_t* v_new;
  unit_t* pool_k;                // layer base already applied
  unit_t* pool_v;
  const int32_t* block_tables;
  const int32_t* q_offsets;
  const int32_t* ctx_lens;
  int32_t max_blocks;
  int32_t num_seqs;
  int32_t total_q;
  int32_t upr;                   // 16-byte units per token row (Hkv * D / 8)
  int32_t tile_tokens;           // tokens per workgroup
};

__global__ __launch_bounds__(kAppendThreads) void kv_append_kernel(AppendParams p) {
  __shared__ int64_t row_base[kMaxTileTokens];     // pool row of each token of the tile, in units
  const int g0 = (int)blockIdx.x * p.tile_tokens;
  const int ntok = min(p.tile_tokens, p.total_q - g0);
  if ((int)threadIdx.x < ntok) {
    const int g = g0 + (int)threadIdx.x;
    // Segment of new token g: the last i with q_offsets[i] <= g.
    int lo = 0, hi = p.num_seqs;                   // answer in [lo, hi)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.q_offsets[mid] <= g) lo = mid; else hi = mid;
    }
    const int q0 = p.q_offsets[lo];
    const int q_len = p.q_offsets[lo + 1] - q0;
    const int pos = p.ctx_lens[lo] - q_len + (g - q0);
    const int64_t blk = p.block_tables[(int64_t)lo * p.max_blocks + pos / kBlockSize];
    row_base[threadIdx.x] = (blk * kBlockSize + pos % kBlockSize) * (int64_t)p.upr;
  }
  __syncthreads();
  const unit_t* src = (blockIdx.y ? p.v_new : p.k_new) + (int64_t)g0 * p.upr;
  unit_t* pool = blockIdx.y ? p.pool_v : p.pool_k;
  const int total = ntok * p.upr;
  for (int u0 = (int)threadIdx.x; u0 < total; u0 += kAppendUnits) {
    unit_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int u = u0 + k * kAppendThreads;
      if (u < total) v[k] = __builtin_nontemporal_load(src + u);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int u = u0 + k * kAppendThreads;
      if (u < total) {
        const int t = u / p.upr;
        pool[row_base[t] + (u - t * p.upr)] = v[k];
      }
    }
  }
}


// fp32 -> E4M3 code (OCP 8-bit float: bias 7, 3 mantissa bits, subnormals m/8 * 2^-6, no
// infinities, 0x7f = NaN, largest finite 448 = 0x7e).  Round to nearest, ties to even; |y| >= 448
// and infinities give +-448; NaN gives 0x7f; the sign of zero is kept.
__device__ __forceinline__ uint32_t e4m3_code(float y) {
  const uint32_t u = __builtin_bit_cast(uint32_t, y);
  const uint32_t sign = (u >> 24) & 0x80u;
  const uint32_t a = u & 0x7fffffffu;
  uint32_t code;
  if (a > 0x7f800000u) {
    code = 0x7fu;
  } else if (a >= 0x43e00000u) {                 // 448.0f
    code = 0x7eu;
  } else if (a >= 0x3c800000u) {                 // 2^-6: keep three mantissa bits of the fp32
    code = ((a + 0x7ffffu + ((a >> 20) & 1u)) >> 20) - (120u << 3);   // rebias 127 -> 7
  } else {                                       // below 2^-6: multiples of 2^-9 (8 -> 2^-6 itself)
    code = (uint32_t)__builtin_rintf(__builtin_bit_cast(float, a) * 512.0f);
  }
  return sign | code;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// Four codes from two registers of bf16 pairs.
__device__ __forceinline__ uint32_t quantise4(uint32_t w0, uint32_t w1, float scale) {
  return e4m3_code(bf16_lo(w0) / scale) | (e4m3_code(bf16_hi(w0) / scale) << 8) |
         (e4m3_code(bf16_lo(w1) / scale) << 16) | (e4m3_code(bf16_hi(w1) / scale) << 24);
}

struct Append8Params {
  AppendParams p;                // upr: 16-byte units of codes per token row (Hkv * D / 16)
  float k_scale, v_scale;
};

__global__ __launch_bounds__(kAppendThreads) void kv_append_fp8_kernel(Append8Params q) {
  const AppendParams& p = q.p;
  __shared__ int64_t row_base[kMaxTileTokens];     // pool row of each token of the tile, in units
  const int g0 = (int)blockIdx.x * p.tile_tokens;
  const int ntok = min(p.tile_tokens, p.total_q - g0);
  if ((int)threadIdx.x < ntok) {
    const int g = g0 + (int)threadIdx.x;
    int lo = 0, hi = p.num_seqs;                   // segment of new token g, in [lo, hi)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.q_offsets[mid] <= g) lo = mid; else hi = mid;
    }
    const int q0 = p.q_offsets[lo];
    const int q_len = p.q_offsets[lo + 1] - q0;
    const int pos = p.ctx_lens[lo] - q_len + (g - q0);
    const int64_t blk = p.block_tables[(int64_t)lo * p.max_blocks + pos / kBlockSize];
    row_base[threadIdx.x] = (blk * kBlockSize + pos % kBlockSize) * (int64_t)p.upr;
  }
  __syncthreads();
  // One 16-byte unit of codes comes from two consecutive 16-byte units of bf16.
  const unit_t* src = (blockIdx.y ? p.v_new : p.k_new) + (int64_t)g0 * p.upr * 2;
  unit_t* pool = blockIdx.y ? p.pool_v : p.pool_k;
  const float scale = blockIdx.y ? q.v_scale : q.k_scale;
  const int total = ntok * p.upr;
  for (int u = (int)threadIdx.x; u < total; u += kAppendThreads) {
    const unit_t x0 = __builtin_nontemporal_load(src + 2 * u);
    const unit_t x1 = __builtin_nontemporal_load(src + 2 * u + 1);
    unit_t c;
    c.x = quantise4(x0.x, x0.y, scale);
    c.y = quantise4(x0.z, x0.w, scale);
    c.z = quantise4(x1.x, x1.y, scale);
    c.w = quantise4(x1.z, x1.w, scale);
    const int t = u / p.upr;
    pool[row_base[t] + (u - t * p.upr)] = c;
  }
}

// Argument checks and parameter block shared by the two entry points; elem_bytes = bytes per
// cached element (2: bf16, 1: codes).
int prepare_append(const void* k_new, const void* v_new, const dsv_kv_pool* pool, int32_t layer,
                   const int32_t* block_tables, int32_t max_blocks_per_seq, const int32_t* q_offsets,
                   const int32_t* ctx_lens, const int32_t* q_offsets_host,
                   const int32_t* ctx_lens_host, int32_t num_seqs, int elem_bytes, AppendParams* out) {
  int rc = check_pool(pool);
  if (rc != DSV_OK) return rc;
  if (num_seqs < 0) return DSV_E_INVALID;
  if (num_seqs == 0) return DSV_OK;
  if (!k_new || !v_new || !block_tables || !q_offsets || !ctx_lens || !q_offsets_host ||
      !ctx_lens_host)
    return DSV_E_INVALID;
  if (layer < 0 || layer >= pool->num_layers || max_blocks_per_seq < 1) return DSV_E_INVALID;
  if (q_offsets_host[0] != 0) return DSV_E_INVALID;
  for (int i = 0; i < num_seqs; ++i) {
    const int64_t q_len = (int64_t)q_offsets_host[i + 1] - q_offsets_host[i];
    if (q_len < 1 || ctx_lens_host[i] < q_len) return DSV_E_INVALID;
    if (((int64_t)ctx_lens_host[i] + kBlockSize - 1) / kBlockSize > max_blocks_per_seq)
      return DSV_E_INVALID;
  }
  const int64_t row_bytes = (int64_t)pool->num_kv_heads * pool->head_dim * elem_bytes;   // multiple of 64
  if (pool->num_layers > 1 && (pool->layer_stride * elem_bytes % 16)) return DSV_E_INVALID;
  if ((reinterpret_cast<uintptr_t>(k_new) & 15) || (reinterpret_cast<uintptr_t>(v_new) & 15) ||
      (reinterpret_cast<uintptr_t>(pool->k_base) & 15) || (reinterpret_cast<uintptr_t>(pool->v_base) & 15))
    return DSV_E_INVALID;
  AppendParams p;
  p.k_new = static_cast<const unit_t*>(k_new);
  p.v_new = static_cast<const unit_t*>(v_new);
  const int64_t layer_u = pool->num_layers > 1 ? (int64_t)layer * (pool->layer_stride * elem_bytes / 16) : 0;
  p.pool_k = static_cast<unit_t*>(pool->k_base) + layer_u;
  p.pool_v = static_cast<unit_t*>(pool->v_base) + layer_u;
  p.block_tables = block_tables;
  p.q_offsets = q_offsets;
  p.ctx_lens = ctx_lens;
  p.max_blocks = max_blocks_per_seq;
  p.num_seqs = num_seqs;
  p.total_q = q_offsets_host[num_seqs];
  p.upr = (int32_t)(row_bytes / 16);
  p.tile_tokens = p.upr >= kAppendUnits ? 1 : kAppendUnits / p.upr;
  if (p.tile_tokens > kMaxTileTokens) p.tile_tokens = kMaxTileTokens;
  *out = p;
  return 1;                                       // there is work to launch
}

}  // namespace
}  // namespace dsv

extern "C" int kv_append(const void* k_new, const void* v_new, const dsv_kv_pool* pool,
                         int32_t layer, const int32_t* block_tables, int32_t max_blocks_per_seq,
                         const int32_t* q_offsets, const int32_t* ctx_lens,
                         const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                         int32_t num_seqs, void* hip_stream) {
  using namespace dsv;
  AppendParams p;
  const int rc = prepare_append(k_new, v_new, pool, layer, block_tables, max_blocks_per_seq, q_offsets,
                                ctx_lens, q_offsets_host, ctx_lens_host, num_seqs, 2, &p);
  if (rc <= 0) return rc;
  const int64_t grid = ((int64_t)p.total_q + p.tile_tokens - 1) / p.tile_tokens;
  if (grid > 0x7fffffffLL) return DSV_E_UNSUPPORTED;
  begin_gpu_work();
  hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)grid, 2u), dim3(kAppendThreads), 0,
                     static_cast<hipStream_t>(hip_stream), p);
  return launch_status();
}

extern "C" int kv_append_fp8(const void* k_new, const void* v_new, const dsv_kv_pool* pool,
                             int32_t layer, const int32_t* block_tables, int32_t max_blocks_per_seq,
                             const int32_t* q_offsets, const int32_t* ctx_lens,
                             const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                             int32_t num_seqs, float k_scale, float v_scale, void* hip_stream) {
  using namespace dsv;
  if (!(k_scale > 0.0f) || isinf(k_scale) || !(v_scale > 0.0f) || isinf(v_scale)) return DSV_E_INVALID;
  Append8Params q;
  const int rc = prepare_append(k_new, v_new, pool, layer, block_tables, max_blocks_per_seq, q_offsets,
                                ctx_lens, q_offsets_host, ctx_lens_host, num_seqs, 1, &q.p);
  if (rc <= 0) return rc;
  q.k_scale = k_scale;
  q.v_scale = v_scale;
  const int64_t grid = ((int64_t)q.p.total_q + q.p.tile_tokens - 1) / q.p.tile_tokens;
  if (grid > 0x7fffffffLL) return DSV_E_UNSUPPORTED;
  begin_gpu_work();
  hipLaunchKernelGGL(kv_append_fp8_kernel, dim3((unsigned)grid, 2u), dim3(kAppendThreads), 0,
                     static_cast<hipStream_t>(hip_stream), q);
  return launch_status();
}
