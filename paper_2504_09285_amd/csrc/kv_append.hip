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

}  // namespace
}  // namespace dsv

extern "C" int kv_append(const void* k_new, const void* v_new, const dsv_kv_pool* pool,
                         int32_t layer, const int32_t* block_tables, int32_t max_blocks_per_seq,
                         const int32_t* q_offsets, const int32_t* ctx_lens,
                         const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                         int32_t num_seqs, void* hip_stream) {
  using namespace dsv;
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
  const int64_t row_elems = (int64_t)pool->num_kv_heads * pool->head_dim;   // multiple of 64
  if (pool->num_layers > 1 && (pool->layer_stride % 8)) return DSV_E_INVALID;
  AppendParams p;
  p.k_new = static_cast<const unit_t*>(k_new);
  p.v_new = static_cast<const unit_t*>(v_new);
  const int64_t layer_u = pool->num_layers > 1 ? (int64_t)layer * (pool->layer_stride / 8) : 0;
  p.pool_k = static_cast<unit_t*>(pool->k_base) + layer_u;
  p.pool_v = static_cast<unit_t*>(pool->v_base) + layer_u;
  p.block_tables = block_tables;
  p.q_offsets = q_offsets;
  p.ctx_lens = ctx_lens;
  p.max_blocks = max_blocks_per_seq;
  p.num_seqs = num_seqs;
  p.total_q = q_offsets_host[num_seqs];
  p.upr = (int32_t)(row_elems / 8);
  p.tile_tokens = p.upr >= kAppendUnits ? 1 : kAppendUnits / p.upr;
  if (p.tile_tokens > kMaxTileTokens) p.tile_tokens = kMaxTileTokens;
  const int64_t grid = ((int64_t)p.total_q + p.tile_tokens - 1) / p.tile_tokens;
  if (grid > 0x7fffffffLL) return DSV_E_UNSUPPORTED;
  hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)grid, 2u), dim3(kAppendThreads), 0,
                     static_cast<hipStream_t>(hip_stream), p);
  return launch_status();
}
