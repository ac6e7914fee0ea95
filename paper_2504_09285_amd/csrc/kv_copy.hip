// kv_pack_chunks / kv_unpack_chunks: the local gather/scatter on either side of chunk-based
// KV transfer (paper section 4.3).  Pure byte movement, HBM-bound: every payload byte is read
// once and written once with 16-byte accesses, a wave covering 1 KiB of contiguous memory per
// instruction on both sides.
//
// Work decomposition: one workgroup per (chunk, layer, K|V, tile of about 16 KiB of tokens), so
// that every thread issues its four loads and then its four stores exactly once: many small
// one-shot workgroups measured faster here than fewer looping ones.  Loads and stores carry the
// nontemporal hint (the data is touched once; it should not displace the attention kernels'
// block tables and queries from L2).  A
// token's row (all KV heads) is num_kv_heads*head_dim*2 bytes, contiguous in the chunk and in
// the pool; consecutive tokens are contiguous in the chunk and, inside one block, in the pool.
#include <stdlib.h>

#include "dsv_common.h"

namespace dsv {
namespace {

constexpr int kCopyThreads = 256;
constexpr int kTileUnits = kCopyThreads * 4;   // 16-byte units per workgroup: one load and one store round
constexpr int kUnroll = 4;

typedef uint32_t unit_t __attribute__((ext_vector_type(4)));   // one 16-byte unit

struct CopyParams {
  unit_t* pool_k;                 // layer 0 bases
  unit_t* pool_v;
  unit_t* chunk_buf;
  const int32_t* block_tables;
  const dsv_chunk_desc* descs;
  int64_t layer_stride_u;        // 16-byte units between layers
  int32_t max_blocks;
  int32_t num_layers;
  int32_t tile_tokens;           // tokens per workgroup: about kTileUnits units, at least one token
  int32_t tiles_per_chunk;       // ceil(max num_tokens / tile_tokens)
  int32_t upr;                   // 16-byte units per token row
  int32_t upr_shift;             // log2(upr) or -1
  int32_t off_shift;             // chunk_offset (elements) -> units: 3 for 2-byte, 4 for 1-byte elements
  uint32_t total_wgs;            // work items (chunk, plane, tile); the grid may be smaller and loop
};

// PACK = true: pool -> chunk.  PACK = false: chunk -> pool.
template <bool PACK>
__global__ __launch_bounds__(kCopyThreads) void kv_copy_kernel(CopyParams p) {
  // work item w = (chunk * 2L + plane) * tiles_per_chunk + tile, plane = layer*2 + (K=0|V=1).
  // Normally one workgroup per item; a launch held to fewer workgroups (see run_copy) strides.
  const uint32_t planes = 2u * (uint32_t)p.num_layers;
  for (uint32_t w = blockIdx.x; w < p.total_wgs; w += gridDim.x) {
  const uint32_t tile = w % (uint32_t)p.tiles_per_chunk;
  const uint32_t cp = w / (uint32_t)p.tiles_per_chunk;
  const uint32_t plane = cp % planes;
  const uint32_t c = cp / planes;

  const dsv_chunk_desc d = p.descs[c];
  const int tok0 = (int)tile * p.tile_tokens;
  if (tok0 >= d.num_tokens) continue;
  const int ntok = min(p.tile_tokens, d.num_tokens - tok0);

  unit_t* pool = ((plane & 1u) ? p.pool_v : p.pool_k) + (int64_t)(plane >> 1) * p.layer_stride_u;
  unit_t* chunk = p.chunk_buf + (d.chunk_offset >> p.off_shift) +
                 ((int64_t)plane * d.num_tokens + tok0) * p.upr;
  const int32_t* table = p.block_tables + (int64_t)d.seq * p.max_blocks;

  const int total = ntok * p.upr;                       // 16-byte units in this tile
  for (int u0 = threadIdx.x; u0 < total; u0 += kCopyThreads * kUnroll) {
    unit_t v[kUnroll];
    int64_t pool_u[kUnroll];
    int idx[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
      const int u = u0 + k * kCopyThreads;
      idx[k] = u;
      if (u < total) {
        const int row = p.upr_shift >= 0 ? (u >> p.upr_shift) : (u / p.upr);
        const int col = u - row * p.upr;
        const int t = d.token_begin + tok0 + row;
        const int64_t blk = table[t >> 4];
        pool_u[k] = (blk * kBlockSize + (t & 15)) * (int64_t)p.upr + col;
      }
    }
#pragma unroll
    for (int k = 0; k < kUnroll; ++k)
      if (idx[k] < total) v[k] = __builtin_nontemporal_load(PACK ? &pool[pool_u[k]] : &chunk[idx[k]]);
#pragma unroll
    for (int k = 0; k < kUnroll; ++k)
      if (idx[k] < total) {
        __builtin_nontemporal_store(v[k], PACK ? &chunk[idx[k]] : &pool[pool_u[k]]);
      }
  }
  }
}

// ---- unpack in the order of the destination ------------------------------------------------------
// Scattered 32 KiB destination blocks cost the plain unpack a tenth of the rate a sequential
// destination gets (writes that keep opening new DRAM rows; reads from scattered blocks, as in
// pack, do not suffer).  When the hand-off fills most of the destination pool, sweeping the pool's
// blocks in ascending order and fetching each one's tokens from wherever they sit in the chunk
// buffer turns the scattered side into the read side.  That needs the inverse of the block table
// for the blocks the chunks touch: inv[b] = (chunk, 16-token block within the chunk), built on the
// device into a caller-provided workspace by the two small kernels below.
__global__ void inv_init_kernel(int2* inv, int32_t num_blocks) {
  const int b = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (b < num_blocks) inv[b] = make_int2(-1, 0);
}

// grid (ceil(max blocks per chunk / 256), num_chunks)
__global__ void inv_build_kernel(int2* inv, int32_t num_blocks, const dsv_chunk_desc* __restrict__ descs,
                                 const int32_t* __restrict__ tables, int32_t max_blocks) {
  const dsv_chunk_desc d = descs[blockIdx.y];
  const int j = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (j * kBlockSize >= d.num_tokens) return;
  const int32_t b = tables[(int64_t)d.seq * max_blocks + d.token_begin / kBlockSize + j];
  if (b >= 0 && b < num_blocks) inv[b] = make_int2((int)blockIdx.y, j);   // (an entry outside the pool is not followed)
}

// Work item w = (plane * num_blocks + block) * tiles_per_block + tile.
__global__ __launch_bounds__(kCopyThreads) void kv_unpack_ordered_kernel(CopyParams p, const int2* __restrict__ inv,
                                                                         int32_t num_blocks, int32_t tiles_per_block) {
  for (uint32_t w = blockIdx.x; w < p.total_wgs; w += gridDim.x) {
    const uint32_t tile = w % (uint32_t)tiles_per_block;
    const uint32_t pb = w / (uint32_t)tiles_per_block;
    const uint32_t b = pb % (uint32_t)num_blocks;
    const uint32_t plane = pb / (uint32_t)num_blocks;
    const int2 cj = inv[b];
    if (cj.x < 0) continue;                                   // a block the hand-off does not touch
    const dsv_chunk_desc d = p.descs[cj.x];
    const int slot0 = (int)tile * p.tile_tokens;              // chunks start on block boundaries: slot = token % 16
    const int tok0 = cj.y * kBlockSize + slot0;               // first token of this item, counted in the chunk
    if (tok0 >= d.num_tokens) continue;
    const int ntok = min(min(p.tile_tokens, kBlockSize - slot0), d.num_tokens - tok0);
    unit_t* pool = ((plane & 1u) ? p.pool_v : p.pool_k) + (int64_t)(plane >> 1) * p.layer_stride_u +
                   ((int64_t)b * kBlockSize + slot0) * p.upr;
    const unit_t* chunk = p.chunk_buf + (d.chunk_offset >> p.off_shift) + ((int64_t)plane * d.num_tokens + tok0) * p.upr;
    const int total = ntok * p.upr;                           // contiguous on both sides
    for (int u0 = threadIdx.x; u0 < total; u0 += kCopyThreads * kUnroll) {
      unit_t v[kUnroll];
#pragma unroll
      for (int k = 0; k < kUnroll; ++k)
        if (u0 + k * kCopyThreads < total) v[k] = __builtin_nontemporal_load(&chunk[u0 + k * kCopyThreads]);
#pragma unroll
      for (int k = 0; k < kUnroll; ++k)
        if (u0 + k * kCopyThreads < total) __builtin_nontemporal_store(v[k], &pool[u0 + k * kCopyThreads]);
    }
  }
}

int run_copy(bool pack, const dsv_kv_pool* pool, const int32_t* block_tables, int32_t max_blocks,
             const dsv_chunk_desc* descs, const dsv_chunk_desc* descs_host, int32_t num_chunks,
             void* chunk_buf, void* hip_stream, int elem_bytes, void* ordered_ws = nullptr) {
  // elem_bytes = 2 (bf16 cache) or 1 (8-bit codes): the copy itself only sees 16-byte units.
  const int epu = 16 / elem_bytes;                 // elements per unit
  int rc = check_pool(pool);
  if (rc) return rc;
  if (num_chunks < 0 || max_blocks < 1) return DSV_E_INVALID;
  if (num_chunks == 0) return DSV_OK;
  if (!block_tables || !descs || !descs_host || !chunk_buf) return DSV_E_INVALID;
  if ((reinterpret_cast<uintptr_t>(chunk_buf) & 15) || (reinterpret_cast<uintptr_t>(pool->k_base) & 15) ||
      (reinterpret_cast<uintptr_t>(pool->v_base) & 15))
    return DSV_E_INVALID;
  const int64_t row_elems = (int64_t)pool->num_kv_heads * pool->head_dim;   // multiple of 64
  if (pool->num_layers > 1 && (pool->layer_stride % epu)) return DSV_E_INVALID;
  if (pool->num_layers > 1 &&
      pool->layer_stride < (int64_t)pool->num_blocks * kBlockSize * row_elems)
    return DSV_E_INVALID;
  int max_tokens = 0;
  bool block_aligned = true;
  int64_t touched_blocks = 0;
  for (int c = 0; c < num_chunks; ++c) {
    const dsv_chunk_desc& d = descs_host[c];
    if (d.seq < 0 || d.token_begin < 0 || d.num_tokens < 1 || d.reserved != 0) return DSV_E_INVALID;
    if (d.chunk_offset < 0 || (d.chunk_offset % epu)) return DSV_E_INVALID;
    if (ceil_div((int64_t)d.token_begin + d.num_tokens, kBlockSize) > max_blocks) return DSV_E_INVALID;
    if (d.num_tokens > max_tokens) max_tokens = d.num_tokens;
    if (d.token_begin % kBlockSize) block_aligned = false;
    touched_blocks += ceil_div(d.num_tokens, kBlockSize);
  }
  CopyParams p;
  p.pool_k = static_cast<unit_t*>(pool->k_base);
  p.pool_v = static_cast<unit_t*>(pool->v_base);
  p.chunk_buf = static_cast<unit_t*>(chunk_buf);
  p.block_tables = block_tables;
  p.descs = descs;
  p.layer_stride_u = pool->num_layers > 1 ? pool->layer_stride / epu : 0;
  p.max_blocks = max_blocks;
  p.num_layers = pool->num_layers;
  p.upr = (int32_t)(row_elems / epu);
  p.off_shift = elem_bytes == 2 ? 3 : 4;
  p.tile_tokens = p.upr >= kTileUnits ? 1 : kTileUnits / p.upr;
  p.tiles_per_chunk = ceil_div(max_tokens, p.tile_tokens);
  p.upr_shift = (p.upr & (p.upr - 1)) == 0 ? __builtin_ctz((unsigned)p.upr) : -1;
  int64_t grid = (int64_t)num_chunks * 2 * pool->num_layers * p.tiles_per_chunk;
  if (grid > 0x7fffffffLL) return DSV_E_UNSUPPORTED;
  p.total_wgs = (uint32_t)grid;
  // A hand-off that runs next to attention on another stream (paper section 4.3: transfers must
  // not stall computation) can be held to a number of workgroups in flight, which caps the
  // share of the memory system it takes: DSV_COPY_MAX_WGS workgroups then stride over the items.
  if (const char* e = getenv("DSV_COPY_MAX_WGS")) {
    const long cap = atol(e);
    if (cap > 0 && cap < grid) grid = cap;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // The destination-ordered form pays when the chunks start on block boundaries (then no block is
  // shared by two chunks) and fill at least half of the pool (else most of the sweep finds
  // nothing to do, and blocks far apart share no DRAM row anyway); otherwise the plain form.
  if (!pack && ordered_ws && block_aligned && 2 * touched_blocks >= pool->num_blocks) {
    const int tile_tokens = p.tile_tokens < kBlockSize ? p.tile_tokens : kBlockSize;
    const int tiles_per_block = ceil_div(kBlockSize, tile_tokens);
    const int64_t items = (int64_t)2 * pool->num_layers * pool->num_blocks * tiles_per_block;
    if (items <= 0x7fffffffLL) {
      int2* inv = static_cast<int2*>(ordered_ws);
      begin_gpu_work();
      hipLaunchKernelGGL(inv_init_kernel, dim3((unsigned)ceil_div(pool->num_blocks, 256)), dim3(256), 0, stream, inv,
                         pool->num_blocks);
      hipLaunchKernelGGL(inv_build_kernel, dim3((unsigned)ceil_div(ceil_div(max_tokens, kBlockSize), 256), (unsigned)num_chunks),
                         dim3(256), 0, stream, inv, pool->num_blocks, descs, block_tables, max_blocks);
      p.tile_tokens = tile_tokens;
      p.total_wgs = (uint32_t)items;
      int64_t ogrid = items;
      if (const char* e = getenv("DSV_COPY_MAX_WGS")) {
        const long cap = atol(e);
        if (cap > 0 && cap < ogrid) ogrid = cap;
      }
      hipLaunchKernelGGL(kv_unpack_ordered_kernel, dim3((unsigned)ogrid), dim3(kCopyThreads), 0, stream, p, inv,
                         pool->num_blocks, tiles_per_block);
      return launch_status();
    }
  }
  begin_gpu_work();
  if (pack)
    hipLaunchKernelGGL(kv_copy_kernel<true>, dim3((unsigned)grid), dim3(kCopyThreads), 0, stream, p);
  else
    hipLaunchKernelGGL(kv_copy_kernel<false>, dim3((unsigned)grid), dim3(kCopyThreads), 0, stream, p);
  return launch_status();
}

}  // namespace
}  // namespace dsv

extern "C" int kv_pack_chunks(const dsv_kv_pool* src, const int32_t* block_tables,
                              int32_t max_blocks_per_seq, const dsv_chunk_desc* descs,
                              const dsv_chunk_desc* descs_host, int32_t num_chunks,
                              void* chunk_buf, void* hip_stream) {
  return dsv::run_copy(true, src, block_tables, max_blocks_per_seq, descs, descs_host, num_chunks,
                       chunk_buf, hip_stream, 2);
}

extern "C" int kv_unpack_chunks(const void* chunk_buf, const dsv_chunk_desc* descs,
                                const dsv_chunk_desc* descs_host, int32_t num_chunks,
                                const dsv_kv_pool* dst, const int32_t* dst_block_tables,
                                int32_t max_blocks_per_seq, void* hip_stream) {
  return dsv::run_copy(false, dst, dst_block_tables, max_blocks_per_seq, descs, descs_host,
                       num_chunks, const_cast<void*>(chunk_buf), hip_stream, 2);
}

extern "C" int kv_pack_chunks_fp8(const dsv_kv_pool* src, const int32_t* block_tables,
                                  int32_t max_blocks_per_seq, const dsv_chunk_desc* descs,
                                  const dsv_chunk_desc* descs_host, int32_t num_chunks,
                                  void* chunk_buf, void* hip_stream) {
  return dsv::run_copy(true, src, block_tables, max_blocks_per_seq, descs, descs_host, num_chunks,
                       chunk_buf, hip_stream, 1);
}

extern "C" int kv_unpack_chunks_fp8(const void* chunk_buf, const dsv_chunk_desc* descs,
                                    const dsv_chunk_desc* descs_host, int32_t num_chunks,
                                    const dsv_kv_pool* dst, const int32_t* dst_block_tables,
                                    int32_t max_blocks_per_seq, void* hip_stream) {
  return dsv::run_copy(false, dst, dst_block_tables, max_blocks_per_seq, descs, descs_host,
                       num_chunks, const_cast<void*>(chunk_buf), hip_stream, 1);
}

extern "C" size_t kv_unpack_chunks_ordered_workspace_bytes(int32_t num_blocks) {
  return num_blocks > 0 ? (size_t)num_blocks * sizeof(int2) : 0;
}

extern "C" int kv_unpack_chunks_ordered(const void* chunk_buf, const dsv_chunk_desc* descs,
                                        const dsv_chunk_desc* descs_host, int32_t num_chunks,
                                        const dsv_kv_pool* dst, const int32_t* dst_block_tables,
                                        int32_t max_blocks_per_seq, void* workspace, size_t workspace_bytes,
                                        void* hip_stream) {
  if (!dst || !workspace || (reinterpret_cast<uintptr_t>(workspace) & 7)) return DSV_E_INVALID;
  if (dst->num_blocks < 1) return DSV_E_INVALID;
  if (num_chunks > 65535) workspace = nullptr;                 // (one grid row per chunk in the table inversion)
  else if (workspace_bytes < kv_unpack_chunks_ordered_workspace_bytes(dst->num_blocks)) return DSV_E_WORKSPACE;
  return dsv::run_copy(false, dst, dst_block_tables, max_blocks_per_seq, descs, descs_host,
                       num_chunks, const_cast<void*>(chunk_buf), hip_stream, 2, workspace);
}
