// Internal interfaces between the attention translation units (not part of the ABI).
#pragma once
#include "dsv_common.h"

namespace dsv {

// How a batch is cut into GPU work.  Computed identically on the host (to size grids and the
// workspace) and on the device (to fill the work lists), from q_offsets / ctx_lens alone.
//
//  * "row" work: one query token against its causal context, cut along the context into
//    partitions of part_tokens tokens (split-K).  Used for decodes and for the smallest
//    prefill spans (fewer than mfma_min_qlen tokens and q_len * ctx_len below mfma_min_work):
//    the row path streams the context once per query token, the MFMA path once per span.  A row with one partition writes its output directly;
//    otherwise each partition writes an unnormalised partial and a merge kernel combines them.
//  * "tile" work: tile_tokens consecutive query tokens of a long prefill span for one KV head,
//    processed by the MFMA kernel.  When the batch holds too few query tiles to fill the device
//    (a short span on a long prefix), a query tile's context is cut into tile_part_tiles-sized
//    partitions as well: each partition is a work item that writes unnormalised partials, and a
//    merge kernel combines them (same arithmetic as for split rows).
struct PlanConfig {
  int32_t part_tokens;     // multiple of 16
  int32_t mfma_min_qlen;   // spans with q_len >= this go to the MFMA kernel
  int32_t mfma_min_work;   // ... and so do shorter spans of 2+ tokens with q_len * ctx_len >= this
  int32_t tile_tokens;     // query tokens per MFMA work item
  int32_t flat_heads;      // 0: a work item is 64 tokens x 4 query heads; h > 0: its 256 rows are
                           // the (token, head) pairs of tile_tokens = 256 / h tokens and h heads
  int32_t head_groups;     // work items per (query tile, KV head)
  int32_t row_nbuf;        // LDS ring slots (blocks) per wave of the row kernel: 2, 3, 4, 6 or 8
  int32_t num_cus;         // compute units of the device (sizes the persistent grid)
  int32_t tile_part_tiles; // 0: query tiles are never cut along the context; else a query tile
                           // that visits n KV tiles is cut into ceil(n / tile_part_tiles) partitions
  // Row work as one stream per workgroup (large row-only launches).  All rows' blocks, each row
  // preceded by stream_row_cost units for its start-up, form one sequence of stream_total units;
  // it is cut into stream_wgs equal runs, one per persistent workgroup, and a row that straddles a
  // cut is partitioned there (part_tokens is not used).  0 workgroups: the item form above.
  int32_t stream_wgs;
  int32_t stream_row_cost;
  int64_t stream_total;
};

// Position of the w-th cut of the row stream, and the run a position falls in.
__host__ __device__ inline int64_t stream_cut(int64_t w, const PlanConfig& c) {
  return (w * c.stream_total + c.stream_wgs - 1) / c.stream_wgs;
}
__host__ __device__ inline int stream_run_of(int64_t pos, const PlanConfig& c) {
  const int64_t g = pos * c.stream_wgs / c.stream_total;      // largest w with stream_cut(w) <= pos
  return (int)(g < c.stream_wgs ? g : c.stream_wgs - 1);
}

struct PlanCounts {
  int64_t rows = 0;        // query tokens on the row path
  int64_t items = 0;       // (row, partition) work items
  int64_t split_items = 0; // items belonging to rows with more than one partition
  int64_t tiles = 0;       // (span, q-tile, context partition) work items of the MFMA path
  int64_t split_qtiles = 0;   // q-tiles cut into more than one partition
  int64_t tile_split_items = 0;  // (query token, partition) partials of those q-tiles
  int32_t max_parts = 0;
  int32_t max_qtiles = 0;  // most query tiles of one segment on the MFMA path
  // Filled only for a cache of 8-bit codes: the MFMA path then reads a bf16 copy of the whole
  // context of every segment it serves.
  int64_t stage_segs = 0;        // segments on the MFMA path
  int64_t stage_blocks = 0;      // KV blocks of their contexts, summed
  int32_t stage_max_blocks = 0;  // largest number of blocks of one of them
};

// Device-resident work lists, carved out of the caller's workspace.
struct WorkLists {
  int32_t* row_qtok;       // [rows] index of the query token in q / out
  int32_t* row_item0;      // [rows] first item of the row
  int32_t* row_nparts;     // [rows]
  int4*    item_rec;       // [items]: {seq, qtok, ctx, part | nparts << 16}: everything a
                           // (row, partition) work item needs, in one 16-byte scalar read
  int32_t* tile_seq;       // [tiles]
  int32_t* tile_q0;        // [tiles] first new-token index j of the tile
  int32_t* tile_part;      // [tiles] partition | partitions << 16
  int32_t* tile_item0;     // [tiles] cut q-tiles: first partial of the q-tile (token j of the tile,
                           // partition p -> item tile_item0 + j * partitions + p), counted
                           // after the row path's items; -1 for uncut q-tiles
  int4*    split_rec;      // [split_qtiles] {seq, q0 of the tile, partitions, first partial}
  int4*    tile_rec;       // [tiles][2]: everything a work item of the MFMA kernel needs, in one
                           // 32-byte scalar read: {seq, q0 of the tile, partition | partitions << 16,
                           // first partial or -1} {first query token of the segment, q_len, ctx_len,
                           // block-table row that serves the segment}
  int32_t* tile_ctr;       // [64] counters of the persistent MFMA grid (next item per KV head,
                           // workgroups finished); zero between launches
  uint32_t* zero_line;     // 256 bytes of zeros (stands in for V rows that must not be read)
  int32_t* item_blk0;      // [items] pool block id of the item's first block
  int32_t* item_order;     // [items] the items in dispatch order: most blocks to stream first
  int4*    item_span;      // [items] stream form: {first block, end block, pool id of the first
                           // block, run (workgroup) the item belongs to}
  int32_t* wg_first;       // [stream_wgs + 1] stream form: first item of each workgroup's run
  float*   part_acc;       // [items][Hq][D]  unnormalised partial outputs
  float*   part_ml;        // [items][Hq][2]  running max (log2 domain) and sum
  // bf16 copy of the MFMA path's contexts (cache of 8-bit codes only, else null)
  int32_t* stage_seq;      // [stage_segs] segment of each staged context
  int32_t* stage_rows;     // [num_seqs] index into stage_seq / row of stage_table, or -1
  int32_t* stage_blk0;     // [stage_segs] first staged block of the context
  int32_t* stage_table;    // [stage_segs][stage_max_blocks] block table over the staged blocks
  uint16_t* stage_k;       // [stage_blocks][16][Hkv][D] bf16
  uint16_t* stage_v;
};

struct AttnArgs {
  const uint16_t* q;
  void* out;
  const uint16_t* k_pool;      // layer base already applied
  const uint16_t* v_pool;
  const int32_t* block_tables;
  const int32_t* q_offsets;
  const int32_t* ctx_lens;
  int32_t max_blocks;
  int32_t num_seqs;
  int32_t Hq, Hkv, D;
  float scale_log2e;           // softmax_scale * log2(e): scores are kept in the log2 domain
                               // (times the K dequantisation scale for a cache of 8-bit codes)
  int32_t out_bf16;
  float out_scale;             // multiplies the normalised output: 1, or the V dequantisation scale
  int32_t kv8;                 // 0: k_pool/v_pool hold bf16; 1: E4M3 codes, one byte per element
                               // (same geometry; the row kernel widens them in registers)
};

int launch_rows(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg,
                const PlanCounts& n, hipStream_t stream);
int launch_merge(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg, const PlanCounts& n,
                 hipStream_t stream);
// Widens the 8-bit contexts of the MFMA path's segments into the staged bf16 blocks.
int launch_stage(const AttnArgs& a, const WorkLists& w, const PlanCounts& n, hipStream_t stream);
int launch_prefill_tiles(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg,
                         const PlanCounts& n, hipStream_t stream);
// Prefill tiles and row items in one launch (same results as the two launches above).
bool mixed_launch_supported(const AttnArgs& a, const PlanConfig& cfg, const PlanCounts& n);
int launch_mixed(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg, const PlanCounts& n,
                 hipStream_t stream);

}  // namespace dsv
