// attn_mixed_batch: host entry point, batch planning (host counts + device work lists) and the
// split-context merge kernel.
//
// One step of a unified instance runs a token-level batch that mixes prefill spans and decode
// tokens (paper section 3.1 "Unified execution instances", section 4.2, Alg. 2).  The host side
// here only validates the batch and sizes the grids; the work lists themselves are produced by
// a small planning kernel on the same stream, so a call never synchronises and never copies
// from host memory.
#include <math.h>
#include <atomic>
#include <stdlib.h>
#include <string.h>

#include "attn_internal.h"

namespace dsv {
namespace {

constexpr int kPlanThreads = 1024;

// Benchmark hook: event pairs recorded around individual kernels (see dsv_profile_events).
thread_local hipEvent_t g_events[6][2] = {};

struct EventScope {
  hipEvent_t stop;
  hipStream_t stream;
  EventScope(int id, hipStream_t s) : stop(g_events[id][1]), stream(s) {
    if (g_events[id][0]) (void)hipEventRecord(g_events[id][0], s);
  }
  ~EventScope() {
    if (stop) (void)hipEventRecord(stop, stream);
  }
};

int env_int(const char* name, int fallback) {
  const char* s = getenv(name);
  if (!s || !*s) return fallback;
  return atoi(s);
}

// Compute units of the current device (256 on MI355X); falls back to that when no device answers.
int device_cus() {
  static int cached[kMaxDevices] = {};
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices) {
    if (cached[dev] > 0) return cached[dev];
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) {
      cached[dev] = n;
      return n;
    }
  }
  (void)hipGetLastError();
  return 256;
}

// ---- plan: counts --------------------------------------------------------------------------

__host__ __device__ inline bool on_row_path(int q_len, int ctx, const PlanConfig& c) {
  if (q_len >= c.mfma_min_qlen) return false;
  return q_len < 2 || (int64_t)q_len * ctx < c.mfma_min_work;
}
__host__ __device__ inline int parts_of(int ctx_eff, const PlanConfig& c) {
  return (ctx_eff + c.part_tokens - 1) / c.part_tokens;
}

// KV tiles the t-th query tile of a span visits: its last row sees tokens [0, prefix + 64(t+1)).
__host__ __device__ inline int kv_tiles_of(int ctx, int q_len, int t, const PlanConfig& c) {
  const int kv_end = min(ctx, ctx - q_len + (t + 1) * c.tile_tokens);
  return (kv_end + 63) / 64;                     // KV tiles are 64 tokens whatever the query tile
}
// Context partitions of a query tile that visits n_kv KV tiles.  With base = n_kv / P and
// rem = n_kv % P, partition p of P covers base + (p < rem) KV tiles from p * base + min(p, rem):
// sizes differ by at most one, none is empty, the shorter ones (diagonal included) come last.
__host__ __device__ inline int tile_parts_of(int n_kv, const PlanConfig& c) {
  return c.tile_part_tiles > 0 ? (n_kv + c.tile_part_tiles - 1) / c.tile_part_tiles : 1;
}

// How the plan kernel walks the query tiles (its has_tiles argument).  Sharing one segment's
// tiles among all threads, segment after segment, pays when a segment has more query tiles than
// there are such segments (a few long spans: config 3's four spans of 32 tiles); with many short
// spans it would be a serial walk over the segments (1,024 spans of one tile each: 0.95 ms
// against 0.02 ms), and each thread takes whole segments instead.
int tile_list_mode(const PlanCounts& n) {
  if (n.tiles == 0) return 0;
  return (n.stage_segs <= kPlanThreads && n.stage_segs <= n.max_qtiles) ? 2 : 1;
}

int validate_batch(int32_t S, const int32_t* qo, const int32_t* cl, int32_t max_blocks) {
  if (S < 0) return DSV_E_INVALID;
  if (S == 0) return DSV_OK;
  if (!qo || !cl) return DSV_E_INVALID;
  if (qo[0] != 0) return DSV_E_INVALID;
  for (int i = 0; i < S; ++i) {
    const int64_t q_len = (int64_t)qo[i + 1] - qo[i];
    if (q_len < 1 || cl[i] < q_len) return DSV_E_INVALID;
    if (max_blocks >= 0 && ceil_div(cl[i], kBlockSize) > max_blocks) return DSV_E_INVALID;
  }
  return DSV_OK;
}

PlanConfig choose_plan(int32_t S, const int32_t* qo, const int32_t* cl, bool kv8, int Hkv, int G) {
  PlanConfig c;
  // Query heads per KV head that do not fill groups of four (5, 6, 7, 9, ...; Qwen-2.5's 40/8
  // heads) would leave most waves of the last group's work items without rows.  Then a work
  // item takes the (token, head) pairs of all heads of a group of up to eight for fewer tokens:
  // 256 rows = 51 tokens x 5 heads, 42 x 6, 36 x 7, 32 x 8, each lane addressing its own head.
  c.flat_heads = 0;
  c.head_groups = ceil_div(G, 4);
  if (G > 4 && G % 4 != 0) {
    c.head_groups = ceil_div(G, 8);
    c.flat_heads = ceil_div(G, c.head_groups);
  }
  const int wgs_per_tile = Hkv * c.head_groups;
  // Which spans take the row path.  It streams the context once per query token, the MFMA path
  // once per span (with mostly empty query tiles, whose idle waves step aside) at a fixed cost
  // of about 10 us per work item, so the MFMA path wins once a span's q_len * ctx_len passes
  // about 1,200 tokens; measured (32/8 heads, D=128, 64 spans): 4 tokens on 2,048 cached ones
  // 0.42 -> 0.18 ms, 15 tokens 1.26 -> 0.19 ms, 4 tokens on 128 cached ones 0.05 ms on the row
  // path against 0.10 on the other.  DSV_MFMA_MIN_QLEN forces a plain length threshold.
  // (8-bit cache: the MFMA path first widens the span's whole context into the staged copy, and
  // the row path streams half the bytes: plain threshold of 16 tokens; measured, spans of 8
  // tokens are about even and 15 tokens win only on long contexts or many spans.)
  c.mfma_min_qlen = 16;
  c.mfma_min_work = kv8 ? 0x7fffffff : 1200;
  const int forced_q = env_int("DSV_MFMA_MIN_QLEN", 0);
  if (forced_q > 0) { c.mfma_min_qlen = forced_q; c.mfma_min_work = 0x7fffffff; }
  c.tile_tokens = c.flat_heads ? 256 / c.flat_heads : 64;
  // LDS ring slots per wave of the row kernel.  (8-bit codes: a slot is half the size; two and
  // four slots measured the same, two keep the mixed launch available.)
  c.row_nbuf = env_int("DSV_ROW_NBUF", 2);
  if (kv8) {
    if (c.row_nbuf != 4 && c.row_nbuf != 8) c.row_nbuf = 2;
  } else {
    if (c.row_nbuf != 3 && c.row_nbuf != 4) c.row_nbuf = 2;
  }
  c.num_cus = device_cus();
  // Partition size: enough (row, partition) items to keep every compute unit streaming to the
  // end of the launch, but not so small that starting an item and the partial results written
  // per partition matter next to the KV bytes read.
  int64_t row_tokens = 0;
  for (int i = 0; i < S; ++i) {
    const int q_len = qo[i + 1] - qo[i];
    if (!on_row_path(q_len, cl[i], c)) continue;
    const int64_t prefix = cl[i] - q_len;
    row_tokens += (int64_t)q_len * prefix + (int64_t)q_len * (q_len + 1) / 2;
  }
  // Items stream side by side, one workgroup of up to eight waves (KV heads, or groups of 16
  // query heads) to a compute unit; `conc` items fill the device.  With the items dispatched longest first (the plan
  // kernel's order) the fewest, largest items that still keep every compute unit busy are
  // fastest, measured on decode batches of 32/8 heads with contexts of 200-2,600 tokens:
  //   0.13M streamed tokens: 640-token partitions (260 items) 96 us per step, 272 tokens 104 us,
  //                          1,024 tokens (180 items) 109 us;
  //   0.22M: 1,024 tokens (300 items) 150 us, 448 tokens 158 us;
  //   0.36M (config 2): 736 tokens (630 items, 2.5 per compute unit) 0.253 ms, 1,024 tokens (476)
  //                          0.258, 336 tokens 0.277; the same optimum on 8-bit codes;
  //   0.55M and more (config 4's decodes, config 5): the cap of 1,024 tokens.
  // So: with at least 1.5 conc items at the cap, 1.9 items per slot; with at least conc items at
  // the cap, the cap; otherwise the smallest partition whose items all start at once (at most
  // conc of them), down to 128 tokens.  A few items more than conc is the worst case: config 3's
  // 16 decodes (64k tokens) take 47 us in 257 items of 256 tokens or 208 of 320, and 62 us in
  // 274 items of 240.  (A small batch is latency-bound: 8 decodes on 1,024 tokens 30 -> 23 us per
  // step with 128-token instead of 256-token partitions; 64-token partitions are slower again.)
  auto items_at = [&](int64_t p) {
    int64_t n = 0;
    for (int i = 0; i < S; ++i) {
      const int q_len = qo[i + 1] - qo[i];
      if (!on_row_path(q_len, cl[i], c)) continue;
      for (int j = 0; j < q_len; ++j) n += (cl[i] - q_len + j + p) / p;        // ceil((ctx_eff) / p)
    }
    return n;
  };
  // (Fewer than eight KV heads: a workgroup is smaller and several share a compute unit, but the
  // measured optimum follows the number of workgroups: 2,048 decodes with one KV head run 3 %
  // faster with the partitions a count of one item per compute unit gives.)
  const int64_t conc = max((int64_t)1, (int64_t)c.num_cus * 8 / max((int64_t)8, (int64_t)Hkv * ceil_div(G, 16)));
  const int64_t n_cap = items_at(1024);
  int64_t part = 1024;
  if (n_cap * 2 >= conc * 3) {
    part = (row_tokens * 10 / (conc * 19) + 15) / 16 * 16;
    if (part > 1024) part = 1024;
    if (part < 128) part = 128;
  } else if (n_cap < conc) {
    int64_t lo = 128 / 16, hi = 1024 / 16;       // smallest multiple of 16 with items_at <= conc
    while (lo < hi) {
      const int64_t mid = (lo + hi) / 2;
      if (items_at(mid * 16) <= conc) hi = mid; else lo = mid + 1;
    }
    part = lo * 16;
  }
  const int forced = env_int("DSV_PART_TOKENS", 0);
  if (forced >= 16) part = forced / 16 * 16;
  if (part > 1024) part = 1024;                 // the row kernel keeps one 64-entry table vector
  c.part_tokens = (int32_t)part;
  // Query tiles are cut along the context only when there are too few of them to fill the
  // device (a short span on a long prefix: 8 query tiles x 8 KV heads would occupy a quarter of
  // the compute units for the whole step).  Then the partitions are sized for about three
  // workgroups per compute unit, and never below 16 KV tiles (1024 tokens), so that the
  // partials a partition writes (64 tokens x 4 heads x D floats) stay small next to the K/V it
  // reads.  DSV_TILE_PART_TILES forces a size (tests), -1 turns cutting off.
  c.tile_part_tiles = 0;
  int64_t kv_visits = 0, largest = 0;
  for (int i = 0; i < S; ++i) {
    const int q_len = qo[i + 1] - qo[i];
    if (on_row_path(q_len, cl[i], c)) continue;
    const int nt = ceil_div(q_len, c.tile_tokens);
    for (int t = 0; t < nt; ++t) {
      const int n_kv = kv_tiles_of(cl[i], q_len, t, c);
      kv_visits += n_kv;
      if (n_kv > largest) largest = n_kv;
    }
  }
  // Uncut, the step lasts at least as long as its largest query tile, and at least its share of
  // all KV tile visits; cutting pays when the former is well above the latter (measured: 512
  // tokens on 131,072 cached ones 2.8 -> 1.3 ms, 64 on 16,384 0.38 -> 0.08 ms; 2,048 on 65,536,
  // which already has one equal workgroup per compute unit, gets 13 % slower and is left alone).
  const int64_t per_cu = (kv_visits * wgs_per_tile + c.num_cus - 1) / c.num_cus;
  if (largest > 16 && 2 * largest > 3 * per_cu) {
    int64_t t = (per_cu + 2) / 3;
    if (t < 16) t = 16;
    if (t > 0x3fffffff) t = 0x3fffffff;
    c.tile_part_tiles = (int32_t)t;
  }
  const int forced_t = env_int("DSV_TILE_PART_TILES", 0);
  if (forced_t > 0) c.tile_part_tiles = forced_t;
  if (forced_t < 0) c.tile_part_tiles = 0;
  // Row work as one stream per workgroup.  A launch of row work alone with enough blocks per
  // compute unit is cut into equal runs instead of (row, partition) items of a fixed size: no
  // launch tail, one start-up per row instead of one per partition, and far fewer partials
  // (rows + workgroups instead of one per 1,024 tokens: the partials' stores are what costs the
  // K/V stream most, see attn_rows_stream.h).  DSV_ROWS_STREAM: 0 never; n >= 1 whenever the
  // geometry allows, with n workgroups (tests).
  c.stream_wgs = 0;
  c.stream_row_cost = 2;        // a row's start-up, in blocks' worth of streaming time
  c.stream_total = 0;
  {
    const int want = env_int("DSV_ROWS_STREAM", -1);
    int64_t rows = 0, blocks = 0, q_tiles = 0;
    for (int i = 0; i < S; ++i) {
      const int q_len = qo[i + 1] - qo[i];
      if (!on_row_path(q_len, cl[i], c)) { q_tiles += ceil_div(q_len, c.tile_tokens); continue; }
      rows += q_len;
      for (int j = 0; j < q_len; ++j) blocks += ceil_div(cl[i] - q_len + j + 1, kBlockSize);
    }
    const bool tiles = q_tiles > 0;
    const bool apart = !tiles || env_int("DSV_MIXED_LAUNCH", 1) == 0;
    const bool geometry = Hkv <= 8 && G <= 16 && c.row_nbuf == 2 && forced < 16;
    const int64_t total = blocks + rows * c.stream_row_cost;
    // Row work alone: three quarters of the compute units stream faster than all of them
    // (config 5: 6.56 / 6.94 / 6.89 / 6.85 TB/s with 160 / 192 / 224 / 256 streams; config 2:
    // 6.10 / 6.39 / 6.30 / 6.28): 192 streams already hold more bytes in flight than the memory
    // system turns round, more only lengthen its queues.
    int wgs = max(8, c.num_cus * 3 / 4 / 8 * 8);
    if (!apart) {
      // Rows and prefill tiles in one launch: the row streams take `wgs` compute units for the
      // whole launch, the tiles' workgroups go through the others one item at a time.  The split
      // that lets both sides end together, from what each side delivers on a share of the device
      // (rows: 3.3 / 4.5 / 5.6 / 6.3 / 6.7 TB/s from 64 / 96 / 128 / 160 / 192 of 256 compute
      // units, measured on config 4's decodes; tiles: 1.9 us per KV tile visited and 8 us per
      // work item on a compute unit when all of them run tiles).  Too few row streams are the
      // worse mistake: streams that end early hand their compute units to the tiles, tiles that
      // end early cannot help the streams; and a compute unit runs tiles about 1.3 times faster
      // when only a share of the device does (clocks).  Hence the factor on the tiles' side,
      // set on config 4: 0.65 ms per step with 144-160 streams, 0.68 with 128, 0.67 with 192.
      // (Both sides scale with the head size alike; 128 stands for it.)
      const double row_gb = (double)blocks * (2.0 * kBlockSize * Hkv * 128 * (kv8 ? 1 : 2)) * 1e-9;
      const double tile_cu_us = 0.7 * ((double)kv_visits * wgs_per_tile * 1.9 + (double)q_tiles * wgs_per_tile * 8.0);
      static const double kShare[] = {0.0, 0.25, 0.375, 0.5, 0.625, 0.75, 1.0};
      static const double kTBs[] = {0.0, 3.34, 4.52, 5.60, 6.33, 6.67, 6.67};
      double best_t = 1e300;
      for (int w8 = 8; w8 + 8 <= c.num_cus; w8 += 8) {
        const double share = (double)w8 / c.num_cus;
        int k = 0;
        while (k < 5 && share > kShare[k + 1]) ++k;
        const double tbs = kTBs[k] + (kTBs[k + 1] - kTBs[k]) * (share - kShare[k]) / (kShare[k + 1] - kShare[k]);
        const double t_rows = row_gb / tbs * 1e3;                       // us
        const double t_tiles = tile_cu_us / (c.num_cus - w8);
        const double t = t_rows > t_tiles ? t_rows : t_tiles;
        if (t < best_t) { best_t = t; wgs = w8; }
      }
    }
    if (want >= 1) wgs = want;
    if (!apart) wgs = wgs / 8 * 8;          // whole groups of eight: the tiles keep KV head k on XCD k
    if (wgs > 4096) wgs = 4096;
    if ((int64_t)wgs > blocks) wgs = (int)blocks;
    if (rows > 0 && geometry && want != 0 && wgs >= 1 && (apart || (wgs >= 8 && wgs + 8 <= c.num_cus)) &&
        (want >= 1 || blocks >= (int64_t)16 * c.num_cus)) {
      c.stream_wgs = wgs;
      c.stream_total = total;
    }
  }
  return c;
}

PlanCounts count_plan(int32_t S, const int32_t* qo, const int32_t* cl, const PlanConfig& c) {
  PlanCounts n;
  for (int i = 0; i < S; ++i) {
    const int q_len = qo[i + 1] - qo[i];
    if (on_row_path(q_len, cl[i], c) && c.stream_wgs > 0) {
      // Stream form: a cut adds one item to the row it falls in; where the cuts fall is worked
      // out on the device, the host only needs bounds (at most stream_wgs - 1 cuts in all).
      n.rows += q_len;
      n.items += q_len;
    } else if (on_row_path(q_len, cl[i], c)) {
      n.rows += q_len;
      for (int j = 0; j < q_len; ++j) {
        const int np = parts_of(cl[i] - q_len + j + 1, c);
        n.items += np;
        if (np > 1) n.split_items += np;
        if (np > n.max_parts) n.max_parts = np;
      }
    } else {
      const int nt = ceil_div(q_len, c.tile_tokens);
      if (nt > n.max_qtiles) n.max_qtiles = nt;
      for (int t = 0; t < nt; ++t) {
        const int np = tile_parts_of(kv_tiles_of(cl[i], q_len, t, c), c);
        n.tiles += np;
        if (np > 1) {
          n.split_qtiles += 1;
          n.tile_split_items += (int64_t)min(c.tile_tokens, q_len - t * c.tile_tokens) * np;
        }
        if (np > n.max_parts) n.max_parts = np;
      }
      const int nblk = ceil_div(cl[i], kBlockSize);
      n.stage_segs += 1;
      n.stage_blocks += nblk;
      if (nblk > n.stage_max_blocks) n.stage_max_blocks = nblk;
    }
  }
  if (c.stream_wgs > 0 && n.rows > 0) {
    n.items += c.stream_wgs - 1;
    n.split_items = c.stream_wgs > 1 ? n.items : 0;
    n.max_parts = max(n.max_parts, c.stream_wgs);
  }
  return n;
}

// ---- workspace layout ----------------------------------------------------------------------

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

size_t carve(const PlanCounts& n, int S, int Hq, int Hkv, int D, bool kv8, char* base, WorkLists* w) {
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off = align_up(off + bytes);
    return p;
  };
  const size_t rows = (size_t)n.rows, items = (size_t)n.items, tiles = (size_t)n.tiles;
  char* p1 = take(rows * 4);
  char* p3 = take(rows * 4); char* p4 = take(rows * 4);
  char* p5 = take(items * 16);
  char* p7 = take(tiles * 4); char* p8 = take(tiles * 4);
  char* p7b = take(tiles * 4); char* p7c = take(tiles * 4);
  char* p7d = take((size_t)n.split_qtiles * 16);
  char* p7e = take(tiles * 32);
  char* p7f = take(64 * 4);
  char* pz = take(256);
  char* pc = take(items * 4);
  char* po = take(items * 4);
  char* psp = take(items * 16);
  char* pwf = take((size_t)(4096 + 1) * 4);
  const size_t partials = items + (size_t)n.tile_split_items;    // row items first, then cut q-tiles
  char* p9 = take(partials * (size_t)Hq * D * 4);
  char* p10 = take(partials * (size_t)Hq * 2 * 4);
  char *s0 = nullptr, *s1 = nullptr, *s2 = nullptr, *s3 = nullptr, *s4 = nullptr, *s5 = nullptr;
  if (kv8 && n.tiles) {
    const size_t blk_bytes = (size_t)kBlockSize * Hkv * D * 2;
    s0 = take((size_t)n.stage_segs * 4); s1 = take((size_t)S * 4); s2 = take((size_t)n.stage_segs * 4);
    s3 = take((size_t)n.stage_segs * n.stage_max_blocks * 4);
    s4 = take((size_t)n.stage_blocks * blk_bytes); s5 = take((size_t)n.stage_blocks * blk_bytes);
  }
  if (w) {
    w->stage_seq = (int32_t*)s0; w->stage_rows = (int32_t*)s1; w->stage_blk0 = (int32_t*)s2;
    w->stage_table = (int32_t*)s3; w->stage_k = (uint16_t*)s4; w->stage_v = (uint16_t*)s5;
    w->row_qtok = (int32_t*)p1;
    w->row_item0 = (int32_t*)p3; w->row_nparts = (int32_t*)p4;
    w->item_rec = (int4*)p5;
    w->tile_seq = (int32_t*)p7; w->tile_q0 = (int32_t*)p8;
    w->tile_part = (int32_t*)p7b; w->tile_item0 = (int32_t*)p7c; w->split_rec = (int4*)p7d;
    w->tile_rec = (int4*)p7e; w->tile_ctr = (int32_t*)p7f;
    w->zero_line = (uint32_t*)pz;
    w->item_blk0 = (int32_t*)pc;
    w->item_order = (int32_t*)po;
    w->item_span = (int4*)psp; w->wg_first = (int32_t*)pwf;
    w->part_acc = (float*)p9; w->part_ml = (float*)p10;
  }
  return off + 256;
}

// ---- plan: device work lists ---------------------------------------------------------------

// Exclusive scan of one int per thread across the block; returns the block total in *total.
// Each wave scans its 64 values with lane shuffles, the wave totals go through LDS, and every
// thread adds the totals of the waves before its own: two barriers instead of two per doubling.
__device__ int block_exclusive_scan(int v, int* smem, int* total) {
  constexpr int kPlanWaves = kPlanThreads / 64;
  const int lane = (int)threadIdx.x & 63, wave = (int)threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(incl, off, 64);
    if (lane >= off) incl += up;
  }
  if (lane == 63) smem[wave] = incl;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int k = 0; k < kPlanWaves; ++k) {
    const int t = smem[k];
    before += k < wave ? t : 0;
    all += t;
  }
  *total = all;
  __syncthreads();
  return before + incl - v;
}

constexpr int kOrderBins = 64;                 // a row item streams 1..64 blocks (part_tokens <= 1024)
// Sort key of a tile: bucket 0 holds the tiles with the most KV tiles to visit.
constexpr int kTileBuckets = 4 * kPlanThreads;
__device__ __forceinline__ int tile_bucket(int kv_tiles) {
  return kTileBuckets - 1 - min(kv_tiles, kTileBuckets - 1);
}
__global__ __launch_bounds__(kPlanThreads) void plan_kernel(const int32_t* __restrict__ q_offsets,
                                                            const int32_t* __restrict__ ctx_lens,
                                                            const int32_t* __restrict__ block_tables,
                                                            int32_t max_blocks, int32_t S, PlanConfig c,
                                                            WorkLists w, int32_t has_tiles,
                                                            int32_t stage, int32_t row_items) {
  __shared__ int smem[kPlanThreads];
  __shared__ int tile_slot[kTileBuckets];
  __shared__ int split_count, split_items;      // cut q-tiles and their partials handed out so far
  __shared__ int tseg_n;                        // segments with tile work, listed for the
  __shared__ int tseg_list[kPlanThreads];       // cooperative passes (has_tiles == 2)
  __shared__ int order_slot[kOrderBins + 1];    // row items by block count (bin kOrderBins - blocks)
  if (threadIdx.x == 0) { split_count = 0; split_items = 0; tseg_n = 0; }
  if (threadIdx.x < 64) w.zero_line[threadIdx.x] = 0u;
  if (threadIdx.x < 64) w.tile_ctr[threadIdx.x] = 0;

  // Tiles are listed heaviest first (most KV tiles to visit), so that the MFMA kernel's
  // workgroups, dispatched in list order, leave no long tile for the end: a counting sort on
  // the KV tile count.  The order of equal keys is left to the atomics; it affects nothing but
  // the dispatch order.
  // has_tiles (uniform): 0 = the host found no tile, the sort is skipped; 2 = at most
  // kPlanThreads segments hold tiles: they are listed first and all threads then share the
  // query tiles of one listed segment after the other (a long span's tiles are not one thread's
  // serial loop); 1 = more such segments than the list holds: each thread walks the query tiles
  // of its own segments.
  for (int b = (int)threadIdx.x; has_tiles && b < kTileBuckets; b += kPlanThreads) tile_slot[b] = 0;
  __syncthreads();
  if (has_tiles == 2) {
    for (int i = (int)threadIdx.x; i < S; i += kPlanThreads) {
      const int q_len = q_offsets[i + 1] - q_offsets[i];
      if (q_len > 0 && !on_row_path(q_len, ctx_lens[i], c)) tseg_list[atomicAdd(&tseg_n, 1)] = i;
    }
    __syncthreads();
  }
  // fn(segment, q_len, ctx, q0, query tile) for every query tile of the batch, spread over the threads.
  auto for_each_query_tile = [&](auto&& fn) {
    if (has_tiles == 2) {
      const int n_list = tseg_n;
      for (int k = 0; k < n_list; ++k) {
        const int i = tseg_list[k];
        const int q0 = q_offsets[i], q_len = q_offsets[i + 1] - q0, ctx = ctx_lens[i];
        const int n_tiles = (q_len + c.tile_tokens - 1) / c.tile_tokens;
        for (int t = (int)threadIdx.x; t < n_tiles; t += kPlanThreads) fn(i, q_len, ctx, t);
      }
    } else if (has_tiles == 1) {
      for (int i = (int)threadIdx.x; i < S; i += kPlanThreads) {
        const int q0 = q_offsets[i], q_len = q_offsets[i + 1] - q0, ctx = ctx_lens[i];
        if (q_len > 0 && !on_row_path(q_len, ctx, c)) {
          const int n_tiles = (q_len + c.tile_tokens - 1) / c.tile_tokens;
          for (int t = 0; t < n_tiles; ++t) fn(i, q_len, ctx, t);
        }
      }
    }
  };
  for_each_query_tile([&](int, int q_len, int ctx, int t) {
    const int n_kv = kv_tiles_of(ctx, q_len, t, c), P = tile_parts_of(n_kv, c);
    const int base_kv = n_kv / P, rem = n_kv - base_kv * P;
    if (rem) atomicAdd(&tile_slot[tile_bucket(base_kv + 1)], rem);
    atomicAdd(&tile_slot[tile_bucket(base_kv)], P - rem);
  });
  __syncthreads();
  if (has_tiles) {
    constexpr int kPer = kTileBuckets / kPlanThreads;
    int cnt[kPer], sum = 0, total;
    for (int k = 0; k < kPer; ++k) { cnt[k] = tile_slot[threadIdx.x * kPer + k]; sum += cnt[k]; }
    int ex = block_exclusive_scan(sum, smem, &total);
    for (int k = 0; k < kPer; ++k) { tile_slot[threadIdx.x * kPer + k] = ex; ex += cnt[k]; }
    __syncthreads();
  }

  int row_carry = 0, item_carry = 0, stage_carry = 0, sblk_carry = 0;
  int64_t cost_carry = 0;                       // stream form: units of the row stream so far
  const bool streamed = c.stream_wgs > 0;       // (uniform)
  for (int base = 0; base < S; base += kPlanThreads) {
    const int i = base + (int)threadIdx.x;
    int q0 = 0, q_len = 0, ctx = 0, n_rows = 0, n_items = 0, n_tiles = 0, seg_cost = 0;
    if (i < S) {
      q0 = q_offsets[i];
      q_len = q_offsets[i + 1] - q0;
      ctx = ctx_lens[i];
      if (on_row_path(q_len, ctx, c)) {
        n_rows = q_len;
        for (int j = 0; j < q_len; ++j) {
          if (streamed) seg_cost += (ctx - q_len + j + kBlockSize) / kBlockSize + c.stream_row_cost;
          else n_items += parts_of(ctx - q_len + j + 1, c);
        }
      } else {
        n_tiles = (q_len + c.tile_tokens - 1) / c.tile_tokens;
      }
    }
    // Stream form: a row occupies [pre, pre + cost) of the stream, its blocks the part behind the
    // first stream_row_cost units; its first item belongs to the run that position pre +
    // stream_row_cost falls in, and every later cut inside its blocks starts another item.
    int64_t seg_pre = 0;
    if (streamed) {
      int tot_cost;
      seg_pre = cost_carry + block_exclusive_scan(seg_cost, smem, &tot_cost);
      cost_carry += tot_cost;
      int64_t pre = seg_pre;
      for (int j = 0; j < n_rows; ++j) {
        const int nb = (ctx - q_len + j + kBlockSize) / kBlockSize;
        const int64_t first = pre + c.stream_row_cost;
        n_items += stream_run_of(first + nb - 1, c) - stream_run_of(first, c) + 1;
        pre += nb + c.stream_row_cost;
      }
    }
    int tot_rows, tot_items;
    int row0 = row_carry + block_exclusive_scan(n_rows, smem, &tot_rows);
    int item0 = item_carry + block_exclusive_scan(n_items, smem, &tot_items);
    for (int j = 0; j < n_rows; ++j) {
      const int ctx_eff = ctx - q_len + j + 1;
      const int r = row0 + j;
      int np;
      if (streamed) {
        const int nb = (ctx_eff + kBlockSize - 1) / kBlockSize;
        const int64_t first = seg_pre + c.stream_row_cost;
        const int g0 = stream_run_of(first, c);
        np = stream_run_of(first + nb - 1, c) - g0 + 1;
        for (int p = 0; p < np; ++p) {
          const int b0 = p == 0 ? 0 : (int)(stream_cut(g0 + p, c) - first);
          const int b1 = p == np - 1 ? nb : (int)(stream_cut(g0 + p + 1, c) - first);
          w.item_rec[item0 + p] = make_int4(i, q0 + j, ctx_eff, p | (np << 16));
          w.item_span[item0 + p] = make_int4(b0, b1, 0, g0 + p);
        }
        seg_pre += nb + c.stream_row_cost;
      } else {
        np = parts_of(ctx_eff, c);
        for (int p = 0; p < np; ++p) w.item_rec[item0 + p] = make_int4(i, q0 + j, ctx_eff, p | (np << 16));
      }
      w.row_qtok[r] = q0 + j;
      w.row_item0[r] = item0;
      w.row_nparts[r] = np;
      item0 += np;
    }
    row_carry += tot_rows;
    item_carry += tot_items;
    if (stage) {
      // Segments on the MFMA path, in segment order, and the staged blocks of their contexts
      // (uniform branch: `stage` is a kernel argument).
      const int is_staged = n_tiles > 0 ? 1 : 0;
      const int n_sblk = is_staged ? (ctx + kBlockSize - 1) / kBlockSize : 0;
      int tot_s, tot_b;
      const int s0 = stage_carry + block_exclusive_scan(is_staged, smem, &tot_s);
      const int sb0 = sblk_carry + block_exclusive_scan(n_sblk, smem, &tot_b);
      if (i < S) w.stage_rows[i] = is_staged ? s0 : -1;
      if (is_staged) {
        w.stage_seq[s0] = i;
        w.stage_blk0[s0] = sb0;
      }
      stage_carry += tot_s;
      sblk_carry += tot_b;
    }
  }
  // Placement: every query tile takes list positions for its partitions (two sizes at most).
  // (After the segment loop above: a record names the block-table row that serves its segment,
  // which for a cache of 8-bit codes is the staged row assigned there.)
  __syncthreads();
  for_each_query_tile([&](int i, int q_len, int ctx, int t) {
    const int n_kv = kv_tiles_of(ctx, q_len, t, c), P = tile_parts_of(n_kv, c);
    int first_partial = -1;
    if (P > 1) {
      // A cut q-tile: its partials (one per query token and partition) sit behind the row
      // path's items; the order in which q-tiles take their ranges does not matter.
      const int ntok = min(c.tile_tokens, q_len - t * c.tile_tokens);
      first_partial = row_items + atomicAdd(&split_items, ntok * P);
      w.split_rec[atomicAdd(&split_count, 1)] = make_int4(i, t * c.tile_tokens, P, first_partial);
    }
    const int base_kv = n_kv / P, rem = n_kv - base_kv * P;
    const int pos_long = rem ? atomicAdd(&tile_slot[tile_bucket(base_kv + 1)], rem) : 0;
    const int pos_short = atomicAdd(&tile_slot[tile_bucket(base_kv)], P - rem);
    for (int pp = 0; pp < P; ++pp) {
      const int pos = pp < rem ? pos_long + pp : pos_short + (pp - rem);
      w.tile_seq[pos] = i;
      w.tile_q0[pos] = t * c.tile_tokens;
      w.tile_part[pos] = pp | (P << 16);
      w.tile_item0[pos] = first_partial;
      w.tile_rec[2 * pos] = make_int4(i, t * c.tile_tokens, pp | (P << 16), first_partial);
      w.tile_rec[2 * pos + 1] = make_int4(q_offsets[i], q_len, ctx, stage ? w.stage_rows[i] : i);
    }
  });

  // Second pass, all threads: the id of each item's first block, so that the row kernel can
  // request its first K/V block as soon as it has read the item record.
  // The same pass lists the items in dispatch order, those with the most blocks first (counting
  // sort by block count, at most 64), so that the row kernel's workgroups, dispatched in list
  // order, end with the short last partitions of the rows instead of with whatever the last
  // segments hold.  Most items are full partitions: a wave counts and places those with one
  // atomic per wave.  The order of equal keys is left to the atomics; it affects nothing but the
  // dispatch order.
  if (streamed) {
    // Stream form: each item's first block id, and the first item of every run.  Items are listed
    // in stream order, so their runs never decrease; an item that opens runs (g_prev, g] is the
    // first item of each of them (a run that starts inside a row's start-up units has no item of
    // its own before the next row begins: it takes that row's first item too).
    __syncthreads();
    int32_t* span_words = reinterpret_cast<int32_t*>(w.item_span);
    for (int it = (int)threadIdx.x; it < item_carry; it += kPlanThreads) {
      const int4 rec = w.item_rec[it];
      const int b0 = span_words[4 * it], g = span_words[4 * it + 3];
      span_words[4 * it + 2] = block_tables[(int64_t)rec.x * max_blocks + b0];
      const int g_prev = it > 0 ? span_words[4 * (it - 1) + 3] : -1;
      for (int r = g_prev + 1; r <= g; ++r) w.wg_first[r] = it;
    }
    if (threadIdx.x == 0) {
      const int g_last = item_carry > 0 ? span_words[4 * (item_carry - 1) + 3] : -1;
      for (int r = g_last + 1; r <= c.stream_wgs; ++r) w.wg_first[r] = item_carry;
    }
    return;
  }
  if (threadIdx.x <= kOrderBins) order_slot[threadIdx.x] = 0;
  __syncthreads();
  const int full_blocks = c.part_tokens / kBlockSize;
  auto blocks_of = [&](const int4& rec) {
    const int part = rec.w & 0xffff;
    const int t1 = min(rec.z, (part + 1) * c.part_tokens);
    return (t1 + kBlockSize - 1) / kBlockSize - part * full_blocks;       // 1 .. full_blocks
  };
  // take(bin, valid): a position counter of the bin, one atomic per wave for the full-size bin.
  auto take = [&](int nb, bool valid) {
    const bool full = valid && nb == full_blocks;
    const unsigned long long m = __ballot(full);
    int pos = 0;
    if (full) {
      const int lane = (int)threadIdx.x & 63;
      const int lead = __ffsll((long long)m) - 1;
      if (lane == lead) pos = atomicAdd(&order_slot[kOrderBins - nb], __popcll(m));
      pos = __shfl(pos, lead, 64) + __popcll(m & ((1ull << lane) - 1ull));
    } else if (valid) {
      pos = atomicAdd(&order_slot[kOrderBins - nb], 1);
    }
    return pos;
  };
  const int item_iters = (item_carry + kPlanThreads - 1) / kPlanThreads;   // uniform trip count
  for (int k = 0; k < item_iters; ++k) {
    const int it = k * kPlanThreads + (int)threadIdx.x;
    const bool valid = it < item_carry;
    int nb = 0;
    if (valid) {
      const int4 rec = w.item_rec[it];
      const int b0 = (rec.w & 0xffff) * full_blocks;
      w.item_blk0[it] = block_tables[(int64_t)rec.x * max_blocks + b0];
      nb = blocks_of(rec);
    }
    take(nb, valid);
  }
  __syncthreads();
  if (threadIdx.x == 0) {                        // bins in order of falling block count
    int run = 0;
    for (int b = 0; b <= kOrderBins; ++b) { const int n = order_slot[b]; order_slot[b] = run; run += n; }
  }
  __syncthreads();
  for (int k = 0; k < item_iters; ++k) {
    const int it = k * kPlanThreads + (int)threadIdx.x;
    const bool valid = it < item_carry;
    const int nb = valid ? blocks_of(w.item_rec[it]) : 0;
    const int pos = take(nb, valid);
    if (valid) w.item_order[pos] = it;
  }
}

// ---- split-context merge -------------------------------------------------------------------
// Row r with n > 1 partitions: m* = max_p m_p; l* = sum_p l_p 2^(m_p-m*);
// out = sum_p acc_p 2^(m_p-m*) / l*.
// One workgroup per (row, group of heads); each thread owns 4 consecutive dims of one head.  The
// (m, l) pairs of up to kMergeChunk partitions are fetched by all threads at once into LDS and
// turned into weights there, and the partial outputs are then read with four independent loads
// in flight per thread, so the kernel is not a chain of dependent memory round trips.
constexpr int kMergeChunk = 64;

// TILES = false: blockIdx.x is a row of the row path.  TILES = true: blockIdx.x / 64 is a cut
// q-tile of the MFMA path and blockIdx.x % 64 the query token in it.
template <int D, bool TILES>
__global__ __launch_bounds__(256) void merge_kernel(AttnArgs a, WorkLists w, int tile_q) {
  constexpr int kThreadsPerHead = D / 4;
  constexpr int kHeadsPerBlock = 256 / kThreadsPerHead;
  __shared__ float s_m[kHeadsPerBlock][kMergeChunk];
  __shared__ float s_l[kHeadsPerBlock][kMergeChunk];
  int np, item0, qtok;
  if constexpr (TILES) {
    const int4 rec = w.split_rec[blockIdx.x / 64];       // {seq, q0 of the tile, partitions, first partial}
    const int j = (int)blockIdx.x % 64;
    if (j >= tile_q) return;                             // a q-tile holds tile_q <= 64 tokens (uniform)
    const int q_begin = a.q_offsets[rec.x];
    if (rec.y + j >= a.q_offsets[rec.x + 1] - q_begin) return;   // ragged last tile (uniform)
    np = rec.z;
    item0 = rec.w + j * np;
    qtok = q_begin + rec.y + j;
  } else {
    const int r = blockIdx.x;
    np = w.row_nparts[r];
    if (np <= 1) return;                                 // uniform for the workgroup
    item0 = w.row_item0[r];
    qtok = w.row_qtok[r];
  }
  const int hl = (int)threadIdx.x / kThreadsPerHead;     // head within the block
  const int h = blockIdx.y * kHeadsPerBlock + hl;
  const bool h_ok = h < a.Hq;
  const int d4 = (int)threadIdx.x % kThreadsPerHead;
  const float2* ml = reinterpret_cast<const float2*>(w.part_ml);
  const float4* pa = reinterpret_cast<const float4*>(w.part_acc);

  float m_run = -INFINITY, l_run = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p0 = 0; p0 < np; p0 += kMergeChunk) {
    const int n = min(kMergeChunk, np - p0);
    __syncthreads();
    for (int i = (int)threadIdx.x; i < kHeadsPerBlock * n; i += 256) {
      const int hh = i / n, p = i - hh * n;
      const int hq = blockIdx.y * kHeadsPerBlock + hh;
      float2 v = make_float2(-INFINITY, 0.f);
      if (hq < a.Hq) v = ml[(int64_t)(item0 + p0 + p) * a.Hq + hq];
      s_m[hh][p] = v.x;
      s_l[hh][p] = v.y;
    }
    __syncthreads();
    float m_new = m_run;
    for (int p = 0; p < n; ++p) m_new = fmaxf(m_new, s_m[hl][p]);
    const float c_old = exp2f(m_run - m_new);            // 0 on the first chunk (m_run = -inf)
    l_run *= c_old;
    acc.x *= c_old; acc.y *= c_old; acc.z *= c_old; acc.w *= c_old;
    m_run = m_new;
    if (h_ok) {
      int p = 0;
      for (; p + 4 <= n; p += 4) {
        float4 x[4];
        float sc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          x[u] = pa[((int64_t)(item0 + p0 + p + u) * a.Hq + h) * kThreadsPerHead + d4];
          sc[u] = exp2f(s_m[hl][p + u] - m_run);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          l_run += s_l[hl][p + u] * sc[u];
          acc.x += x[u].x * sc[u]; acc.y += x[u].y * sc[u]; acc.z += x[u].z * sc[u]; acc.w += x[u].w * sc[u];
        }
      }
      for (; p < n; ++p) {
        const float4 x = pa[((int64_t)(item0 + p0 + p) * a.Hq + h) * kThreadsPerHead + d4];
        const float sc = exp2f(s_m[hl][p] - m_run);
        l_run += s_l[hl][p] * sc;
        acc.x += x.x * sc; acc.y += x.y * sc; acc.z += x.z * sc; acc.w += x.w * sc;
      }
    }
  }
  if (!h_ok) return;
  const float inv = a.out_scale / l_run;
  acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
  const int64_t o = ((int64_t)qtok * a.Hq + h) * D + d4 * 4;
  if (a.out_bf16) {
    ushort4 ob;
    ob.x = f32_to_bf16_rne(acc.x); ob.y = f32_to_bf16_rne(acc.y);
    ob.z = f32_to_bf16_rne(acc.z); ob.w = f32_to_bf16_rne(acc.w);
    *reinterpret_cast<ushort4*>(reinterpret_cast<uint16_t*>(a.out) + o) = ob;
  } else {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out) + o) = acc;
  }
}


// ---- bf16 staging of 8-bit contexts ----------------------------------------------------------
// With a cache of E4M3 codes the MFMA kernel does not widen K/V itself: every K/V tile is read
// by many query tiles, so the contexts of the segments it serves are widened once, here, into a
// private run of bf16 blocks with a block table of its own, and the MFMA kernel runs on that
// copy unchanged.  The copy is exact (every E4M3 value is a bf16 value); the dequantisation
// scales are applied to the scores and to the normalised output instead.
// One workgroup per (block of a staged context): reads 16 bytes of codes per thread and writes
// 32 bytes of bf16, K then V.
__global__ __launch_bounds__(256) void stage_kernel(AttnArgs a, WorkLists w, int32_t table_stride) {
  const int s = blockIdx.y, b = blockIdx.x;
  const int seq = w.stage_seq[s];
  const int nblk = (a.ctx_lens[seq] + kBlockSize - 1) / kBlockSize;
  if (b >= nblk) return;                                   // uniform for the workgroup
  const int64_t src = a.block_tables[(int64_t)seq * a.max_blocks + b];
  const int64_t dst = w.stage_blk0[s] + b;
  if (threadIdx.x == 0) w.stage_table[(int64_t)s * table_stride + b] = (int32_t)dst;
  const int units = a.Hkv * a.D;                           // 16-byte units of codes per block and tensor
  const int64_t blk_elems = (int64_t)kBlockSize * a.Hkv * a.D;
#pragma unroll
  for (int kv = 0; kv < 2; ++kv) {
    const uint4* in = reinterpret_cast<const uint4*>(
        reinterpret_cast<const unsigned char*>(kv ? a.v_pool : a.k_pool) + src * blk_elems);
    uint4* outp = reinterpret_cast<uint4*>((kv ? w.stage_v : w.stage_k) + dst * blk_elems);
    for (int u = (int)threadIdx.x; u < units; u += 256) {
      const uint4 c = in[u];
      const uint32_t cw[4] = {c.x, c.y, c.z, c.w};
      uint32_t r[8];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        r[2 * k] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)cw[k], 1.0f, false));
        r[2 * k + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)cw[k], 1.0f, true));
      }
      outp[2 * u] = make_uint4(r[0], r[1], r[2], r[3]);
      outp[2 * u + 1] = make_uint4(r[4], r[5], r[6], r[7]);
    }
  }
}

}  // namespace

int launch_stage(const AttnArgs& a, const WorkLists& w, const PlanCounts& n, hipStream_t stream) {
  if (!a.kv8 || n.tiles == 0) return DSV_OK;
  dim3 grid((unsigned)n.stage_max_blocks, (unsigned)n.stage_segs);
  if (n.stage_segs > 65535) return DSV_E_UNSUPPORTED;
  hipLaunchKernelGGL(stage_kernel, grid, dim3(256), 0, stream, a, w, n.stage_max_blocks);
  return launch_status();
}

int launch_merge(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg, const PlanCounts& n,
                 hipStream_t stream) {
  const unsigned gy = (unsigned)ceil_div(a.Hq, a.D == 128 ? 8 : 16);
  if (n.split_items) {
    dim3 grid((unsigned)n.rows, gy);
    if (a.D == 128) hipLaunchKernelGGL((merge_kernel<128, false>), grid, dim3(256), 0, stream, a, w, cfg.tile_tokens);
    else hipLaunchKernelGGL((merge_kernel<64, false>), grid, dim3(256), 0, stream, a, w, cfg.tile_tokens);
    if (launch_status()) return DSV_E_LAUNCH;
  }
  if (n.split_qtiles) {
    if (n.split_qtiles * 64 > 0x7fffffffLL) return DSV_E_UNSUPPORTED;
    dim3 grid((unsigned)(n.split_qtiles * 64), gy);
    if (a.D == 128) hipLaunchKernelGGL((merge_kernel<128, true>), grid, dim3(256), 0, stream, a, w, cfg.tile_tokens);
    else hipLaunchKernelGGL((merge_kernel<64, true>), grid, dim3(256), 0, stream, a, w, cfg.tile_tokens);
    if (launch_status()) return DSV_E_LAUNCH;
  }
  return DSV_OK;
}

}  // namespace dsv

using namespace dsv;

namespace {

size_t workspace_bytes_for(bool kv8, int32_t num_seqs, const int32_t* q_offsets_host,
                           const int32_t* ctx_lens_host, int32_t num_q_heads, int32_t num_kv_heads,
                           int32_t head_dim) {
  if (num_q_heads < 1 || num_kv_heads < 1 || num_q_heads % num_kv_heads) return 0;
  if (head_dim != 64 && head_dim != 128) return 0;
  if (validate_batch(num_seqs, q_offsets_host, ctx_lens_host, -1) != DSV_OK) return 0;
  const PlanConfig c = choose_plan(num_seqs, q_offsets_host, ctx_lens_host, kv8, num_kv_heads,
                                   num_q_heads / num_kv_heads);
  const PlanCounts n = count_plan(num_seqs, q_offsets_host, ctx_lens_host, c);
  return carve(n, num_seqs, num_q_heads, num_kv_heads, head_dim, kv8, nullptr, nullptr);
}

// What a call does: the whole step, the work lists only, or the step on lists a plan call left
// in the workspace (one plan per batch serves every layer of the model).
enum class Phase { kPlanAndRun, kPlanOnly, kRunPlanned };

// Host-side record of a plan call, kept in the caller's dsv_attn_plan: everything the lists in
// the workspace depend on, so that a planned call made with anything else is refused.
struct PlanStamp {
  uint64_t magic, lists_hash;
  const void *workspace, *block_tables, *q_offsets, *ctx_lens;
  int32_t num_seqs, Hq, Hkv, D, kv8, max_blocks;
  int32_t part_tokens, mfma_min_qlen, mfma_min_work, tile_tokens, tile_part_tiles, num_cus;
  int32_t flat_heads, head_groups;
  int32_t stream_wgs, stream_row_cost;
  int64_t stream_total;
};
static_assert(sizeof(PlanStamp) <= sizeof(dsv_attn_plan), "dsv_attn_plan too small");
constexpr uint64_t kPlanMagic = 0x6473765f706c616eull;

uint64_t hash_lists(const int32_t* qo, const int32_t* cl, int32_t S) {
  uint64_t h = 0xcbf29ce484222325ull;                            // FNV-1a over both arrays
  auto mix = [&](uint32_t v) { h = (h ^ v) * 0x100000001b3ull; };
  for (int i = 0; i <= S; ++i) mix((uint32_t)qo[i]);
  for (int i = 0; i < S; ++i) mix((uint32_t)cl[i]);
  return h;
}

PlanStamp make_stamp(const PlanConfig& c, bool kv8, const void* workspace, const int32_t* block_tables,
                     int32_t max_blocks, const int32_t* q_offsets, const int32_t* ctx_lens,
                     const int32_t* qo_host, const int32_t* cl_host, int32_t S, int32_t Hq, int32_t Hkv,
                     int32_t D) {
  PlanStamp st;
  memset(&st, 0, sizeof st);
  st.magic = kPlanMagic;
  st.lists_hash = hash_lists(qo_host, cl_host, S);
  st.workspace = workspace; st.block_tables = block_tables; st.q_offsets = q_offsets; st.ctx_lens = ctx_lens;
  st.num_seqs = S; st.Hq = Hq; st.Hkv = Hkv; st.D = D; st.kv8 = kv8 ? 1 : 0; st.max_blocks = max_blocks;
  st.part_tokens = c.part_tokens; st.mfma_min_qlen = c.mfma_min_qlen; st.mfma_min_work = c.mfma_min_work;
  st.flat_heads = c.flat_heads; st.head_groups = c.head_groups;
  st.tile_tokens = c.tile_tokens; st.tile_part_tiles = c.tile_part_tiles; st.num_cus = c.num_cus;
  st.stream_wgs = c.stream_wgs; st.stream_row_cost = c.stream_row_cost; st.stream_total = c.stream_total;
  return st;
}

// All attention entry points.  kv8: the pool holds E4M3 codes (one byte per element) with the two
// dequantisation scales; otherwise bf16 and both scales are 1.  In a plan-only call q, out and the
// pool's base pointers are not looked at.
int run_attention(Phase phase, dsv_attn_plan* plan, bool kv8, float k_scale, float v_scale, const void* q, void* out,
                  const dsv_kv_pool* pool, int32_t layer, const int32_t* block_tables,
                  int32_t max_blocks_per_seq, const int32_t* q_offsets, const int32_t* ctx_lens,
                  const int32_t* q_offsets_host, const int32_t* ctx_lens_host, int32_t num_seqs,
                  int32_t num_q_heads, float softmax_scale, int32_t out_dtype, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
  int rc = check_pool(pool);
  if (rc) return rc;
  if (num_seqs < 0) return DSV_E_INVALID;
  if (phase != Phase::kPlanAndRun && !plan) return DSV_E_INVALID;
  if (num_seqs == 0) {
    if (phase == Phase::kPlanOnly) memset(plan, 0, sizeof *plan);    // no lists: a planned call of
    return DSV_OK;                                                 // an empty batch does nothing either
  }
  const bool data = phase != Phase::kPlanOnly;
  if ((data && (!q || !out)) || !block_tables || !q_offsets || !ctx_lens || !workspace) return DSV_E_INVALID;
  if (layer < 0 || layer >= pool->num_layers || max_blocks_per_seq < 1) return DSV_E_INVALID;
  if (num_q_heads < 1 || num_q_heads % pool->num_kv_heads) return DSV_E_INVALID;
  if (out_dtype != DSV_OUT_F32 && out_dtype != DSV_OUT_BF16) return DSV_E_INVALID;
  if (!(softmax_scale >= 0.0f) || isinf(softmax_scale)) return DSV_E_INVALID;
  if (!(k_scale > 0.0f) || isinf(k_scale) || !(v_scale > 0.0f) || isinf(v_scale)) return DSV_E_INVALID;
  if (data && ((reinterpret_cast<uintptr_t>(q) & 15) || (reinterpret_cast<uintptr_t>(out) & 15) ||
               (reinterpret_cast<uintptr_t>(pool->k_base) & 15) || (reinterpret_cast<uintptr_t>(pool->v_base) & 15)))
    return DSV_E_INVALID;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return DSV_E_INVALID;
  const int elem_bytes = kv8 ? 1 : 2;
  if (pool->num_layers > 1 && (pool->layer_stride * elem_bytes % 16)) return DSV_E_INVALID;
  rc = validate_batch(num_seqs, q_offsets_host, ctx_lens_host, max_blocks_per_seq);
  if (rc) return rc;

  const PlanConfig cfg = choose_plan(num_seqs, q_offsets_host, ctx_lens_host, kv8, pool->num_kv_heads,
                                     num_q_heads / pool->num_kv_heads);
  const PlanCounts n = count_plan(num_seqs, q_offsets_host, ctx_lens_host, cfg);
  if (n.items > 0x7fffffffLL || n.tiles > 0x7fffffffLL || n.rows > 0x7fffffffLL ||
      n.max_parts > 0x7fff || n.stage_blocks > 0x7fffffffLL ||
      n.items + n.tile_split_items > 0x7fffffffLL)
    return DSV_E_UNSUPPORTED;
  WorkLists w;
  const size_t need = carve(n, num_seqs, num_q_heads, pool->num_kv_heads, pool->head_dim, kv8,
                            static_cast<char*>(workspace), &w);
  if (workspace_bytes < need) return DSV_E_WORKSPACE;
  const PlanStamp stamp = make_stamp(cfg, kv8, workspace, block_tables, max_blocks_per_seq, q_offsets, ctx_lens,
                                     q_offsets_host, ctx_lens_host, num_seqs, num_q_heads,
                                     pool->num_kv_heads, pool->head_dim);
  if (phase == Phase::kRunPlanned) {
    // The lists in the workspace are only as good as the plan call that wrote them: same batch
    // arrays (host copies by content, device arrays by address), same geometry, same knobs.
    PlanStamp made;
    memcpy(&made, plan, sizeof made);
    if (memcmp(&made, &stamp, sizeof stamp) != 0) return DSV_E_INVALID;
  }

  AttnArgs a;
  const int64_t layer_off = pool->num_layers > 1 ? (int64_t)layer * pool->layer_stride * elem_bytes : 0;
  a.q = static_cast<const uint16_t*>(q);
  a.out = out;
  a.k_pool = reinterpret_cast<const uint16_t*>(static_cast<const unsigned char*>(pool->k_base) + layer_off);
  a.v_pool = reinterpret_cast<const uint16_t*>(static_cast<const unsigned char*>(pool->v_base) + layer_off);
  a.block_tables = block_tables;
  a.q_offsets = q_offsets;
  a.ctx_lens = ctx_lens;
  a.max_blocks = max_blocks_per_seq;
  a.num_seqs = num_seqs;
  a.Hq = num_q_heads;
  a.Hkv = pool->num_kv_heads;
  a.D = pool->head_dim;
  a.scale_log2e = kv8 ? softmax_scale * k_scale * 1.4426950408889634f : softmax_scale * 1.4426950408889634f;
  // A scale of exactly zero (uniform weights) would turn masked scores, -inf, into NaN when it
  // multiplies them; a scale too small to move any finite score does the same job.
  if (a.scale_log2e == 0.0f) a.scale_log2e = 1e-30f;
  a.out_bf16 = out_dtype == DSV_OUT_BF16;
  a.out_scale = kv8 ? v_scale : 1.0f;
  a.kv8 = kv8 ? 1 : 0;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  begin_gpu_work();
  const bool stage = kv8 && n.tiles > 0;
  if (phase != Phase::kRunPlanned) {
    EventScope ev(DSV_KERNEL_PLAN, stream);
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, stream, q_offsets, ctx_lens,
                       block_tables, max_blocks_per_seq, num_seqs, cfg, w, tile_list_mode(n),
                       stage ? 1 : 0, (int32_t)n.items);
    if ((rc = launch_status())) return rc;
  }
  if (phase == Phase::kPlanOnly) {
    memset(plan, 0, sizeof *plan);
    memcpy(plan, &stamp, sizeof stamp);
    return DSV_OK;
  }
  if (stage) {
    EventScope ev(DSV_KERNEL_STAGE, stream);
    if ((rc = launch_stage(a, w, n, stream))) return rc;
  }
  // A batch with both prefill tiles and row items runs them in one launch: some compute units
  // stream KV for the rows while the others run the spans' MFMAs, and one launch gap goes.
  // Measured over the batch shapes a local scheduler emits (one span of 64-4,096 tokens, 4-256
  // decodes on 1,024 or 8,192 tokens, 32/8 heads): up to 20 % faster than the two kernels one
  // after the other where one side is small (a 512-token span with 16 decodes: 67 -> 55 us), 14 %
  // on config 4, 3 % on config 3, never more than 1 % slower.  DSV_MIXED_LAUNCH=0 keeps them apart.
  bool mix = mixed_launch_supported(a, cfg, n);
  if (mix && env_int("DSV_MIXED_LAUNCH", 1) == 0) mix = false;
  if (mix) {
    EventScope ev(DSV_KERNEL_MIXED, stream);
    if ((rc = launch_mixed(a, w, cfg, n, stream))) return rc;
  } else {
    if (n.tiles) {
      EventScope ev(DSV_KERNEL_TILES, stream);
      if ((rc = launch_prefill_tiles(a, w, cfg, n, stream))) return rc;
    }
    if (n.items) {
      EventScope ev(DSV_KERNEL_ROWS, stream);
      if ((rc = launch_rows(a, w, cfg, n, stream))) return rc;
    }
  }
  if (n.split_items || n.split_qtiles) {
    EventScope ev(DSV_KERNEL_MERGE, stream);
    if ((rc = launch_merge(a, w, cfg, n, stream))) return rc;
  }
  return DSV_OK;
}

}  // namespace

extern "C" size_t attn_mixed_batch_workspace_bytes(int32_t num_seqs, const int32_t* q_offsets_host,
                                                   const int32_t* ctx_lens_host, int32_t num_q_heads,
                                                   int32_t num_kv_heads, int32_t head_dim) {
  return workspace_bytes_for(false, num_seqs, q_offsets_host, ctx_lens_host, num_q_heads,
                             num_kv_heads, head_dim);
}

extern "C" int attn_mixed_batch_plan_info(int32_t num_seqs, const int32_t* q_offsets_host,
                                          const int32_t* ctx_lens_host, int32_t num_q_heads,
                                          int32_t num_kv_heads, int32_t head_dim, int32_t kv_elem_bytes,
                                          int32_t* info) {
  if (!info || num_q_heads < 1 || num_kv_heads < 1 || num_q_heads % num_kv_heads) return DSV_E_INVALID;
  if (head_dim != 64 && head_dim != 128) return DSV_E_UNSUPPORTED;
  if (kv_elem_bytes != 1 && kv_elem_bytes != 2) return DSV_E_INVALID;
  const int rc = validate_batch(num_seqs, q_offsets_host, ctx_lens_host, -1);
  if (rc) return rc;
  for (int k = 0; k < 8; ++k) info[k] = 0;
  if (num_seqs == 0) return DSV_OK;
  const PlanConfig c = choose_plan(num_seqs, q_offsets_host, ctx_lens_host, kv_elem_bytes == 1, num_kv_heads,
                                   num_q_heads / num_kv_heads);
  const PlanCounts n = count_plan(num_seqs, q_offsets_host, ctx_lens_host, c);
  auto clip = [](int64_t v) { return (int32_t)(v > 0x7fffffffLL ? 0x7fffffffLL : v); };
  info[0] = c.stream_wgs;
  info[1] = c.stream_wgs > 0 ? 0 : c.part_tokens;
  info[2] = clip(n.rows);
  info[3] = clip(n.items);
  info[4] = clip(n.tiles);
  info[5] = c.tile_part_tiles;
  info[6] = (n.tiles > 0 && n.items > 0 && env_int("DSV_MIXED_LAUNCH", 1) != 0) ? 1 : 0;
  info[7] = c.tile_tokens;
  return DSV_OK;
}

extern "C" size_t attn_mixed_batch_fp8kv_workspace_bytes(int32_t num_seqs, const int32_t* q_offsets_host,
                                                         const int32_t* ctx_lens_host,
                                                         int32_t num_q_heads, int32_t num_kv_heads,
                                                         int32_t head_dim) {
  return workspace_bytes_for(true, num_seqs, q_offsets_host, ctx_lens_host, num_q_heads,
                             num_kv_heads, head_dim);
}

extern "C" int attn_mixed_batch(const void* q, void* out, const dsv_kv_pool* pool, int32_t layer,
                                const int32_t* block_tables, int32_t max_blocks_per_seq,
                                const int32_t* q_offsets, const int32_t* ctx_lens,
                                const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                                int32_t num_seqs, int32_t num_q_heads, float softmax_scale,
                                int32_t out_dtype, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
  return run_attention(Phase::kPlanAndRun, nullptr, false, 1.0f, 1.0f, q, out, pool, layer, block_tables,
                       max_blocks_per_seq, q_offsets, ctx_lens, q_offsets_host, ctx_lens_host, num_seqs,
                       num_q_heads, softmax_scale, out_dtype, workspace, workspace_bytes, hip_stream);
}

extern "C" int attn_mixed_batch_fp8kv(const void* q, void* out, const dsv_kv_pool* pool, int32_t layer,
                                      const int32_t* block_tables, int32_t max_blocks_per_seq,
                                      const int32_t* q_offsets, const int32_t* ctx_lens,
                                      const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                                      int32_t num_seqs, int32_t num_q_heads, float softmax_scale,
                                      float k_scale, float v_scale, int32_t out_dtype,
                                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  return run_attention(Phase::kPlanAndRun, nullptr, true, k_scale, v_scale, q, out, pool, layer, block_tables,
                       max_blocks_per_seq, q_offsets, ctx_lens, q_offsets_host, ctx_lens_host,
                       num_seqs, num_q_heads, softmax_scale, out_dtype, workspace, workspace_bytes,
                       hip_stream);
}

extern "C" int attn_mixed_batch_plan(dsv_attn_plan* plan, const int32_t* block_tables,
                                     int32_t max_blocks_per_seq, const int32_t* q_offsets,
                                     const int32_t* ctx_lens, const int32_t* q_offsets_host,
                                     const int32_t* ctx_lens_host, int32_t num_seqs,
                                     int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                                     int32_t kv_elem_bytes, void* workspace, size_t workspace_bytes,
                                     void* hip_stream) {
  if (kv_elem_bytes != 1 && kv_elem_bytes != 2) return DSV_E_INVALID;
  // Geometry only: the plan does not touch K/V (the base pointers below are never dereferenced).
  dsv_kv_pool geo;
  geo.k_base = &geo; geo.v_base = &geo;
  geo.layer_stride = 0; geo.num_layers = 1; geo.num_blocks = 1; geo.block_size = kBlockSize;
  geo.num_kv_heads = num_kv_heads; geo.head_dim = head_dim;
  return run_attention(Phase::kPlanOnly, plan, kv_elem_bytes == 1, 1.0f, 1.0f, nullptr, nullptr, &geo, 0,
                       block_tables, max_blocks_per_seq, q_offsets, ctx_lens, q_offsets_host,
                       ctx_lens_host, num_seqs, num_q_heads, 1.0f, DSV_OUT_BF16, workspace,
                       workspace_bytes, hip_stream);
}

extern "C" int attn_mixed_batch_planned(const dsv_attn_plan* plan, const void* q, void* out,
                                        const dsv_kv_pool* pool, int32_t layer,
                                        const int32_t* block_tables, int32_t max_blocks_per_seq,
                                        const int32_t* q_offsets, const int32_t* ctx_lens,
                                        const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                                        int32_t num_seqs, int32_t num_q_heads, float softmax_scale,
                                        int32_t out_dtype, void* workspace, size_t workspace_bytes,
                                        void* hip_stream) {
  return run_attention(Phase::kRunPlanned, const_cast<dsv_attn_plan*>(plan), false, 1.0f, 1.0f, q, out, pool,
                       layer, block_tables, max_blocks_per_seq, q_offsets, ctx_lens, q_offsets_host,
                       ctx_lens_host, num_seqs, num_q_heads, softmax_scale, out_dtype, workspace,
                       workspace_bytes, hip_stream);
}

extern "C" int attn_mixed_batch_fp8kv_planned(const dsv_attn_plan* plan, const void* q, void* out,
                                              const dsv_kv_pool* pool, int32_t layer,
                                              const int32_t* block_tables, int32_t max_blocks_per_seq,
                                              const int32_t* q_offsets, const int32_t* ctx_lens,
                                              const int32_t* q_offsets_host,
                                              const int32_t* ctx_lens_host, int32_t num_seqs,
                                              int32_t num_q_heads, float softmax_scale, float k_scale,
                                              float v_scale, int32_t out_dtype, void* workspace,
                                              size_t workspace_bytes, void* hip_stream) {
  return run_attention(Phase::kRunPlanned, const_cast<dsv_attn_plan*>(plan), true, k_scale, v_scale, q, out,
                       pool, layer, block_tables, max_blocks_per_seq, q_offsets, ctx_lens,
                       q_offsets_host, ctx_lens_host, num_seqs, num_q_heads, softmax_scale, out_dtype,
                       workspace, workspace_bytes, hip_stream);
}

// ---- the entry point that allocates nothing --------------------------------------------------
// attn_mixed_batch for callers that cannot bring a workspace: the work lists and split-context
// partials live in a fixed array in device memory that belongs to the library.  Each device the
// library's code object is loaded on holds its own copy of the array at its own address; in host
// code the array's name is only a handle for hipGetSymbolAddress, never a device pointer.
namespace {

constexpr size_t kStaticScratchBytes = (size_t)DSV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];      // device address of `scratch`, per device

// Device address of the scratch array on the current device (looked up once per device).
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return DSV_E_LAUNCH; }
  if (dev < 0 || dev >= kMaxDevices) return DSV_E_UNSUPPORTED;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return DSV_E_LAUNCH;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread finds the same address
  }
  *out = p;
  return DSV_OK;
}

}  // namespace

extern "C" size_t attn_mixed_batch_static_max_bytes(void) { return kStaticScratchBytes; }

extern "C" int attn_mixed_batch_static(const void* q, void* out, const dsv_kv_pool* pool, int32_t layer,
                                       const int32_t* block_tables, int32_t max_blocks_per_seq,
                                       const int32_t* q_offsets, const int32_t* ctx_lens,
                                       const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                                       int32_t num_seqs, int32_t num_q_heads, float softmax_scale,
                                       int32_t out_dtype, void* hip_stream) {
  int rc = check_pool(pool);
  if (rc) return rc;
  if (num_seqs < 0) return DSV_E_INVALID;
  if (num_seqs == 0) return DSV_OK;
  if (num_q_heads < 1 || num_q_heads % pool->num_kv_heads) return DSV_E_INVALID;
  // The batch must fit the fixed array: refused here, before anything is enqueued.
  const size_t need = workspace_bytes_for(false, num_seqs, q_offsets_host, ctx_lens_host, num_q_heads,
                                          pool->num_kv_heads, pool->head_dim);
  if (need == 0) return DSV_E_INVALID;
  if (need > kStaticScratchBytes) return DSV_E_WORKSPACE;
  void* ptr = nullptr;
  if ((rc = static_scratch(&ptr))) return rc;
  // Nothing in the array has to start at zero: the plan kernel writes every list, the zero line
  // included, and the attention kernels write every partial the merge kernel reads.
  return run_attention(Phase::kPlanAndRun, nullptr, false, 1.0f, 1.0f, q, out, pool, layer, block_tables,
                       max_blocks_per_seq, q_offsets, ctx_lens, q_offsets_host, ctx_lens_host, num_seqs,
                       num_q_heads, softmax_scale, out_dtype, ptr, kStaticScratchBytes, hip_stream);
}

extern "C" int dsv_profile_events(int32_t kernel_id, void* start_event, void* stop_event) {
  if (kernel_id < 0 || kernel_id > 5) return DSV_E_INVALID;
  g_events[kernel_id][0] = static_cast<hipEvent_t>(start_event);
  g_events[kernel_id][1] = static_cast<hipEvent_t>(stop_event);
  return DSV_OK;
}

extern "C" const char* dsv_build_info(void) { return "dsv_attn gfx950 " __DATE__ " " __TIME__; }
