// Attention of long prefill spans on the matrix cores, persistent form, built on the 16x16x32 MFMA.
//
// Who runs what - persistent workgroups, the stream of ring positions, requests that run three
// tiles ahead and across item boundaries, the order of the items - is attn_prefill_persistent.h's
// (read that header first; paper sections 2.1, 3.1, 4.2 for what is computed).  What differs is
// the shape of the products: S^T = K Q^T and O^T = V^T P^T are made of 16x16x32 MFMAs, which on
// operands like these cost about a tenth less energy per flop than the 32x32x16 ones, and this
// kernel runs at the board's power limit.
//
// A wave still owns 32 query rows of one head, now as two 16-row blocks of MFMA columns (qt = 0, 1):
// lane l holds query rows 16*qt + l%16 and, of every 16-token group, the tokens 4*(l/16) .. +3.
//   - K fragment (A operand, 16 tokens x 32 dims): lane (token l%16, dims 8*(l/16) .. +7 of the
//     k-step), one ds_read_b128; each is used for both query blocks.
//   - Q fragment (B operand): lane (row l%16 of the block, the same dims), in registers.
//   - S^T block (16 tokens x 16 rows): lane (row l%16, tokens 4*(l/16) + r).  The two blocks of a
//     32-token sub-tile give a lane 8 values per query block, which are, in that order, the B
//     operand of O^T += V^T P^T once V^T enumerates the tokens alike: 4g..4g+3 of the first 16
//     tokens, then of the second 16 (g = l/16).
//   - V^T fragment (A operand, 16 dims x 32 tokens): two transpose reads (one per 16 tokens),
//     each used for both query blocks.
//   - O^T block (16 dims x 16 rows): lane (row l%16, dims 4*(l/16) + r).
// Row sums are kept per lane over the lane's own tokens and added up over the four lane groups
// at the end; the row maximum (first sub-tile, robust pass) is taken over the four groups.
#pragma once
#include "attn_prefill_persistent.h"

namespace dsv {
namespace prefill_impl {

// Row swizzle of the V tile for this form's transpose reads (8 token rows x 32 bytes per half
// wave: rows that differ in their low three bits must sit in different 32-byte groups).
template <int CPR> __device__ __forceinline__ int v_swz16(int row) { return 2 * (row & (CPR / 2 - 1)); }

template <int D>
__device__ __forceinline__ void prefill_tiles_persistent16(const TilesParams& prm, params_ptr prm_mem, int wg,
                                                         int num_wgs, unsigned char* smem) {
  using Geo = TileGeom<D>;
  constexpr int ROWB = Geo::ROWB, CPR = Geo::CPR, RPP = Geo::RPP, PPW = Geo::PPW;
  constexpr int KS = D / 32;             // k-steps of K Q^T
  constexpr int DT = D / 16;             // 16-dim blocks of O^T
  constexpr int QT = 2;                  // 16-row query blocks per wave
  static_assert(NH == 1 && (KS == 4 || KS == 2) && DT % 4 == 0, "fragment reads are issued in groups of four");
  static_assert(kRing == 4 && (Geo::TILE_BYTES & (Geo::TILE_BYTES - 1)) == 0, "XOR stepping of the ring");
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  using i0 = std::integral_constant<int, 0>;
  using i1 = std::integral_constant<int, 1>;

  const AttnArgs& a = prm.a;
  auto P = [&]() __attribute__((always_inline)) -> params_ptr {
    params_ptr p = prm_mem;
    asm volatile("" : "+s"(p));
    return p;
  };
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
  // The lane index, made afresh wherever the code between two items needs it (and what derives
  // from it: row lane % 16 of a 16-row query block, lane group lane / 16), so that none
  // of it occupies a vector register across the tile loop, which has none to spare.
  auto lane_id = [&]() __attribute__((always_inline)) -> int {
    int l = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(l));        // opaque: what derives from it is computed where it is used
    return l;
  };
  const int lane = lane_id();
#define DSV_TID0_16 (wave == 0 && lane_id() == 0)

  const int kvh = wg % a.Hkv;
  const int wgs_per_head = num_wgs / a.Hkv;                     // the grid is a multiple of Hkv
  const int rank = wg / a.Hkv;                                  // this workgroup among those of its head
  const int items = prm.num_tiles * prm.head_groups;            // per KV head
  const int G = prm.G;
  const float scale = a.scale_log2e;
  // List position of this workgroup's k-th item (>= items: there is none).
  auto item_of_round = [&](int k) __attribute__((always_inline)) -> int {
    return k * wgs_per_head + ((k & 1) ? wgs_per_head - 1 - rank : rank);
  };

  // ---- fixed for the workgroup: this wave's pieces of a tile request, fragment addresses ----
  const unsigned char* const zero_line = reinterpret_cast<const unsigned char*>(prm.w.zero_line);
  const uint32_t tok_stride = (uint32_t)a.Hkv * D;
  const int blk_in_tile = wave / kWavesPerBlock, half = wave % kWavesPerBlock;
  uint32_t k_src[PPW], v_src[PPW];
  int slot_n[PPW];
#pragma unroll
  for (int ii = 0; ii < PPW; ++ii) {
    const int n = (half * (PPW) + ii) * RPP + lane / CPR;
    const int row = blk_in_tile * kBlockSize + n;
    const int pos = lane % CPR;
    slot_n[ii] = n;
    k_src[ii] = ((uint32_t)n * tok_stride + (uint32_t)((pos ^ k_swz<CPR>(row)) * 8)) * 2u;
    v_src[ii] = ((uint32_t)n * tok_stride + (uint32_t)((pos ^ v_swz16<CPR>(row)) * 8)) * 2u;
  }
  const uint32_t zero_src = (uint32_t)(lane % CPR) * 16u;
  const unsigned char* const k_head = reinterpret_cast<const unsigned char*>(a.k_pool + (uint32_t)kvh * D);
  const unsigned char* const v_head = reinterpret_cast<const unsigned char*>(a.v_pool + (uint32_t)kvh * D);
  // ---- work items (everything here is uniform for the workgroup) ----
  struct Item {
    int j0, q0, q_len, ctx, prefix, nblk, t_first, n_tiles, pos0, part, nparts, first_partial, bz;
    const_i32_ptr table;
    int trailing;              // zero-line positions requested behind the item's last tile
  };
  auto load_item = [&](int r) __attribute__((always_inline)) -> Item {
    const params_ptr pp = P();
    const int head_groups = pp->head_groups;
    const int tile = __builtin_amdgcn_readfirstlane(r / head_groups);
    const const_i32_ptr rp = (const_i32_ptr)(uintptr_t)pp->w.tile_rec + 8 * (int64_t)tile;   // one 32-byte scalar read
    const ItemRec rec = {rp[0], rp[1], rp[2], rp[3], rp[4], rp[5], rp[6], rp[7]};
    Item it;
    it.bz = __builtin_amdgcn_readfirstlane(r - tile * head_groups);
    it.j0 = rec.j0; it.q0 = rec.q0; it.q_len = rec.q_len; it.ctx = rec.ctx;
    it.prefix = rec.ctx - rec.q_len;
    it.nblk = (rec.ctx + kBlockSize - 1) / kBlockSize;
    it.table = (const_i32_ptr)(uintptr_t)(pp->a.block_tables + (int64_t)rec.table_row * pp->a.max_blocks);
    const int kv_end = min(rec.ctx, it.prefix + rec.j0 + pp->tile_q);
    const int n_kv = (kv_end + kTileKV - 1) / kTileKV;
    it.part = rec.part_rec & 0xffff;
    it.nparts = rec.part_rec >> 16;
    const int base_kv = n_kv / it.nparts, rem_kv = n_kv - base_kv * it.nparts;
    it.t_first = it.part * base_kv + min(it.part, rem_kv);
    it.n_tiles = base_kv + (it.part < rem_kv ? 1 : 0);
    it.pos0 = it.t_first * kTileKV;
    it.first_partial = rec.first_partial;
    it.trailing = 0;
    return it;
  };

  // ---- the request side of the tile stream ----
  // A cursor names a tile: `which` 0 = of the current item, 1 = of the next item, 2 = none (the
  // request fetches the zero line).  A tile's block id is read from the table (scalar load) one
  // request before the tile itself is requested, so two cursors walk the same sequence one step
  // apart: `req` (its block id is on its way) and `ahead` (the tile after it).
  Item cur, nxt;
  bool has_nxt = false;
  int item_round = 0;                  // how many items this workgroup has finished
  int req_which = 2, req_t = 0, ahead_which = 2, ahead_t = 0;
  int req_bid = 0;
  int pos_req = 0;                     // ring position the next request fills
  int pos_use = 0;                     // ring position of the tile the computing side takes next
  int ahead = 0;                       // positions requested and not yet taken
  // (Selects, no branches: a tile step must stay one basic block, so that its MFMAs and the
  // softmax of the same step can be interleaved by the scheduler.)
  auto advance = [&](int& which, int& t) __attribute__((always_inline)) {
    const int n = which == 1 ? nxt.n_tiles : cur.n_tiles;
    const bool last = which != 2 && t + 1 >= n;
    const int after = (which == 0 && has_nxt) ? 1 : 2;
    t = (which == 2 || last) ? 0 : t + 1;
    which = last ? after : which;
  };
  auto block_id_of = [&](int which, int t) __attribute__((always_inline)) -> int {
    const bool second = which == 1;
    const int t_first = second ? nxt.t_first : cur.t_first;
    const int nblk = second ? nxt.nblk : cur.nblk;
    const const_i32_ptr tbl = second ? nxt.table : cur.table;
    const int b = (t_first + (which == 2 ? 0 : t)) * (kTileKV / kBlockSize) + blk_in_tile;
    return tbl[min(b, nblk - 1)];      // clamped into the row; used only if the block exists
  };
  // Point the cursors at tile 0 of the current item, or of the next one.
  auto prime = [&](bool from_cur) __attribute__((always_inline)) {
    req_which = from_cur ? 0 : (has_nxt ? 1 : 2);
    req_t = 0;
    req_bid = block_id_of(req_which, req_t);
    ahead_which = req_which; ahead_t = req_t;
    advance(ahead_which, ahead_t);
  };
  // One request: the tile under `req` (or the zero line) goes to ring position pos_req, the block
  // id of the tile after it is asked for, both cursors step.  Every request is the same number of
  // loads, so that a count of loads in flight tells which requests have landed.
  auto request = [&]() __attribute__((always_inline)) {
    const bool second = req_which == 1;
    const int t_first = second ? nxt.t_first : cur.t_first;
    const int nblk = second ? nxt.nblk : cur.nblk;
    const int ctx = second ? nxt.ctx : cur.ctx;
    const int b = (t_first + req_t) * (kTileKV / kBlockSize) + blk_in_tile;
    unsigned char* kdst = smem + (pos_req & (kRing - 1)) * Geo::TILE_BYTES + blk_in_tile * (kBlockSize * ROWB) +
                          half * (PPW) * 1024;
    unsigned char* vdst = kdst + Geo::TENSOR_BYTES;
    // Past the table every lane reads the zero line.  In a block that straddles ctx, K may hold
    // anything (its columns are masked) but V rows that must not be read come from the zero line.
    const bool have = req_which != 2 && b < nblk;
    const int64_t blk_bytes = (int64_t)req_bid * kBlockSize * tok_stride * 2;
    const unsigned char* kb = k_head + blk_bytes;
    const unsigned char* vb = v_head + blk_bytes;
    const int visible = ctx - b * kBlockSize;
#pragma unroll
    for (int ii = 0; ii < PPW; ++ii) {
      const unsigned char* kp = have ? kb + k_src[ii] : zero_line + zero_src;
      const unsigned char* vp = (have && slot_n[ii] < visible) ? vb + v_src[ii] : zero_line + zero_src;
      __builtin_amdgcn_global_load_lds((gbl_void_t)kp, (lds_void_t)(kdst + ii * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gbl_void_t)vp, (lds_void_t)(vdst + ii * 1024), 16, 0, 0);
    }
    nxt.trailing += (req_which == 2 && has_nxt) ? 1 : 0;     // held back behind the next item's last tile
    ++pos_req;
    ++ahead;
    req_which = ahead_which; req_t = ahead_t;
    req_bid = block_id_of(ahead_which, ahead_t);
    advance(ahead_which, ahead_t);
  };

  // ---- per-item state of the computing side ----
  typedef __attribute__((ext_vector_type(4))) float f32x4_t;
  constexpr int KREADS = 2 * KS;         // K fragment reads of a sub-tile (two 16-token groups)
  constexpr int VREADS = DT;             // V^T fragment reads of half a sub-tile's dim blocks
  static_assert(KREADS <= 15 && VREADS <= 15, "the LDS read counter has four bits");
  f32x4_t o[QT][DT];
  float m_run[QT], l_run[QT];            // l_run: over the lane's own tokens
  f32x4_t scb[2][QT][2];                 // [buffer][query block][16-token group of the sub-tile]
  uint4 pfb[2][QT];                      // a sub-tile's probabilities, B operand of O^T += V^T P^T
  float corr[QT];
  bool any_corr = false;
  u32x4_t kf[2][KS];                     // K fragments of a sub-tile: [16-token group][k-step]
  u32x2_t vf[DT][2];                     // V^T fragments of a sub-tile: [dim block][16-token group]
  uint32_t k_adr[KS], v_adr[DT];
  uint4 qf[QT][KS];
  int p_j[QT] = {0, 0};       // the lane's query positions in the item's partition, minus 4 * (lane / 16)
  int mask_from = 0;          // (wave-uniform) sub-tiles reaching past this need the causal mask
  int prio_sel = 0;           // (wave-uniform) which of the two waves of a SIMD this one is
  int pos_item0 = 0;          // ring position of the item's first tile
  bool wave_has_rows = false;
  bool overflow = false;

  // Exchange with lane ^ 16 (see half_swap for lane ^ 32): max / sum over the four lane groups
  // that share a query row.
  auto pair16 = [](float x, float& lo, float& hi) __attribute__((always_inline)) {
    uint32_t a = __float_as_uint(x), b;
    asm("" : "=v"(b) : "0"(a));
    typedef unsigned int u32x2v __attribute__((ext_vector_type(2)));
    const u32x2v r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
    lo = __uint_as_float(r[0]);
    hi = __uint_as_float(r[1]);
  };
  auto groups_max = [&](float x) __attribute__((always_inline)) -> float {
    float lo, hi;
    pair16(x, lo, hi);
    return other_half_max(fmaxf(lo, hi));
  };
  auto groups_sum = [&](float x) __attribute__((always_inline)) -> float {
    float lo, hi;
    pair16(x, lo, hi);
    return other_half_sum(lo + hi);
  };

  // Query row `row` (0..31) of this wave in an item: its token (counted from the span's first new
  // token), its head, and whether it exists.  Wave-uniform extras: whether any of the wave's rows
  // exists, its first token, and which of the two waves of its SIMD it is.
  auto row_geometry = [&](const Item& it, int row, int& jq_o, int& head_o, bool& ok_o) __attribute__((always_inline)) {
    const params_ptr pp = P();
    const int gh = pp->flat_heads, tile_q = pp->tile_q, fmagic = pp->flat_magic;
    const bool flat = gh > 0;
    const bool few_heads = G - it.bz * 4 <= 2;
    const int tg = few_heads ? wave % 2 : wave / kHeadWaves;
    const int hp = few_heads ? wave / 2 : wave % kHeadWaves;
    const int r_item = 32 * wave + row;
    const int jq_flat = flat_div(r_item, fmagic);
    jq_o = flat ? it.j0 + jq_flat : it.j0 + 32 * tg + row;
    const int hsub = flat ? it.bz * gh + (r_item - jq_flat * gh) : it.bz * 4 + hp * NH;
    ok_o = hsub < G && jq_o < it.q_len && (!flat || r_item < tile_q * gh);
    head_o = kvh * G + (hsub < G ? hsub : 0);
  };
  auto wave_geometry = [&](const Item& it, bool& rows_o, int& first_tok_o, int& prio_o) __attribute__((always_inline)) {
    const params_ptr pp = P();
    const int gh = pp->flat_heads, tile_q = pp->tile_q, fmagic = pp->flat_magic;
    const bool flat = gh > 0;
    const bool few_heads = G - it.bz * 4 <= 2;
    const int tg = few_heads ? wave % 2 : wave / kHeadWaves;
    const int hp = few_heads ? wave / 2 : wave % kHeadWaves;
    first_tok_o = flat ? flat_div(32 * wave, fmagic) : 32 * tg;
    rows_o = flat ? (it.j0 + first_tok_o < it.q_len && 32 * wave < tile_q * gh)
                  : (it.j0 + 32 * tg < it.q_len && it.bz * 4 + hp * NH < G);
    prio_o = flat ? wave / 4 : tg;
  };
  // Query fragments of an item (B operand of S^T = K Q^T; lane (row l%16 of block qt, group g)
  // holds dims 32*ks + 8*g .. +8).  A row that does not exist reads the zero line instead: the
  // choice is made on the address, so nothing has to wait for the loads here.
  auto load_q = [&](const Item& it) __attribute__((always_inline)) {
    static_assert(D * 2 <= 256, "a query row fits the zero line");
    const int ln = lane_id(), r16 = ln % 16, g = ln / 16;
    const params_ptr pp = P();
    // (Pointers read from the argument segment carry no address space: named global here, or the
    // loads would be issued as flat ones, which LDS waits wait for too.)
    typedef const __attribute__((address_space(1))) uint16_t* gbl_u16;
    typedef const __attribute__((address_space(1))) u32x4_t* gbl_u4;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      int jq_n, head_n;
      bool ok_n;
      row_geometry(it, 16 * qt + r16, jq_n, head_n, ok_n);
      const gbl_u16 src = ok_n ? (gbl_u16)(uintptr_t)pp->a.q + (((int64_t)(it.q0 + jq_n) * pp->a.Hq + head_n) * D + g * 8)
                               : (gbl_u16)(uintptr_t)zero_line + g * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qf[qt][ks] = __builtin_bit_cast(uint4, *(gbl_u4)(src + ks * 32));
    }
  };
  auto begin_item = [&]() __attribute__((always_inline)) {
    int first_tok;
    const int ln = lane_id(), r16 = ln % 16, g = ln / 16;
    wave_geometry(cur, wave_has_rows, first_tok, prio_sel);
    mask_from = cur.prefix + cur.j0 + first_tok - cur.pos0;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      int jq, head0;
      bool ok0;
      row_geometry(cur, 16 * qt + r16, jq, head0, ok0);
      p_j[qt] = cur.prefix + jq - cur.pos0 - g * 4;      // (the lane's group folded in: see the mask in stage())
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[qt][dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      m_run[qt] = kMinusBig;
      l_run[qt] = 0.f;
    }
    any_corr = false;
    pos_item0 = pos_use;
    // Fragment addresses in the item's first ring buffer.  K fragment: token row l%16 of a
    // 16-token group, chunk 4*ks + g.  V^T fragment: a transpose read's 16 lanes fetch 4 token rows
    // x 16 dims (lane: row 4g + (l%16)/4, 8 bytes at dims 16*dt + 4*(l%4)).
    const uint32_t buf = lds0 + (uint32_t)(pos_use & (kRing - 1)) * Geo::TILE_BYTES;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_adr[ks] = buf + r16 * ROWB + (((4 * ks + g) ^ k_swz<CPR>(r16)) * 16);
    {
      const int row = g * 4 + (ln % 16) / 4;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const int chunk = 2 * dt + (ln % 4) / 2;
        v_adr[dt] = buf + Geo::TENSOR_BYTES + row * ROWB + ((chunk ^ v_swz16<CPR>(row)) * 16) + (ln % 2) * 8;
      }
    }
  };

  auto ring_step = [&](int pos) __attribute__((always_inline)) {
    return (uint32_t)((pos & 1) ? 3 * Geo::TILE_BYTES : Geo::TILE_BYTES);
  };
  // K fragments of sub-tile s (its parity given as a constant): both 16-token groups; after the
  // odd sub-tile the addresses move on to the next tile.
  auto issue_k = [&](int s, auto odd_c) __attribute__((always_inline)) {
    constexpr int ODD = decltype(odd_c)::value;
    lds_issue4_b128<ODD * 32 * ROWB>(k_adr[0], k_adr[1], k_adr[2], k_adr[3], kf[0][0], kf[0][1], kf[0][2], kf[0][3]);
    lds_issue4_b128<ODD * 32 * ROWB + 16 * ROWB>(k_adr[0], k_adr[1], k_adr[2], k_adr[3], kf[1][0], kf[1][1], kf[1][2], kf[1][3]);
    if constexpr (ODD) {
      const uint32_t x = ring_step(pos_item0 + (s >> 1));
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) k_adr[ks] ^= x;
    }
  };
  auto ready_k = [&]() __attribute__((always_inline)) {
    lds_ready4(kf[0][0], kf[0][1], kf[0][2], kf[0][3]);
    lds_ready4(kf[1][0], kf[1][1], kf[1][2], kf[1][3]);
  };
  // V^T fragments of sub-tile sv for one half of the dim blocks (both 16-token groups each).
  auto issue_v = [&](int sv, auto odd_c, auto half_c) __attribute__((always_inline)) {
    constexpr int ODD = decltype(odd_c)::value;
    constexpr int HALF = decltype(half_c)::value;
#pragma unroll
    for (int d2 = 0; d2 < DT / 2; d2 += 2) {
      const int dt = HALF * (DT / 2) + d2;
      lds_issue4_tr<ODD * 32 * ROWB, 16 * ROWB>(v_adr[dt], v_adr[dt + 1], vf[dt][0], vf[dt][1], vf[dt + 1][0], vf[dt + 1][1]);
    }
    if constexpr (ODD && HALF == 1) {
      const uint32_t x = ring_step(pos_item0 + (sv >> 1));
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) v_adr[dt] ^= x;
    }
  };
  auto ready_v = [&](int half) __attribute__((always_inline)) {
#pragma unroll
    for (int d2 = 0; d2 < DT / 2; d2 += 2) {
      const int dt = half * (DT / 2) + d2;
      lds_ready4(vf[dt][0], vf[dt][1], vf[dt + 1][0], vf[dt + 1][1]);
    }
  };
  // S^T = K Q^T of a sub-tile: four 16x16 blocks (16-token group x query block), KS steps each.
  auto qk = [&](f32x4_t (&sc)[QT][2]) __attribute__((always_inline)) {
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) sc[qt][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          sc[qt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf[tt][ks]),
                                                               __builtin_bit_cast(bf16x8_t, qf[qt][ks]), sc[qt][tt], 0, 0, 0);
  };
  // O^T += V^T P^T for one half of the dim blocks.
  auto pv = [&](const uint4 (&pf)[QT], int half) __attribute__((always_inline)) {
#pragma unroll
    for (int d = 0; d < DT / 2; ++d) {
      const int dt = half * (DT / 2) + d;
      const u32x4_t vv = {vf[dt][0][0], vf[dt][0][1], vf[dt][1][0], vf[dt][1][1]};
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
        o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vv),
                                                            __builtin_bit_cast(bf16x8_t, pf[qt]), o[qt][dt], 0, 0, 0);
    }
  };
  // Softmax of one sub-tile: the fast and robust modes of attn_prefill_kernel.h.
  auto softmax = [&](f32x4_t (&sc)[QT][2], uint4 (&pf)[QT], auto robust_c, auto first_c) __attribute__((always_inline)) {
    constexpr bool robust = decltype(robust_c)::value;
    constexpr bool first = decltype(first_c)::value;
    any_corr = false;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      corr[qt] = 1.0f;
      if constexpr (robust || first) {
        float mx = sc[qt][0][0];
#pragma unroll
        for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sc[qt][e / 4][e % 4]);
        mx = groups_max(mx);
        const float m_cand = fmaxf(mx * scale, kMinusBig);
        const float m_new = (first || m_cand > m_run[qt] + kMaxSlack) ? m_cand : m_run[qt];
        if constexpr (robust && !first) {
          corr[qt] = __builtin_amdgcn_exp2f(m_run[qt] - m_new);
          any_corr |= m_new != m_run[qt];
        }
        m_run[qt] = m_new;
      }
      const float m_ref = m_run[qt];
      float t[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) t[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[qt][e / 4][e % 4], scale, -m_ref));
      pf[qt].x = pack_bf16(t[0], t[1]);
      pf[qt].y = pack_bf16(t[2], t[3]);
      pf[qt].z = pack_bf16(t[4], t[5]);
      pf[qt].w = pack_bf16(t[6], t[7]);
      float ps = robust ? l_run[qt] * corr[qt] : l_run[qt];
      ps = sum2_bf16(pf[qt].x, ps);
      ps = sum2_bf16(pf[qt].y, ps);
      ps = sum2_bf16(pf[qt].z, ps);
      ps = sum2_bf16(pf[qt].w, ps);
      l_run[qt] = ps;
    }
  };
  auto rescale = [&](const float (&cf)[QT]) __attribute__((always_inline)) {
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[qt][dt] *= cf[qt];
  };
  // The barrier of a tile step: the tile after the one in use must have landed in every wave's
  // share, and the buffer of the tile before it is handed to the next request.
  auto next_tile = [&]() __attribute__((always_inline)) {
    asm volatile("" : "+s"(req_bid));    // taken over where no LDS read is outstanding
    wait_vmcnt<Geo::LOADS>();
    __builtin_amdgcn_s_barrier();
    request();
    --ahead;
    ++pos_use;
  };
  auto no_sync = []() __attribute__((always_inline)) {};
  auto stage = [&](int s, auto cur_c, auto with_pv_c, auto robust_c, auto&& tile_sync) __attribute__((always_inline)) {
    constexpr int CUR = decltype(cur_c)::value;
    constexpr bool with_pv = decltype(with_pv_c)::value;
    constexpr bool robust = decltype(robust_c)::value;
    if (prio_sel) __builtin_amdgcn_s_setprio(CUR); else __builtin_amdgcn_s_setprio(CUR ^ 1);
    if constexpr (with_pv) {
      issue_v(s - 1, std::integral_constant<int, CUR ^ 1>{}, i0{});
      lds_wait<VREADS>();                // the K fragments (older than these reads) are in
    } else {
      lds_wait<0>();
    }
    ready_k();
    if (s * 32 + 31 > mask_from) {
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (s * 32 + (e / 4) * 16 + (e % 4) > p_j[qt]) scb[CUR][qt][e / 4][e % 4] = -INFINITY;
    }
    if constexpr (with_pv && robust) {
      if (__any(any_corr)) rescale(corr);
    }
    qk(scb[CUR ^ 1]);
    asm volatile("" : "+v"(kf[1][KS - 1]));
    if constexpr (with_pv) {
      issue_v(s - 1, std::integral_constant<int, CUR ^ 1>{}, i1{});
      lds_wait<VREADS>();                // first half of V^T in
      ready_v(0);
      pv(pfb[CUR ^ 1], 0);
      asm volatile("" : "+v"(vf[DT / 2 - 1][1]));
    }
    if constexpr (CUR == 0) {
      lds_wait<0>();
      tile_sync();
      issue_k(s + 2, std::integral_constant<int, CUR>{});
    } else {
      issue_k(s + 2, std::integral_constant<int, CUR>{});
      lds_wait<KREADS>();                // second half of V^T in (the K reads may be in flight)
    }
    if constexpr (with_pv) {
      ready_v(1);
      pv(pfb[CUR ^ 1], 1);
    }
    softmax(scb[CUR], pfb[CUR], robust_c, std::integral_constant<bool, !with_pv>{});
    // One MFMA (16 cycles here), then a few of the softmax's vector instructions, repeated.
#pragma unroll
    for (int i = 0; i < (with_pv ? 2 * QT * 2 * KS : QT * 2 * KS); ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x402, with_pv ? (robust ? 3 : 2) : 6, 0);
    }
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
      asm volatile("" ::"v"(pfb[CUR][qt].x), "v"(pfb[CUR][qt].y), "v"(pfb[CUR][qt].z), "v"(pfb[CUR][qt].w));
  };

  // One pass over the current item's KV tiles.  On entry its query fragments are on their way (or
  // in), and `ahead` of its first tiles are requested; the rest is requested here.
  auto attend = [&](auto robust_c) __attribute__((always_inline)) {
    while (ahead < kRing - 1) request();
    begin_item();
    // Everything this wave has in flight: the item's first tiles, its query rows, the previous
    // item's output stores.
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        asm volatile("" : "+v"(qf[qt][ks].x), "+v"(qf[qt][ks].y), "+v"(qf[qt][ks].z), "+v"(qf[qt][ks].w));
    const int n_tiles = cur.n_tiles;
    if (!wave_has_rows) {
      // None of this wave's 32 query rows exists in this item: it fetches its share of every tile
      // and keeps the barriers, leaving the SIMD to the wave that has rows.
      for (int u = 0; u < n_tiles; ++u) next_tile();
    } else {
      issue_k(0, i0{});
      lds_wait<0>();
      ready_k();
      qk(scb[0]);
      issue_k(1, i1{});
      stage(0, i0{}, std::false_type{}, robust_c, next_tile);
      stage(1, i1{}, std::true_type{}, robust_c, no_sync);
      for (int u = 1; u < n_tiles; ++u) {
        stage(2 * u, i0{}, std::true_type{}, robust_c, next_tile);
        stage(2 * u + 1, i1{}, std::true_type{}, robust_c, no_sync);
      }
      lds_wait<0>();                       // the K fragment reads of the last stage
      if constexpr (decltype(robust_c)::value) {
        if (__any(any_corr)) rescale(corr);
      }
    }
    // The query registers are free from here on: the next item's rows are requested now, ahead of
    // the last product and the output stores.  (Unconditionally - without a next item `nxt` still
    // names a valid one - so that the loads write the query registers themselves: a load on one
    // path only would go to other registers and be copied over, behind a wait for it.)
    load_q(nxt);
    if (wave_has_rows) {
      const int NS = 2 * n_tiles;
      issue_v(NS - 1, i1{}, i0{});
      issue_v(NS - 1, i1{}, i1{});
      lds_wait<0>();
      ready_v(0);
      ready_v(1);
      pv(pfb[1], 0);
      pv(pfb[1], 1);
    }
  };

  // Output of the current item.  A lane holds, for each of its two query rows, four dims of every
  // 16-dim block: stored as they are, every store instruction would touch 16 rows with 8 or 16
  // bytes each.  The values go through LDS instead (the ring buffer that the next request will
  // fill, free since the barrier behind the last product; 4 KiB per wave), 32 rows x 128 bytes per
  // pass, and come back as eight rows x 128 contiguous bytes per store instruction: whole cache
  // lines.  Staged rows are XOR-swizzled by 16-byte chunk so that neither side has bank conflicts.
  // A cut q-tile writes unnormalised partials (accumulators, and the reference / sum pair per row
  // and head) for the merge kernel; an uncut one the normalised output, fp32 or bf16.
  auto store_item = [&]() __attribute__((always_inline)) {
    float l_tot[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) l_tot[qt] = groups_sum(l_run[qt]);
    if (!wave_has_rows) return;                                   // (wave-uniform)
    const params_ptr pp = P();
    const int Hq = pp->a.Hq;
    const int ln = lane_id(), r16 = ln % 16, g = ln / 16;
    const bool partial = cur.nparts > 1;
    float inv[QT];
    uint32_t w_row[QT], w_swz[QT];
    const uint32_t stage = lds0 + (Geo::STAGE_IN_RING ? (uint32_t)(pos_req & (kRing - 1)) * Geo::TILE_BYTES
                                                      : (uint32_t)Geo::STAGE_OFFSET) + (uint32_t)wave * 4096u;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      int jq, head0;
      bool ok0;
      row_geometry(cur, 16 * qt + r16, jq, head0, ok0);
      inv[qt] = partial ? 1.0f : pp->a.out_scale / l_tot[qt];
      if (partial && ok0 && g == 0) {
        const int64_t ph = ((int64_t)cur.first_partial + (int64_t)(jq - cur.j0) * cur.nparts + cur.part) * Hq + head0;
        typedef __attribute__((address_space(1))) f32x2_t* gbl_f2;
        *(gbl_f2)((__attribute__((address_space(1))) float*)(uintptr_t)pp->w.part_ml + ph * 2) = f32x2_t{m_run[qt], l_tot[qt]};
      }
      const int row = 16 * qt + r16;
      w_row[qt] = stage + (uint32_t)row * 128u;
      w_swz[qt] = (uint32_t)((row >> 1) & 7);
    }
    // Reading side: lane l takes chunk l % 8 of rows l / 8 + 8 * pass.
    const int rr = ln / 8, ch = ln % 8;
    uint32_t r_adr[4];
    int64_t r_dst[4];                                             // element offset of the row in its destination
    bool r_ok[4];
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
      const int row = ps * 8 + rr;
      r_adr[ps] = stage + (uint32_t)row * 128u + (uint32_t)((ch ^ ((row >> 1) & 7)) * 16);
      int jq_r, head_r;
      row_geometry(cur, row, jq_r, head_r, r_ok[ps]);
      r_dst[ps] = partial ? (((int64_t)cur.first_partial + (int64_t)(jq_r - cur.j0) * cur.nparts + cur.part) * Hq + head_r) * D
                          : ((int64_t)(cur.q0 + jq_r) * Hq + head_r) * D;
    }
    const bool as_bf16 = !partial && pp->a.out_bf16;
    if (!as_bf16) {
      // fp32: a pass is 32 dims (two dim blocks); the lane's four dims of a block are one 16-byte chunk.
      typedef __attribute__((address_space(1))) float* gbl_f32;
      typedef __attribute__((address_space(1))) u32x4_t* gbl_x4;
      const gbl_f32 dst = partial ? (gbl_f32)(uintptr_t)pp->w.part_acc : (gbl_f32)(uintptr_t)pp->a.out;
#pragma unroll
      for (int p2 = 0; p2 < DT / 2; ++p2) {
#pragma unroll
        for (int dl = 0; dl < 2; ++dl)
#pragma unroll
          for (int qt = 0; qt < QT; ++qt) {
            const f32x4_t x = o[qt][2 * p2 + dl] * inv[qt];
            const u32x4_t v = {__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])};
            const uint32_t adr = w_row[qt] + (((uint32_t)(dl * 4 + g) ^ w_swz[qt]) * 16u);
            asm volatile("ds_write_b128 %0, %1" ::"v"(adr), "v"(v) : "memory");
          }
        u32x4_t r0, r1, r2, r3;
        lds_issue4_b128<0>(r_adr[0], r_adr[1], r_adr[2], r_adr[3], r0, r1, r2, r3);   // (LDS serves a wave in order)
        lds_wait<0>();
        lds_ready4(r0, r1, r2, r3);
        const u32x4_t rv[4] = {r0, r1, r2, r3};
#pragma unroll
        for (int ps = 0; ps < 4; ++ps)
          if (r_ok[ps]) *(gbl_x4)(dst + r_dst[ps] + p2 * 32 + ch * 4) = rv[ps];
      }
    } else {
      // bf16: a pass is 64 dims (four dim blocks); the lane's four dims of a block are 8 bytes.
      typedef __attribute__((address_space(1))) uint16_t* gbl_u16w;
      typedef __attribute__((address_space(1))) u32x4_t* gbl_x4;
      const gbl_u16w dst = (gbl_u16w)(uintptr_t)pp->a.out;
#pragma unroll
      for (int p4 = 0; p4 < DT / 4; ++p4) {
#pragma unroll
        for (int dl = 0; dl < 4; ++dl)
#pragma unroll
          for (int qt = 0; qt < QT; ++qt) {
            const f32x4_t x = o[qt][4 * p4 + dl] * inv[qt];
            const u32x2_t v = {pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3])};
            const uint32_t adr = w_row[qt] + (((uint32_t)(dl * 2 + g / 2) ^ w_swz[qt]) * 16u) + (uint32_t)(g % 2) * 8u;
            asm volatile("ds_write_b64 %0, %1" ::"v"(adr), "v"(v) : "memory");
          }
        u32x4_t r0, r1, r2, r3;
        lds_issue4_b128<0>(r_adr[0], r_adr[1], r_adr[2], r_adr[3], r0, r1, r2, r3);
        lds_wait<0>();
        lds_ready4(r0, r1, r2, r3);
        const u32x4_t rv[4] = {r0, r1, r2, r3};
#pragma unroll
        for (int ps = 0; ps < 4; ++ps)
          if (r_ok[ps]) *(gbl_x4)(dst + r_dst[ps] + p4 * 64 + ch * 8) = rv[ps];
      }
    }
  };

  // ---- the workgroup's life ----
  // (Two flags behind the ring, used by alternate items: a wave that saw a row sum leave the safe
  // range in the fast pass raises the item's flag, and the workgroup repeats the item in robust mode.)
  // (Read and written with LDS instructions in assembly, like the fragments: through a generic
  // pointer they would become flat accesses, which wait for every tile request in flight.)
  const uint32_t flags_lds = lds0 + (uint32_t)Geo::RING_BYTES;
  auto flag_write = [&](int which, int value) __attribute__((always_inline)) {
    asm volatile("ds_write_b32 %0, %1" ::"v"(flags_lds + 4u * (uint32_t)which), "v"(value) : "memory");
  };
  auto flag_read = [&](int which) __attribute__((always_inline)) -> int {
    int v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(flags_lds + 4u * (uint32_t)which) : "memory");
    return __builtin_amdgcn_readfirstlane(v);        // the same in every lane
  };
  if (DSV_TID0_16) { flag_write(0, 0); flag_write(1, 0); }
  cur = load_item(item_of_round(0));
  {
    const int r1 = item_of_round(1);
    has_nxt = r1 < items;
    nxt = load_item(has_nxt ? r1 : item_of_round(0));
  }
  load_q(cur);
  prime(true);
  for (;;) {
    const int par = item_round & 1;
    attend(std::false_type{});
    // The fast pass's row sums only grow, so one look at the end tells whether any of them left
    // the safe range (or stopped being a number) on the way.
    overflow = false;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) overflow |= wave_has_rows && !(l_run[qt] < kSumLimit);
    if (__any(overflow) && lane_id() == 0) flag_write(par, 1);
    lds_wait<0>();
    __builtin_amdgcn_s_barrier();
    const int redo = flag_read(par);
    if (DSV_TID0_16) flag_write(par ^ 1, 0);
    if (redo) {
      // Rare.  Everything in flight is let land (the next item's first tiles among it) and the
      // stream restarts at this item, which then runs alone: no look-ahead past its end.
      wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
      const bool keep_nxt = has_nxt;
      has_nxt = false;
      pos_req = pos_use;
      ahead = 0;
      prime(true);
      load_q(cur);
      attend(std::true_type{});
      wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
      has_nxt = keep_nxt;
      pos_req = pos_use;
      ahead = 0;
      cur.trailing = 0;
      nxt.trailing = 0;
      prime(false);
      if (has_nxt) load_q(nxt);
    }
    store_item();
    if (redo) {
      // After a repeated item nothing is requested ahead, so the next item's first requests come
      // before its first barrier: they must not land in the buffer other waves are still staging
      // their output rows through.
      lds_wait<0>();
      __builtin_amdgcn_s_barrier();
    }
    if (!has_nxt) break;
    // Positions that fetched the zero line behind this item's last tile (it had fewer tiles than
    // the look-ahead when it was the next item): passed over, one tile step each.
    for (int k = 0; k < cur.trailing; ++k) next_tile();
    // The next item becomes the current one; the cursors keep their tiles.
    ++item_round;
    cur = nxt;
    {
      const int r2 = item_of_round(item_round + 1);
      has_nxt = r2 < items;
      if (has_nxt) nxt = load_item(r2);
    }
    if (req_which == 1) {
      req_which = 0;
      if (ahead_which == 1) ahead_which = 0;
      else { ahead_which = has_nxt ? 1 : 2; ahead_t = 0; }
    } else {
      prime(false);
    }
  }
  wait_vmcnt<0>();                         // the last zero-line requests
}

#undef DSV_TID0_16

}  // namespace prefill_impl
}  // namespace dsv
