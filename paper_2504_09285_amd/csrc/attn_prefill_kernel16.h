// Attention of long prefill spans on the matrix cores, one work item per workgroup, built on the
// 16x16x32 MFMA (head_dim 128).
//
// Work items, the K/V tile ring, the software pipeline over 32-token sub-tiles and the two softmax
// modes are attn_prefill_kernel.h's (read that header first; paper sections 2.1, 3.1, 4.2 for what
// is computed); the shape of the products and the fragment layouts are those of
// attn_prefill_persistent16.h: a wave owns its 32 query rows as two 16-row blocks, lane l holding
// rows 16*qt + l%16 and the tokens 4*(l/16) .. +3 of every 16-token group.  This body serves the
// launches that mix prefill tiles with row work.
#pragma once
#include "attn_prefill_persistent16.h"

namespace dsv {
namespace prefill_impl {

template <int D>
__device__ __forceinline__ void prefill_tiles_body16(const TilesParams& prm, int bx, int bz, unsigned char* smem) {
  using Geo = TileGeom<D>;
  constexpr int ROWB = Geo::ROWB, CPR = Geo::CPR, RPP = Geo::RPP, PPW = Geo::PPW;
  constexpr int KS = D / 32;             // k-steps of K Q^T
  constexpr int DT = D / 16;             // 16-dim blocks of O^T
  constexpr int QT = 2;                  // 16-row query blocks per wave
  static_assert(NH == 1 && KS == 4 && DT % 4 == 0, "fragment reads are issued in groups of four");
  typedef __attribute__((ext_vector_type(4))) float f32x4_t;
  constexpr int KREADS = 2 * KS, VREADS = DT;
  static_assert(KREADS <= 15 && VREADS <= 15, "the LDS read counter has four bits");
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  const AttnArgs& a = prm.a;
  const int tid = (int)threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int lane = tid % kWave;
  const int r16 = lane % 16;             // query row within a 16-row block / token row of a 16-token group
  const int g = lane / 16;               // lane group: tokens 4g..4g+3 of a group, dims 8g..8g+7 of a k-step
  // Wave w runs on SIMD w % 4.  With four query heads per KV head, SIMD s hosts both halves of
  // the query tile for head s.  With one or two heads per KV head most head slots are empty
  // (their waves only fetch tiles): the waves that have rows are then spread over the SIMDs
  // instead of sharing SIMD 0 (and 1).
  const bool few_heads = prm.G - bz * 4 <= 2;
  const int tg = few_heads ? wave % 2 : wave / kHeadWaves;          // which 32 query tokens of the tile
  const int hp = few_heads ? wave / 2 : wave % kHeadWaves;          // which query head of the group of four
  // Flat rows (head groups that are not four heads): row r = 32 * wave + (the wave's row) of the work item is
  // the pair (token j0 + r / gh, head bz * gh + r % gh) of a group of gh heads; rows
  // tile_q * gh .. 255 do not exist.  Everything below that is per query row (its token's
  // position, its head's rows of Q and of the output) is per lane already.
  const int gh = prm.flat_heads;
  const bool flat = gh > 0;
  const int fmagic = prm.flat_magic;
  const int wave_first_tok = flat ? flat_div(32 * wave, fmagic) : 32 * tg;   // first query token of the wave, from j0

  // Workgroups are dispatched in index order (bx) and dealt round-robin to the eight XCDs: the
  // KV head is the fastest index, so the heaviest tiles (the list is sorted) of every head start
  // first and (with eight KV heads) all tiles of one head share one XCD's L2.
  const int kvh = bx % a.Hkv;
  const int tile = bx / a.Hkv;
  const int seq = prm.w.tile_seq[tile];
  const int j0 = prm.w.tile_q0[tile];
  const int q0 = a.q_offsets[seq];
  const int q_len = a.q_offsets[seq + 1] - q0;
  const int ctx = a.ctx_lens[seq];
  const int prefix = ctx - q_len;
  const int table_row = prm.stage_rows ? prm.stage_rows[seq] : seq;
  const int32_t* table = a.block_tables + (int64_t)table_row * a.max_blocks;
  const int nblk = (ctx + kBlockSize - 1) / kBlockSize;
  const int kv_end = min(ctx, prefix + j0 + prm.tile_q);      // exclusive: last visible token + 1
  // The work item covers KV tiles [t_first, t_first + n_tiles) of the n_kv the query tile
  // visits: all of them, or one of several nearly equal partitions whose results a merge kernel
  // combines.  Tile and sub-tile indices below are relative to t_first.
  const int n_kv = (kv_end + kTileKV - 1) / kTileKV;
  const int part_rec = prm.w.tile_part[tile];
  const int part = part_rec & 0xffff, nparts = part_rec >> 16;
  const int base_kv = n_kv / nparts, rem_kv = n_kv - base_kv * nparts;
  const int t_first = part * base_kv + min(part, rem_kv);
  const int n_tiles = base_kv + (part < rem_kv ? 1 : 0);
  const int pos0 = t_first * kTileKV;                          // position of the partition's first token
  const int NS = 2 * n_tiles;                                  // 32-token sub-tiles

  // Query fragments: B operand of S^T = K Q^T; lane (row r16 of block qt, group g) holds dims
  // 32*ks + 8*g .. +8.  Row 16*qt + r16 of the wave is row 32*wave + 16*qt + r16 of the work item.
  // (wave-uniform) Does any of this wave's 32 query rows exist?
  const bool wave_has_rows = flat ? (j0 + wave_first_tok < q_len && 32 * wave < prm.tile_q * gh)
                                  : (j0 + 32 * tg < q_len && bz * 4 + hp * NH < prm.G);
  bool head_ok[QT];
  int head[QT], jq[QT], p_j[QT];
  uint4 qf[QT][KS];
  static_assert(D * 2 <= 256, "a query row fits the zero line");
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int row = 16 * qt + r16, r_item = 32 * wave + row;
    jq[qt] = flat ? j0 + flat_div(r_item, fmagic) : j0 + 32 * tg + row;       // new-token index of this query row
    p_j[qt] = prefix + jq[qt] - pos0 - 4 * g;                    // its position in the partition, the lane's group folded in
    const int hsub = flat ? bz * gh + (r_item - flat_div(r_item, fmagic) * gh) : bz * 4 + hp * NH;
    head_ok[qt] = hsub < prm.G && jq[qt] < q_len && (!flat || r_item < prm.tile_q * gh);
    head[qt] = kvh * prm.G + (hsub < prm.G ? hsub : 0);
    // A row that does not exist reads the zero line: the choice is made on the address, so the
    // loads stay in flight next to the tile requests below instead of being waited for here.
    const uint16_t* src = head_ok[qt] ? a.q + (((int64_t)(q0 + jq[qt]) * a.Hq + head[qt]) * D + g * 8)
                                      : reinterpret_cast<const uint16_t*>(prm.w.zero_line) + g * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[qt][ks] = *reinterpret_cast<const uint4*>(src + ks * 32);
  }

  // ---- direct global->LDS loads: waves 2i and 2i+1 fetch one half each of block 4t+i of tile t ----
  // The block id comes from the table by a scalar load (constant address space: the table is
  // not written while the kernel runs), requested one tile ahead of its use, so it never queues
  // behind, or waits for, the vector-memory tile requests.  Everything per lane is a 32-bit
  // offset fixed for the whole kernel; per tile only the scalar block base changes.
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const const_i32_ptr ctable = (const_i32_ptr)(uintptr_t)table;
  const unsigned char* const zero_line = reinterpret_cast<const unsigned char*>(prm.w.zero_line);
  const uint32_t tok_stride = (uint32_t)a.Hkv * D;             // elements between tokens of a block
  const int blk_in_tile = wave / kWavesPerBlock, half = wave % kWavesPerBlock;
  uint32_t k_src[PPW], v_src[PPW];                     // byte offsets from the block's head slice
  int slot_n[PPW];                                         // token slot in the block
#pragma unroll
  for (int ii = 0; ii < PPW; ++ii) {
    const int n = (half * (PPW) + ii) * RPP + lane / CPR;
    const int row = blk_in_tile * kBlockSize + n;              // row in the tile
    const int pos = lane % CPR;
    slot_n[ii] = n;
    k_src[ii] = ((uint32_t)n * tok_stride + (uint32_t)((pos ^ k_swz<CPR>(row)) * 8)) * 2u;
    v_src[ii] = ((uint32_t)n * tok_stride + (uint32_t)((pos ^ v_swz16<CPR>(row)) * 8)) * 2u;
  }
  const uint32_t zero_src = (uint32_t)(lane % CPR) * 16u;
  const unsigned char* const k_head = reinterpret_cast<const unsigned char*>(a.k_pool + (uint32_t)kvh * D);
  const unsigned char* const v_head = reinterpret_cast<const unsigned char*>(a.v_pool + (uint32_t)kvh * D);
  // Table entry for this wave's block of tile t, clamped into the table so that the load never
  // needs a branch; whether the block exists is decided when the id is used, so nothing waits
  // for the load here.
  auto block_id = [&](int t) __attribute__((always_inline)) -> int {
    const int b = (t_first + t) * (kTileKV / kBlockSize) + blk_in_tile;
    return ctable[min(b, nblk - 1)];
  };
  auto issue_tile = [&](int t, int bid) __attribute__((always_inline)) {
    const int b = (t_first + t) * (kTileKV / kBlockSize) + blk_in_tile;
    unsigned char* kdst = smem + (t % kRing) * Geo::TILE_BYTES + blk_in_tile * (kBlockSize * ROWB) +
                          half * (PPW) * 1024;
    unsigned char* vdst = kdst + Geo::TENSOR_BYTES;
    // Past the table every lane reads the zero line.  In a block that straddles ctx, K may hold
    // anything (its columns are masked) but V rows that must not be read come from the zero
    // line as well.  Branch-free: selects on the source address.
    const bool have = t < n_tiles && b < nblk;
    const int64_t blk_bytes = (int64_t)bid * kBlockSize * tok_stride * 2;
    const unsigned char* kb = k_head + blk_bytes;
    const unsigned char* vb = v_head + blk_bytes;
    const int visible = ctx - b * kBlockSize;                  // token slots < visible may be read
#pragma unroll
    for (int ii = 0; ii < PPW; ++ii) {
      const unsigned char* kp = have ? kb + k_src[ii] : zero_line + zero_src;
      const unsigned char* vp = (have && slot_n[ii] < visible) ? vb + v_src[ii] : zero_line + zero_src;
      __builtin_amdgcn_global_load_lds((gbl_void_t)kp, (lds_void_t)(kdst + ii * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gbl_void_t)vp, (lds_void_t)(vdst + ii * 1024), 16, 0, 0);
    }
  };

  // ---- LDS fragment addresses (bytes, relative to the tile buffer) ----
  // K fragment: token row r16 of a 16-token group, chunk 4*ks + g.  V^T fragment: a transpose
  // read's 16 lanes fetch 4 token rows x 16 dims (lane: row 4g + r16/4, 8 bytes at dims 16*dt + 4*(l%4)).
  uint32_t k_off[KS], v_off[DT];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_off[ks] = lds0 + r16 * ROWB + (((4 * ks + g) ^ k_swz<CPR>(r16)) * 16);
  {
    const int row = g * 4 + r16 / 4;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const int chunk = 2 * dt + (lane % 4) / 2;
      v_off[dt] = lds0 + Geo::TENSOR_BYTES + row * ROWB + ((chunk ^ v_swz16<CPR>(row)) * 16) + (lane % 2) * 8;
    }
  }

  f32x4_t o[QT][DT];
  float m_run[QT], l_run[QT];            // l_run: over the lane's own tokens
  const float scale = a.scale_log2e;
  f32x4_t scb[2][QT][2];                 // [buffer][query block][16-token group of the sub-tile]
  uint4 pfb[2][QT];                      // a sub-tile's probabilities, B operand of O^T += V^T P^T
  float corr[QT];
  bool any_corr;
  u32x4_t kf[2][KS];                     // K fragments of a sub-tile: [16-token group][k-step]
  u32x2_t vf[DT][2];                     // V^T fragments of a sub-tile: [dim block][16-token group]
  static_assert(kRing == 4 && (Geo::TILE_BYTES & (Geo::TILE_BYTES - 1)) == 0, "XOR stepping of the ring");
  uint32_t k_adr[KS], v_adr[DT];
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

  auto ring_step = [&](int tile) __attribute__((always_inline)) {
    return (uint32_t)((tile & 1) ? 3 * Geo::TILE_BYTES : Geo::TILE_BYTES);
  };
  // K fragments of sub-tile s (its parity given as a constant): both 16-token groups; after the
  // odd sub-tile the addresses move on to the next tile.
  auto issue_k = [&](int s, auto odd_c) __attribute__((always_inline)) {
    constexpr int ODD = decltype(odd_c)::value;
    lds_issue4_b128<ODD * 32 * ROWB>(k_adr[0], k_adr[1], k_adr[2], k_adr[3], kf[0][0], kf[0][1], kf[0][2], kf[0][3]);
    lds_issue4_b128<ODD * 32 * ROWB + 16 * ROWB>(k_adr[0], k_adr[1], k_adr[2], k_adr[3], kf[1][0], kf[1][1], kf[1][2], kf[1][3]);
    if constexpr (ODD) {
      const uint32_t x = ring_step(s >> 1);
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
      const uint32_t x = ring_step(sv >> 1);
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
  auto stage = [&](int s, auto cur_c, auto with_pv_c, auto robust_c, auto&& tile_sync) __attribute__((always_inline)) {
    constexpr int CUR = decltype(cur_c)::value;
    constexpr bool with_pv = decltype(with_pv_c)::value;
    constexpr bool robust = decltype(robust_c)::value;
    if (flat ? wave / 4 : tg) __builtin_amdgcn_s_setprio(CUR); else __builtin_amdgcn_s_setprio(CUR ^ 1);
    if constexpr (with_pv) {
      issue_v(s - 1, std::integral_constant<int, CUR ^ 1>{}, std::integral_constant<int, 0>{});
      lds_wait<VREADS>();                // the K fragments (older than these reads) are in
    } else {
      lds_wait<0>();
    }
    ready_k();
    if (s * 32 + 31 > prefix + j0 + wave_first_tok - pos0) {
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
      issue_v(s - 1, std::integral_constant<int, CUR ^ 1>{}, std::integral_constant<int, 1>{});
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


  using i0 = std::integral_constant<int, 0>;
  using i1 = std::integral_constant<int, 1>;
  // (The flag lives behind the ring in the dynamic LDS: the kernel must own no static LDS, so
  // that the ring starts at LDS address 0; the launchers check that.)
  volatile int& wg_overflow = *reinterpret_cast<volatile int*>(smem + Geo::RING_BYTES);
  if (tid == 0) wg_overflow = 0;
  // One pass over the KV tiles of this work item, in fast or robust mode.
  auto attend = [&](auto robust_c) __attribute__((always_inline)) {
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[qt][dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      m_run[qt] = kMinusBig;
      l_run[qt] = 0.f;
    }
    any_corr = false;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_adr[ks] = k_off[ks];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) v_adr[dt] = v_off[dt];
    // ---- prologue: tiles 0..2 requested, tile 0 awaited ----
    issue_tile(0, block_id(0));
    issue_tile(1, block_id(1));
    issue_tile(2, block_id(2));
    int next_bid = block_id(3);
    wait_vmcnt<2 * Geo::LOADS>();
    __builtin_amdgcn_s_barrier();
    // The query fragments were requested before the tiles, so they have arrived.  Redefining them
    // here keeps the compiler from guarding their first use inside the loop with a wait that
    // would drain the tile requests in flight on every iteration.
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        asm volatile("" : "+v"(qf[qt][ks].x), "+v"(qf[qt][ks].y), "+v"(qf[qt][ks].z), "+v"(qf[qt][ks].w));

    // Barrier of tile u, inside stage 2u, after the wave's last read of tile u-1 (the second half
    // of the V^T fragments of sub-tile 2u-1) and before its first read of tile u+1 (the K
    // fragments of sub-tile 2u+2): tile u+1 must be complete, while tile u+2 may still be in
    // flight, and the buffer of tile u-1 now takes tile u+3.
    // (A bare s_barrier: __syncthreads() would add a fence that drains every load in flight.
    // Each wave has waited for its own loads and for its own LDS reads.)
    int u_sync = 0;
    auto next_tile = [&]() __attribute__((always_inline)) {
      // Called with no LDS read outstanding: the block id requested a tile ago is taken over
      // here, so that the wait the compiler puts before its first use is already satisfied and
      // is not moved up to where fragment reads are in flight.
      asm volatile("" : "+s"(next_bid));
      wait_vmcnt<Geo::LOADS>();
      __builtin_amdgcn_s_barrier();
      issue_tile(u_sync + 3, next_bid);
      next_bid = block_id(u_sync + 4);
      ++u_sync;
    };
    auto no_sync = []() __attribute__((always_inline)) {};
    if (!wave_has_rows) {
      // All 32 query rows of this wave lie beyond the span (a short span, or the ragged last tile
      // of one), or its query head beyond the group: the wave only fetches its share of every
      // tile and keeps the barriers - the one above and one per tile, as in the stages below -
      // and leaves the SIMD to the wave that has rows.
      for (int u = 0; u < n_tiles; ++u) next_tile();
      wait_vmcnt<0>();
      return;
    }
    issue_k(0, i0{});
    lds_wait<0>();
    ready_k();
    qk(scb[0]);
    issue_k(1, i1{});
    stage(0, i0{}, std::false_type{}, robust_c, next_tile);
    stage(1, i1{}, std::true_type{}, robust_c, no_sync);
    for (int u = 1; u < n_tiles; ++u) {
      stage(2 * u, i0{}, std::true_type{}, robust_c, next_tile);
      // The last stages also fetch and score sub-tiles past the end: their buffers hold the
      // zeros of tile requests past the end, and the results are never used.
      stage(2 * u + 1, i1{}, std::true_type{}, robust_c, no_sync);
    }
    lds_wait<0>();                         // the K fragment reads of the last stage
    // V^T P^T of the last sub-tile.
    if constexpr (decltype(robust_c)::value) {
      if (__any(any_corr)) rescale(corr);
    }
    issue_v(NS - 1, i1{}, i0{});           // NS - 1 is odd: the second sub-tile of the last tile
    issue_v(NS - 1, i1{}, i1{});
    lds_wait<0>();
    ready_v(0);
    ready_v(1);
    pv(pfb[1], 0);
    pv(pfb[1], 1);
    wait_vmcnt<0>();                     // the last (dummy) tile requests
  };
  attend(std::false_type{});
  // The fast pass's row sums only grow, so one look at the end tells whether any of them left the
  // safe range (or stopped being a number) on the way.  Any wave that saw that makes the whole
  // workgroup (the tile requests and barriers are collective) repeat the work item in robust mode.
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) overflow |= wave_has_rows && !(l_run[qt] < kSumLimit);
  if (__any(overflow) && lane == 0) wg_overflow = 1;
  __syncthreads();
  if (wg_overflow) attend(std::true_type{});

  // Output.  A lane holds, for each of its two query rows, four dims of every 16-dim block: stored
  // as they are, every store instruction would touch 16 rows with 8 or 16 bytes each.  The values
  // go through LDS instead (the ring is free: every request has landed and every wave is past its
  // last fragment read; 4 KiB per wave), 32 rows x 128 bytes per pass, and come back as eight rows x
  // 128 contiguous bytes per store instruction: whole cache lines.  Staged rows are XOR-swizzled by
  // 16-byte chunk so that neither side has bank conflicts.
  // A cut q-tile writes unnormalised partials (accumulators, and the reference / sum pair per row
  // and head) for the merge kernel; token j of the tile, partition p -> partial
  // first + j * partitions + p.  An uncut one writes the normalised output, fp32 or bf16.
  static_assert(kWaves * 4096 <= Geo::RING_BYTES, "the staging area fits the ring");
  __syncthreads();
  {
    float l_tot[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) l_tot[qt] = groups_sum(l_run[qt]);
    if (!wave_has_rows) return;                                   // (wave-uniform)
    const bool partial = nparts > 1;
    const int first_partial = partial ? prm.w.tile_item0[tile] : -1;
    const uint32_t stage_lds = lds0 + (uint32_t)wave * 4096u;
    float inv[QT];
    uint32_t w_row[QT], w_swz[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      inv[qt] = partial ? 1.0f : a.out_scale / l_tot[qt];
      if (partial && head_ok[qt] && g == 0) {
        const int64_t ph = ((int64_t)first_partial + (int64_t)(jq[qt] - j0) * nparts + part) * a.Hq + head[qt];
        *reinterpret_cast<float2*>(prm.w.part_ml + ph * 2) = make_float2(m_run[qt], l_tot[qt]);
      }
      const int row = 16 * qt + r16;
      w_row[qt] = stage_lds + (uint32_t)row * 128u;
      w_swz[qt] = (uint32_t)((row >> 1) & 7);
    }
    const int rr = lane / 8, ch = lane % 8;               // reading side: chunk ch of rows rr + 8 * pass
    uint32_t r_adr[4];
    int64_t r_dst[4];                                             // element offset of the row in its destination
    bool r_ok[4];
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
      const int row = ps * 8 + rr;
      r_adr[ps] = stage_lds + (uint32_t)row * 128u + (uint32_t)((ch ^ ((row >> 1) & 7)) * 16);
      const int r_item = 32 * wave + row;
      const int jq_r = flat ? j0 + flat_div(r_item, fmagic) : j0 + 32 * tg + row;
      const int hsub = flat ? bz * gh + (r_item - flat_div(r_item, fmagic) * gh) : bz * 4 + hp * NH;
      r_ok[ps] = hsub < prm.G && jq_r < q_len && (!flat || r_item < prm.tile_q * gh);
      const int head_r = kvh * prm.G + (hsub < prm.G ? hsub : 0);
      r_dst[ps] = partial ? (((int64_t)first_partial + (int64_t)(jq_r - j0) * nparts + part) * a.Hq + head_r) * D
                          : ((int64_t)(q0 + jq_r) * a.Hq + head_r) * D;
    }
    const bool as_bf16 = !partial && a.out_bf16;
    if (!as_bf16) {
      // fp32: a pass is 32 dims (two dim blocks); the lane's four dims of a block are one 16-byte chunk.
      float* const dst = partial ? prm.w.part_acc : reinterpret_cast<float*>(a.out);
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
          if (r_ok[ps]) *reinterpret_cast<u32x4_t*>(dst + r_dst[ps] + p2 * 32 + ch * 4) = rv[ps];
      }
    } else {
      // bf16: a pass is 64 dims (four dim blocks); the lane's four dims of a block are 8 bytes.
      uint16_t* const dst = reinterpret_cast<uint16_t*>(a.out);
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
          if (r_ok[ps]) *reinterpret_cast<u32x4_t*>(dst + r_dst[ps] + p4 * 64 + ch * 8) = rv[ps];
      }
    }
  }
}

// The body a launch uses for head_dim D: the 16x16x32 one where it exists.
template <int D>
__device__ __forceinline__ void prefill_tiles_item(const TilesParams& prm, int bx, int bz, unsigned char* smem) {
  if constexpr (D == 128) prefill_tiles_body16<D>(prm, bx, bz, smem);
  else prefill_tiles_body<D>(prm, bx, bz, smem);
}

}  // namespace prefill_impl
}  // namespace dsv
