// Single-query-token attention over a paged KV cache, split along the context ("row" work).
//
// Serves the decode tokens of a mixed batch - one new token attending to its whole cached
// context, the memory-bound part of a step (paper sections 2.1 and 4.2) - and the tokens of
// prefill spans too short for the tile kernel.  The job is to stream K and V from HBM once, at
// full bandwidth, with as little else in the way as possible:
//
//  * A work item is (query token, context partition); a workgroup takes one item and gives
//    each of its waves one KV head, so the waves of a workgroup together stream whole 16-token
//    blocks (all heads of a block are contiguous in the pool).
//  * Each wave owns a private ring of block slots in LDS and fills it with direct
//    global->LDS loads (16 bytes per lane, no staging registers).  R-1 blocks are always in
//    flight behind the one being consumed; with the whole 160 KB of LDS of a CU used this way
//    the bytes in flight cover the HBM latency.  No workgroup barrier is needed: a wave only
//    ever reads what it loaded itself, ordered by the vector-memory counter.
//  * The arithmetic runs on the matrix cores so that the vector ALU stays nearly idle: the G
//    query heads that share the KV head (padded to 16 rows) form the MFMA column, scores are
//    S^T = K Q^T (16x16x32), the output is O^T = V^T P^T (16x16x16) with the V^T operand fetched
//    by LDS transpose reads.  S^T comes out with lane (head, j) holding tokens 4j..4j+3, which
//    is exactly the B operand layout of the second product; P stays in registers.
//  * LDS rows are XOR-swizzled (free: each lane picks which 16 bytes of the row it loads) so
//    that both the K fragment reads and the V transpose reads are bank-conflict free.
// Scores are kept in the log2 domain (scale*log2(e) folded in, exp2 for exp).  Token slots
// beyond the partition are excluded by select, and their V rows are replaced by zeros at load
// time, so pool garbage (possibly NaN/Inf) cannot reach the output.
#pragma once
#include "attn_internal.h"

namespace dsv {
namespace rows_impl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef __attribute__((address_space(3))) void* lds_void_t;
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_t;
typedef const __attribute__((address_space(1))) void* gbl_void_t;

constexpr float kMinusBig = -1.0e30f;    // finite stand-in for "no token seen yet"
constexpr int kRowHeads = 16;            // query heads per wave (MFMA column count)
// Cache policy of the K/V block requests: the "nt" bit.  Every K/V byte is read exactly once by
// this kernel, so it should not displace block tables, queries, work lists and the partials
// that the merge kernel re-reads from L2 (measured: rows kernel -4 %, merge kernel -25 %).
constexpr int kStreamOnce = 2;

struct RowsParams {
  AttnArgs a;
  WorkLists w;
  int32_t part_tokens;
  int32_t G;            // query heads per KV head
  int32_t gy;           // workgroups per item along the KV heads (a workgroup covers `waves` of them)
};

// Work item of the wg-th row workgroup: the workgroups of one item (KV head groups, and groups of
// kRowHeads query heads per KV head) follow each other, so the longest-first order of the items holds
// for the whole launch.
__device__ __forceinline__ void row_work_item(uint32_t wg, int gy, int G, int& bx, int& by, int& bz) {
  const uint32_t per_item = (uint32_t)gy * (uint32_t)((G + kRowHeads - 1) / kRowHeads), sub = wg % per_item;
  bx = (int)(wg / per_item);
  by = (int)(sub % (uint32_t)gy);
  bz = (int)(sub / (uint32_t)gy);
}

// EB = bytes per cached element: 2 (bf16) or 1 (E4M3 codes, widened to bf16 in registers).
template <int D, int EB>
struct RowGeom {
  static constexpr int ROWB = D * EB;             // bytes per token row of one head
  static constexpr int CPR = ROWB / 16;           // 16-byte chunks per row
  static constexpr int TPI = kWave / CPR;         // token rows per load instruction
  static constexpr int IPB = kBlockSize / TPI;    // load instructions per block, per tensor
  static constexpr int KS = D / 32;               // 16x16x32 k-steps of K Q^T
  static constexpr int DB = D / 16;               // 16-dim blocks of O^T
  static constexpr int TENSOR_BYTES = kBlockSize * ROWB;
  static constexpr int SLOT_BYTES = 2 * TENSOR_BYTES;
  static constexpr int LOADS_PER_BLOCK = 2 * IPB;
  static constexpr int ROWS_PER_WRAP = 256 / ROWB;   // token rows before the LDS banks repeat
};

// Row swizzles: 16-byte chunk c of token row n is stored at chunk position c ^ swz(n), chosen so
// that the rows which share LDS banks are read at different chunk positions.
template <int D, int EB> __device__ __forceinline__ int k_swz(int n) {
  using Geo = RowGeom<D, EB>;
  if (EB == 2) return n & (Geo::CPR - 1);
  return (n / Geo::ROWS_PER_WRAP) & (Geo::CPR - 1);
}
template <int D, int EB> __device__ __forceinline__ int v_swz(int n) {
  using Geo = RowGeom<D, EB>;
  if (EB == 2) return 2 * (n & (Geo::CPR / 2 - 1));
  return 2 * ((n / Geo::ROWS_PER_WRAP) & (Geo::CPR / 2 - 1));
}

// Two E4M3 codes (bytes 0,1 or 2,3 of w) widened to a bf16 pair; exact, every code is a bf16 value.
template <bool HI>
__device__ __forceinline__ bf16x2_t widen2(uint32_t w) {
  return __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)w, 1.0f, HI);
}
// Eight codes (two registers) -> eight bf16 in the same order.
__device__ __forceinline__ bf16x8_t widen8(u32x2_t w) {
  const bf16x2_t a = widen2<false>(w.x), b = widen2<true>(w.x), c = widen2<false>(w.y), d = widen2<true>(w.y);
  const bf16x4_t ab = __builtin_shufflevector(a, b, 0, 1, 2, 3), cd = __builtin_shufflevector(c, d, 0, 1, 2, 3);
  return __builtin_shufflevector(ab, cd, 0, 1, 2, 3, 4, 5, 6, 7);
}

// max / sum across the four lane groups j (lanes l, l^16, l^32, l^48).
__device__ __forceinline__ float cross16_max(float x) {
  x = fmaxf(x, __shfl_xor(x, 16));
  return fmaxf(x, __shfl_xor(x, 32));
}
__device__ __forceinline__ float cross16_sum(float x) {
  x += __shfl_xor(x, 16);
  return x + __shfl_xor(x, 32);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// LDS transpose reads of the V^T fragments, issued as one group and waited for together.  They
// are written in assembly because the compiler, not knowing which LDS bytes the direct
// global->LDS loads in flight will write, would otherwise drain every one of those loads
// before each transpose read and serialise the ring.  The caller has already waited (vmcnt)
// for the block that is read here.
__device__ __forceinline__ void read_vt4(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3,
                                         s16x4_t& v0, s16x4_t& v1, s16x4_t& v2, s16x4_t& v3) {
  asm volatile(
      "ds_read_b64_tr_b16 %0, %4\n\t"
      "ds_read_b64_tr_b16 %1, %5\n\t"
      "ds_read_b64_tr_b16 %2, %6\n\t"
      "ds_read_b64_tr_b16 %3, %7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3)
      : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
      : "memory");
}
// The K fragments of a block of 8-bit codes (8 bytes per lane and k-step), in assembly for the
// same reason.
__device__ __forceinline__ void read_k4(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3,
                                        u32x2_t& v0, u32x2_t& v1, u32x2_t& v2, u32x2_t& v3) {
  asm volatile(
      "ds_read_b64 %0, %4\n\t"
      "ds_read_b64 %1, %5\n\t"
      "ds_read_b64 %2, %6\n\t"
      "ds_read_b64 %3, %7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3)
      : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
      : "memory");
}
__device__ __forceinline__ void read_k2(uint32_t a0, uint32_t a1, u32x2_t& v0, u32x2_t& v1) {
  asm volatile(
      "ds_read_b64 %0, %2\n\t"
      "ds_read_b64 %1, %3\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(v0), "=&v"(v1)
      : "v"(a0), "v"(a1)
      : "memory");
}
__device__ __forceinline__ void read_vt2(uint32_t a0, uint32_t a1, s16x4_t& v0, s16x4_t& v1) {
  asm volatile(
      "ds_read_b64_tr_b16 %0, %2\n\t"
      "ds_read_b64_tr_b16 %1, %3\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(v0), "=&v"(v1)
      : "v"(a0), "v"(a1)
      : "memory");
}

// One 16-token block of a wave's KV head against the wave's query heads: scores, running softmax
// and the update of the output accumulators.  `slot_lds` is the LDS address of the block's ring
// slot (K rows, then V rows), k_off / v_off the lane's fragment offsets inside a slot (v_off
// counted from the slot's start), `tok` the context position of the lane's first token
// (block * 16 + 4 * lane group), t1 the end of the item's token range.
template <int D, bool KV8>
__device__ __forceinline__ void row_block_step(uint32_t slot_lds, const int (&k_off)[RowGeom<D, KV8 ? 1 : 2>::KS],
                                               const uint32_t (&v_off)[KV8 ? RowGeom<D, 1>::DB / 2 : RowGeom<D, 2>::DB],
                                               const bf16x8_t (&qf)[RowGeom<D, KV8 ? 1 : 2>::KS], int tok, int t1,
                                               float scale, f32x4_t (&o)[RowGeom<D, KV8 ? 1 : 2>::DB], float& m_run,
                                               float& l_run) {
  constexpr int EB = KV8 ? 1 : 2;
  using Geo = RowGeom<D, EB>;
  constexpr int KS = Geo::KS, DB = Geo::DB;
  constexpr int VT = KV8 ? DB / 2 : DB;                  // transpose reads per block
  // S^T = K Q^T: lane (head qcol, jj) gets tokens 4jj..4jj+3 of the block.
  f32x4_t s = {0.f, 0.f, 0.f, 0.f};
  if constexpr (KV8) {
    const uint32_t kb = slot_lds;
    u32x2_t kc[KS];
    if constexpr (KS == 4) read_k4(kb + k_off[0], kb + k_off[1], kb + k_off[2], kb + k_off[3], kc[0], kc[1], kc[2], kc[3]);
    else read_k2(kb + k_off[0], kb + k_off[1], kc[0], kc[1]);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(widen8(kc[ks]), qf[ks], s, 0, 0, 0);
  } else {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      typedef const __attribute__((address_space(3))) bf16x8_t* lds_frag_t;
      const bf16x8_t kf = *(lds_frag_t)(uintptr_t)(slot_lds + (uint32_t)k_off[ks]);
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[ks], s, 0, 0, 0);
    }
  }
  if (tok + 3 >= t1) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (tok + e >= t1) s[e] = -INFINITY;
  }
  const float mx = cross16_max(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])));
  const float m_new = fmaxf(m_run, mx * scale);
  const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
  m_run = m_new;
  float p[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], scale, -m_new));
  const f32x2_t p01 = {p[0], p[1]}, p23 = {p[2], p[3]};
  const bf16x2_t b01 = __builtin_convertvector(p01, bf16x2_t), b23 = __builtin_convertvector(p23, bf16x2_t);
  const bf16x4_t pf = __builtin_shufflevector(b01, b23, 0, 1, 2, 3);
  // The row sum is taken over the bf16-rounded probabilities that enter the PV product, so
  // that the weights actually applied sum to one.
  const uint32_t u01 = __builtin_bit_cast(uint32_t, b01), u23 = __builtin_bit_cast(uint32_t, b23);
  l_run = l_run * corr + (__builtin_bit_cast(float, u01 << 16) + __builtin_bit_cast(float, u01 & 0xffff0000u)) +
          (__builtin_bit_cast(float, u23 << 16) + __builtin_bit_cast(float, u23 & 0xffff0000u));

  // O^T = O^T * corr + V^T P^T.
  constexpr int VG = VT >= 4 ? 4 : 2;                  // transpose reads issued together
#pragma unroll
  for (int d4 = 0; d4 < VT; d4 += VG) {
    s16x4_t vt[VG];
    if constexpr (VG == 4)
      read_vt4(slot_lds + v_off[d4], slot_lds + v_off[d4 + 1], slot_lds + v_off[d4 + 2],
               slot_lds + v_off[d4 + 3], vt[0], vt[1], vt[2], vt[3]);
    else
      read_vt2(slot_lds + v_off[d4], slot_lds + v_off[d4 + 1], vt[0], vt[1]);
#pragma unroll
    for (int u = 0; u < VG; ++u) {
      if constexpr (KV8) {
        // vt[u]: 16-bit unit e = token 4jj+e, low byte dim 32(d4+u) + 2m, high byte the next
        // dim (m = lane % 16).  Gather the even-dim and the odd-dim codes of the four tokens
        // and widen them: two A fragments, rows m <-> dims 32(d4+u) + 2m (+1).
        const u32x2_t w = __builtin_bit_cast(u32x2_t, vt[u]);
        const uint32_t ev = __builtin_amdgcn_perm(w.y, w.x, 0x06040200u);
        const uint32_t od = __builtin_amdgcn_perm(w.y, w.x, 0x07050301u);
        const bf16x4_t a_ev = __builtin_shufflevector(widen2<false>(ev), widen2<true>(ev), 0, 1, 2, 3);
        const bf16x4_t a_od = __builtin_shufflevector(widen2<false>(od), widen2<true>(od), 0, 1, 2, 3);
        const int db = 2 * (d4 + u);
        o[db] *= corr;
        o[db + 1] *= corr;
        o[db] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, a_ev), __builtin_bit_cast(s16x4_t, pf), o[db], 0, 0, 0);
        o[db + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, a_od), __builtin_bit_cast(s16x4_t, pf), o[db + 1], 0, 0, 0);
      } else {
        o[d4 + u] *= corr;
        o[d4 + u] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vt[u], __builtin_bit_cast(s16x4_t, pf), o[d4 + u], 0, 0, 0);
      }
    }
  }
}

// The kernel body as a device function, so that the same code serves the kernel of its own and
// the launch that mixes row work with prefill tiles.  (bx, by, bz) stand in for the block
// index, `waves` is the number of waves per workgroup that are given a KV head, `smem` the
// dynamic LDS.
template <int D, int R, bool KV8>
__device__ __forceinline__ void rows_body(const RowsParams& prm, int bx, int by, int bz, int waves,
                                          unsigned char* smem) {
  constexpr int EB = KV8 ? 1 : 2;
  using Geo = RowGeom<D, EB>;
  constexpr int ROWB = Geo::ROWB, CPR = Geo::CPR, TPI = Geo::TPI, IPB = Geo::IPB, KS = Geo::KS, DB = Geo::DB;

  const AttnArgs& a = prm.a;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
  const int lane = (int)threadIdx.x % kWave;
  const int kvh = by * waves + wave;
  if (wave >= waves || kvh >= a.Hkv) return;                      // no workgroup barrier below: safe
  const int h0 = kvh * prm.G + bz * kRowHeads;   // first query head of this wave
  const int nh = min(kRowHeads, prm.G - bz * kRowHeads);

  const int item = prm.w.item_order[bx];         // workgroups are dispatched longest item first
  const int4 rec = prm.w.item_rec[item];         // {seq, qtok, ctx, part | nparts << 16}
  const int bid0 = prm.w.item_blk0[item];        // id of the partition's first block
  const int qtok = rec.y;
  const int ctx = rec.z;
  const int part = rec.w & 0xffff;
  const int nparts = (int)((uint32_t)rec.w >> 16);
  const int32_t* table = a.block_tables + (int64_t)rec.x * a.max_blocks;

  const int t0 = part * prm.part_tokens;
  const int t1 = min(ctx, t0 + prm.part_tokens);
  const int b0 = t0 / kBlockSize;
  const int b1 = (t1 + kBlockSize - 1) / kBlockSize;   // b1 - b0 <= 64 (part_tokens <= 1024)

  const int qcol = lane % 16;                    // query head within the wave (MFMA column)
  const int jj = lane / 16;                      // lane group

  // Block ids of the partition: lane i holds the id of block b0+i; a uniform readlane hands one
  // to the address computation.
  const int tab_vec = table[min(b0 + lane, b1 - 1)];

  // Query fragments, B operand of S^T = K Q^T: lane (head qcol, jj) holds dims 32*ks + 8*jj .. +8.
  bf16x8_t qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (qcol < nh)
      v = *reinterpret_cast<const uint4*>(a.q + ((int64_t)qtok * a.Hq + h0 + qcol) * D + ks * 32 + jj * 8);
    qf[ks] = __builtin_bit_cast(bf16x8_t, v);
  }

  // ---- loader: lane l fills 16-byte position l of each 1 KiB piece of the slot ----
  unsigned char* const ring = smem + (size_t)wave * R * Geo::SLOT_BYTES;
  const int ld_row = lane / CPR;                 // token row inside a piece
  const int ld_pos = lane % CPR;                 // chunk position inside the row
  const uint32_t tok_stride = (uint32_t)a.Hkv * ROWB;       // bytes between token slots
  const int64_t blk_bytes = (int64_t)kBlockSize * tok_stride;
  const unsigned char* const k_bytes = reinterpret_cast<const unsigned char*>(a.k_pool);
  const unsigned char* const v_bytes = reinterpret_cast<const unsigned char*>(a.v_pool);
  const unsigned char* const zero_line = reinterpret_cast<const unsigned char*>(prm.w.zero_line);
  const int blast = b1 - 1;
  auto issue_block_id = [&](int bid, int b, int slot) {
    const unsigned char* kb = k_bytes + (int64_t)bid * blk_bytes + (uint32_t)kvh * ROWB;
    const unsigned char* vb = v_bytes + (int64_t)bid * blk_bytes + (uint32_t)kvh * ROWB;
    unsigned char* ks_base = ring + slot * Geo::SLOT_BYTES;
    unsigned char* vs_base = ks_base + Geo::TENSOR_BYTES;
#pragma unroll
    for (int i = 0; i < IPB; ++i) {
      const int n = i * TPI + ld_row;            // token slot in the block
      const unsigned char* kp = kb + (uint32_t)n * tok_stride + ((ld_pos ^ k_swz<D, EB>(n)) * 16);
      const unsigned char* vp = vb + (uint32_t)n * tok_stride + ((ld_pos ^ v_swz<D, EB>(n)) * 16);
      if (b * kBlockSize + n >= t1) vp = zero_line + ld_pos * 16;    // beyond the partition: V := 0
      if (b > blast) kp = zero_line + ld_pos * 16;                   // a refill nobody reads (see the loop)
      __builtin_amdgcn_global_load_lds((gbl_void_t)kp, (lds_void_t)(ks_base + i * 1024), 16, 0, kStreamOnce);
      __builtin_amdgcn_global_load_lds((gbl_void_t)vp, (lds_void_t)(vs_base + i * 1024), 16, 0, kStreamOnce);
    }
  };
  auto issue_block = [&](int b, int slot) {
    issue_block_id(__builtin_amdgcn_readlane(tab_vec, min(b, blast) - b0), b, slot);
  };

  // ---- per-lane state: lane (qcol, jj) owns head qcol; O^T rows are dims 16*db + 4*jj + e ----
  f32x4_t o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) o[db] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = kMinusBig, l_run = 0.f;
  const float scale = a.scale_log2e;

  // LDS read offsets (bytes) inside a slot.
  // K fragment (A operand, rows = tokens): lane (token qcol, jj) reads dims 32*ks + 8*jj .. +8,
  // 16 bytes of bf16 or 8 bytes of codes.
  int k_off[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    if constexpr (KV8)
      k_off[ks] = qcol * ROWB + (((ks * 2 + jj / 2) ^ k_swz<D, EB>(qcol)) * 16) + (jj % 2) * 8;
    else
      k_off[ks] = qcol * ROWB + (((ks * 4 + jj) ^ k_swz<D, EB>(qcol)) * 16);
  }
  // V^T fragment by transpose read: the 16 lanes of group jj fetch token rows 4jj..4jj+3 x 32
  // bytes, i.e. 16 dims of bf16, or 32 dims of codes (a 16-bit unit is then a pair of dims).
  constexpr int VT = KV8 ? DB / 2 : DB;                  // transpose reads per block
  const int v_row = jj * 4 + (lane % 16) / 4;
  const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring;
  uint32_t v_off[VT];
#pragma unroll
  for (int db = 0; db < VT; ++db)
    v_off[db] = Geo::TENSOR_BYTES + v_row * ROWB + (((2 * db + (lane % 4) / 2) ^ v_swz<D, EB>(v_row)) * 16) + (lane % 2) * 8;

  // The first block is requested at once (its id came with the item); the table slice and the
  // query rows are only waited for where they are first used.
  issue_block_id(bid0, b0, 0);
#pragma unroll
  for (int u = 1; u + 1 < R; ++u) issue_block(b0 + u, u);

  for (int b = b0; b < b1; ++b) {
    const int slot = (b - b0) % R;
    // Refill the slot consumed in the previous step (unconditionally, so that the number of
    // loads in flight is static), then wait until only the R-1 younger blocks are outstanding.
    // Past the partition's last block the refill is never consumed: it reads the zero line (a
    // cached 256 bytes) instead of fetching the last block from HBM once more.
    issue_block(b + R - 1, (b - b0 + R - 1) % R);
    wait_vmcnt<(R - 1) * Geo::LOADS_PER_BLOCK>();
    row_block_step<D, KV8>(ring_lds + (uint32_t)slot * Geo::SLOT_BYTES, k_off, v_off, qf, b * kBlockSize + jj * 4, t1,
                           scale, o, m_run, l_run);
  }
  wait_vmcnt<0>();                               // drain the (duplicate) prefetches before exit

  const float l_tot = cross16_sum(l_run);
  if (qcol >= nh) return;
  const int h = h0 + qcol;
  // Lane (head qcol, jj) holds, for every 16-dim block db, the dims 16db + 4jj + e (bf16 cache),
  // or, for every 32-dim block j, the dims 32j + 8jj + 2e (+1) in o[2j] (o[2j+1]) (code cache).
  if (nparts == 1) {
    const float inv = a.out_scale / l_tot;
    if constexpr (KV8) {
      const int64_t ob = ((int64_t)qtok * a.Hq + h) * D + jj * 8;
#pragma unroll
      for (int j = 0; j < DB / 2; ++j) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) { x[2 * e] = o[2 * j][e] * inv; x[2 * e + 1] = o[2 * j + 1][e] * inv; }
        if (a.out_bf16) {
          uint4 pk;
          pk.x = (uint32_t)f32_to_bf16_rne(x[0]) | ((uint32_t)f32_to_bf16_rne(x[1]) << 16);
          pk.y = (uint32_t)f32_to_bf16_rne(x[2]) | ((uint32_t)f32_to_bf16_rne(x[3]) << 16);
          pk.z = (uint32_t)f32_to_bf16_rne(x[4]) | ((uint32_t)f32_to_bf16_rne(x[5]) << 16);
          pk.w = (uint32_t)f32_to_bf16_rne(x[6]) | ((uint32_t)f32_to_bf16_rne(x[7]) << 16);
          *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(a.out) + ob + j * 32) = pk;
        } else {
          float* dst = reinterpret_cast<float*>(a.out) + ob + j * 32;
          *reinterpret_cast<float4*>(dst) = make_float4(x[0], x[1], x[2], x[3]);
          *reinterpret_cast<float4*>(dst + 4) = make_float4(x[4], x[5], x[6], x[7]);
        }
      }
    } else {
      const int64_t ob = ((int64_t)qtok * a.Hq + h) * D + jj * 4;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const float x0 = o[db][0] * inv, x1 = o[db][1] * inv, x2 = o[db][2] * inv, x3 = o[db][3] * inv;
        if (a.out_bf16) {
          uint2 pk;
          pk.x = (uint32_t)f32_to_bf16_rne(x0) | ((uint32_t)f32_to_bf16_rne(x1) << 16);
          pk.y = (uint32_t)f32_to_bf16_rne(x2) | ((uint32_t)f32_to_bf16_rne(x3) << 16);
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + ob + db * 16) = pk;
        } else {
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out) + ob + db * 16) = make_float4(x0, x1, x2, x3);
        }
      }
    }
  } else {
    // Partials leave with the nontemporal hint: written once, read once by the merge kernel.
    // Plain stores of these 16 KiB per item cost the K/V stream a tenth of its rate on long
    // contexts (config 5: 58 MB of partials next to 14.6 GB read: 6.26 TB/s; with the hint 6.60;
    // with every item's partials aimed at one cached spot, a timing experiment, 6.96).
    const int64_t ph = (int64_t)item * a.Hq + h;
    if constexpr (KV8) {
      f32x4_t* pa = reinterpret_cast<f32x4_t*>(prm.w.part_acc + ph * D + jj * 8);
#pragma unroll
      for (int j = 0; j < DB / 2; ++j) {
        __builtin_nontemporal_store(f32x4_t{o[2 * j][0], o[2 * j + 1][0], o[2 * j][1], o[2 * j + 1][1]}, pa + j * 8);
        __builtin_nontemporal_store(f32x4_t{o[2 * j][2], o[2 * j + 1][2], o[2 * j][3], o[2 * j + 1][3]}, pa + j * 8 + 1);
      }
    } else {
      f32x4_t* pa = reinterpret_cast<f32x4_t*>(prm.w.part_acc + ph * D + jj * 4);
#pragma unroll
      for (int db = 0; db < DB; ++db) __builtin_nontemporal_store(o[db], pa + db * 4);
    }
    if (jj == 0) *reinterpret_cast<float2*>(prm.w.part_ml + ph * 2) = make_float2(m_run, l_tot);
  }
}

}  // namespace rows_impl
}  // namespace dsv
