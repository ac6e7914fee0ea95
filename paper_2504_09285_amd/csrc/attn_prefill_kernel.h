// Attention of long prefill spans on the matrix cores ("tile" work).
//
// A prefill span of a mixed batch is q_len new tokens that resume on ctx_len-q_len cached
// tokens (paper section 3.1, micro-requests) and attend causally over prefix and new tokens
// alike, all read from the paged pool.  This is the compute-bound part of a step (paper
// sections 2.1, 4.2): QK^T and PV are dense contractions and run on bf16 MFMA with fp32
// accumulation and an online softmax.
//
// Work item: (span, 64 consecutive query tokens, KV head, group of 4 query heads).  One
// workgroup of eight waves per item, two per SIMD, so that one wave's MFMAs run while the other
// does its softmax on the vector ALU; wave w takes query tokens 32*(w/4)..+32 of query head
// w%4 of the group (32 query rows).  All eight share every K/V tile in LDS.
//
// K/V tiles of 64 tokens (four 16-token blocks gathered through the block table, half a block
// per wave) go straight from global memory into a ring of four LDS buffers with direct loads;
// tile t+3 is requested while tile t is used.  One workgroup barrier per tile.  The ring starts
// at LDS address 0 (the kernel owns no static LDS; the launchers check), so the fragment read
// addresses step from buffer to buffer by an XOR of two address bits.
//
// (This header holds the tile geometry, the ring, the helpers and the body built on the 32x32x16
// MFMA, which serves head_dim 64; head_dim 128 runs the same schedule on the 16x16x32 MFMA:
// attn_prefill_kernel16.h, attn_prefill_persistent16.h.)
//
// The products are computed transposed, S^T = K Q^T and O^T = V^T P^T, with the 32x32x16 MFMA:
//   - the query row is the MFMA column, so a lane owns one query row for the whole kernel: row
//     max / sum / rescale are per-lane scalars (one exchange with the lane holding the other 16
//     tokens of the row);
//   - S^T comes out with lane (row j, half h) holding tokens 8a+4h+b (a,b = 0..3) of a 32-token
//     sub-tile, which is a valid B operand of the next MFMA once the contraction index (token)
//     of the A operand V^T is enumerated in the same order: P never leaves registers;
//   - V^T as A operand needs, per lane, consecutive tokens of one dim while memory is
//     dim-contiguous: the LDS transpose read (ds_read_b64_tr_b16) delivers that from the natural
//     [token][dim] layout.  LDS rows are XOR-swizzled at load time (each lane chooses which
//     16 bytes of a row it fetches) so that both kinds of fragment reads are conflict-free.
//
// The loop over 32-token sub-tiles is software-pipelined: stage s issues the MFMAs for the scores
// of sub-tile s+1 and for V^T P^T of sub-tile s-1 together with the softmax of sub-tile s, one
// basic block whose instructions interleave; the fragment reads from LDS roll along with the
// MFMAs that consume them.  LDS reads are written in assembly: the compiler cannot know which
// bytes the direct loads in flight will write and would drain all of them before every read.
//
// A first, fast pass keeps the softmax reference of a row fixed after its first sub-tile (no
// per-stage row max, no accumulator rescale); if a row sum leaves the safe range the workgroup
// repeats its work item in a robust pass with the usual running max.
//
// Scores are kept in the log2 domain.  Slots past the span's context (pool garbage) are fetched
// from a line of zeros instead, and masked scores are excluded by select, so NaN/Inf there
// cannot leak.
#pragma once
#include "attn_internal.h"

#include <type_traits>

namespace dsv {
namespace prefill_impl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef uint32_t __attribute__((ext_vector_type(4))) u32x4_t;
typedef uint32_t __attribute__((ext_vector_type(2))) u32x2_t;
typedef __attribute__((address_space(3))) void* lds_void_t;
typedef const __attribute__((address_space(1))) void* gbl_void_t;

constexpr int kTileQ = 64;        // query tokens per work item
constexpr int kTileKV = 64;       // KV tokens per LDS tile
constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kWave;
constexpr int NH = 1;             // query heads (32-row MFMA columns) per wave
constexpr int kWavesPerBlock = kWaves / (kTileKV / kBlockSize);   // waves sharing the fetch of one KV block
constexpr int kHeadWaves = 4 / NH;                                 // waves that cover a group of four query heads
constexpr int kRing = 4;          // LDS tile buffers
constexpr float kMinusBig = -1.0e30f;
constexpr float kMaxSlack = 8.0f;
constexpr float kSumLimit = 1.0e19f;   // about 2^63: far from the fp32 range, reached only by extreme inputs

struct TilesParams {
  AttnArgs a;
  WorkLists w;
  int32_t num_tiles;
  int32_t G;
  const int32_t* stage_rows;   // null, or [num_seqs]: row of a.block_tables that serves a segment
                               // (a cache of 8-bit codes is attended through a bf16 copy of the
                               // spans' contexts with a table of its own)
  int32_t tile_q;              // query tokens per work item (64, or 256 / flat_heads)
  int32_t flat_heads;          // see PlanConfig
  int32_t head_groups;
  int32_t flat_magic;          // ceil(65536 / flat_heads) (0 if flat_heads is 0): see flat_div()
};

// Row r (< 256) of a flat work item is the pair (token r / gh, head r % gh).  The quotient comes
// from a multiplication, not from the thirty-odd instructions of an integer division (the row
// geometry is worked out for a dozen rows at every item boundary, where no MFMA hides it): with
// magic = ceil(65536 / gh), (r * magic) >> 16 == r / gh for every r < 256 and gh < 256.
__host__ __device__ inline int flat_div(int r, int magic) { return (r * magic) >> 16; }

// Parameters of a launch over the tile list.  A cache of 8-bit codes is attended through the
// staged bf16 copy of the spans' contexts and its own block table.
inline TilesParams make_tiles_params(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg,
                                     const PlanCounts& n) {
  TilesParams prm{a, w, (int32_t)n.tiles, a.Hq / a.Hkv, nullptr, cfg.tile_tokens, cfg.flat_heads, cfg.head_groups,
                  cfg.flat_heads > 0 ? (65536 + cfg.flat_heads - 1) / cfg.flat_heads : 0};
  if (a.kv8) {
    prm.a.k_pool = w.stage_k;
    prm.a.v_pool = w.stage_v;
    prm.a.block_tables = w.stage_table;
    prm.a.max_blocks = n.stage_max_blocks;
    prm.a.kv8 = 0;
    prm.stage_rows = w.stage_rows;
  }
  return prm;
}

template <int D>
struct TileGeom {
  static constexpr int KS = D / 16;          // MFMA k-steps of K Q^T
  static constexpr int DB = D / 32;          // 32-dim blocks of O^T
  static constexpr int ROWB = D * 2;         // bytes per token row of one head
  static constexpr int CPR = D / 8;          // 16-byte chunks per row
  static constexpr int RPP = kWave / CPR;    // token rows per 1 KiB load piece
  static constexpr int PPB = kBlockSize / RPP;       // pieces per 16-token block
  static constexpr int TENSOR_BYTES = kTileKV * ROWB;
  static constexpr int TILE_BYTES = 2 * TENSOR_BYTES;
  static constexpr int RING_BYTES = kRing * TILE_BYTES;
  static constexpr int LDS_BYTES = RING_BYTES + 16;  // the ring, then the workgroup's overflow flag
  // Persistent form: output rows are staged through LDS, 4 KiB per wave.  A tile buffer of that
  // size (head_dim 128) lends itself, being free at that moment; smaller ones (head_dim 64) get an
  // area of their own behind the flags.
  static constexpr int STAGE_BYTES = kWaves * 4096;
  static constexpr bool STAGE_IN_RING = TILE_BYTES >= STAGE_BYTES;
  static constexpr int STAGE_OFFSET = RING_BYTES + 256;
  static constexpr int LDS_BYTES_PERSISTENT = STAGE_IN_RING ? LDS_BYTES : STAGE_OFFSET + STAGE_BYTES;
  static constexpr int PPW = PPB / kWavesPerBlock;   // pieces per wave
  static constexpr int LOADS = 2 * PPW;      // direct loads per wave per tile (its share of a block of K and of V)
};

template <int CPR> __device__ __forceinline__ int k_swz(int row) { return row & (CPR - 1); }
// V: a transpose read covers 8 token rows x 64 bytes, and the LDS serves 32 lanes (4 rows x 64
// bytes = all 64 banks) per cycle, so rows that share banks must sit in different 64-byte
// groups: bits 2.. of the chunk index are swizzled by the row (measured with 8 waves reading:
// 2.8 cycles per read against 4.0 with a swizzle that only separates 32-byte pairs).
template <int CPR> __device__ __forceinline__ int v_swz(int row) {
  constexpr int GPR = CPR / 4;      // 64-byte groups per row
  constexpr int RW = 16 / CPR;      // rows per 256 bytes (one pass over the banks)
  return (4 * ((row / RW) % GPR)) ^ (2 * ((row >> 2) & 1));
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// LDS reads of data written by the direct loads.  A stage issues all its fragment reads back to
// back (lds_issue4_*), waits (lds_wait) and then passes every result through
// lds_ready4(): an empty asm that redefines the registers, so that no consumer can be scheduled
// ahead of the wait while the read results are still in flight.
// (OFF: byte offset carried in the instruction.)
template <int OFF>
__device__ __forceinline__ void lds_issue4_b128(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3,
                                                u32x4_t& v0, u32x4_t& v1, u32x4_t& v2, u32x4_t& v3) {
  asm volatile(
      "ds_read_b128 %0, %4 offset:%8\n\t"
      "ds_read_b128 %1, %5 offset:%8\n\t"
      "ds_read_b128 %2, %6 offset:%8\n\t"
      "ds_read_b128 %3, %7 offset:%8"
      : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3)
      : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "n"(OFF)
      : "memory");
}
// Two addresses, each read at byte offsets OFF and OFF + STEP (immediates of the instruction).
template <int OFF, int STEP>
__device__ __forceinline__ void lds_issue4_tr(uint32_t a0, uint32_t a1, u32x2_t& v0, u32x2_t& v1, u32x2_t& v2,
                                              u32x2_t& v3) {
  asm volatile(
      "ds_read_b64_tr_b16 %0, %4 offset:%6\n\t"
      "ds_read_b64_tr_b16 %1, %4 offset:%7\n\t"
      "ds_read_b64_tr_b16 %2, %5 offset:%6\n\t"
      "ds_read_b64_tr_b16 %3, %5 offset:%7"
      : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3)
      : "v"(a0), "v"(a1), "n"(OFF), "n"(OFF + STEP)
      : "memory");
}
// Waits until at most N of the LDS reads issued so far are outstanding (they complete in order,
// so all but the youngest N are in).  A scalar load in flight only makes the wait longer.
template <int N>
__device__ __forceinline__ void lds_wait() {
  static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void lds_ready4(u32x4_t& v0, u32x4_t& v1, u32x4_t& v2, u32x4_t& v3) {
  asm volatile("" : "+v"(v0), "+v"(v1), "+v"(v2), "+v"(v3));
}
__device__ __forceinline__ void lds_ready4(u32x2_t& v0, u32x2_t& v1, u32x2_t& v2, u32x2_t& v3) {
  asm volatile("" : "+v"(v0), "+v"(v1), "+v"(v2), "+v"(v3));
}

// acc + lo + hi of a packed bf16 pair.
__device__ __forceinline__ float sum2_bf16(uint32_t pair, float acc) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pair), __builtin_bit_cast(bf16x2_t, 0x3f803f80u),
                                         acc, false);
}

// Exchange with lane ^ 32: after v_permlane32_swap lo holds the value of the lower half-wave
// lane and hi that of the upper one, in both lanes.  Given the same value for both operands
// the compiler folds the two results into one, so the second operand is passed through an
// empty asm that hides where it came from.
__device__ __forceinline__ void half_swap(float x, float& lo, float& hi) {
  uint32_t a = __float_as_uint(x), b;
  asm("" : "=v"(b) : "0"(a));
  typedef unsigned int u32x2v __attribute__((ext_vector_type(2)));
  const u32x2v r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  lo = __uint_as_float(r[0]);
  hi = __uint_as_float(r[1]);
}
__device__ __forceinline__ float other_half_max(float x) {       // max with lane ^ 32
  float lo, hi;
  half_swap(x, lo, hi);
  return fmaxf(lo, hi);
}
__device__ __forceinline__ float other_half_sum(float x) {
  float lo, hi;
  half_swap(x, lo, hi);
  return lo + hi;
}

// Work item of the wg-th prefill workgroup.  The tile list is sorted heaviest first and
// workgroups are dispatched in index order, so the groups of query heads of one (tile, KV
// head) follow each other (all head groups of the heavy tiles start before any light tile),
// while the KV head stays the fastest index: with eight KV heads, eight consecutive workgroups
// go to the eight XCDs and KV head k always lands on XCD k.
__device__ __forceinline__ void tile_work_item(uint32_t wg, int Hkv, int head_groups, int& bx, int& bz) {
  const uint32_t nbz = (uint32_t)head_groups;
  const uint32_t kvh = wg % (uint32_t)Hkv, r = wg / (uint32_t)Hkv;
  bz = (int)(r % nbz);
  bx = (int)((r / nbz) * (uint32_t)Hkv + kvh);
}

// The kernel body as a device function, so that the same code serves the kernel of its own and
// the launch that mixes prefill tiles with row work.  bx = tile * Hkv + KV head and bz = group
// of four query heads stand in for the block index; `smem` is the dynamic LDS (LDS_BYTES).
template <int D>
__device__ __forceinline__ void prefill_tiles_body(const TilesParams& prm, int bx, int bz, unsigned char* smem) {
  using Geo = TileGeom<D>;
  constexpr int KS = Geo::KS, DB = Geo::DB, ROWB = Geo::ROWB, CPR = Geo::CPR, RPP = Geo::RPP, PPW = Geo::PPW;
  static_assert(KS % 4 == 0, "K fragments are fetched in groups of four");
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  const AttnArgs& a = prm.a;
  const int tid = (int)threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int lane = tid % kWave;
  const int jrow = lane % 32;            // query row of the wave (MFMA column) / token row of a K sub-tile
  const int hh = lane / 32;
  // Wave w runs on SIMD w % 4.  With four query heads per KV head, SIMD s hosts both halves of
  // the query tile for head s.  With one or two heads per KV head most head slots are empty
  // (their waves only fetch tiles): the waves that have rows are then spread over the SIMDs
  // instead of sharing SIMD 0 (and 1).
  const bool few_heads = prm.G - bz * 4 <= 2;
  const int tg = few_heads ? wave % 2 : wave / kHeadWaves;          // which 32 query tokens of the tile
  const int hp = few_heads ? wave / 2 : wave % kHeadWaves;          // which query head of the group of four
  // Flat rows (head groups that are not four heads): row r = 32 * wave + jrow of the work item is
  // the pair (token j0 + r / gh, head bz * gh + r % gh) of a group of gh heads; rows
  // tile_q * gh .. 255 do not exist.  Everything below that is per query row (its token's
  // position, its head's rows of Q and of the output) is per lane already.
  const int gh = prm.flat_heads;
  const bool flat = gh > 0;
  const int row_in_item = 32 * wave + jrow;
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

  // Query fragments: B operand of S^T = K Q^T; lane (jrow, hh) holds dims 16*ks + 8*hh .. +8.
  const int jq = flat ? j0 + flat_div(row_in_item, fmagic) : j0 + 32 * tg + jrow;    // new-token index of this lane's query row
  const int p_j = prefix + jq - pos0;    // its position, counted from the partition's first token
  // (wave-uniform) Does any of this wave's 32 query rows, for any of its heads, exist?
  const bool wave_has_rows = flat ? (j0 + wave_first_tok < q_len && 32 * wave < prm.tile_q * gh)
                                  : (j0 + 32 * tg < q_len && bz * 4 + hp * NH < prm.G);
  bool head_ok[NH];
  int head[NH];
  uint4 qf[NH][KS];
  static_assert(D * 2 <= 256, "a query row fits the zero line");
#pragma unroll
  for (int c = 0; c < NH; ++c) {
    const int hsub = flat ? bz * gh + (row_in_item - flat_div(row_in_item, fmagic) * gh) : bz * 4 + hp * NH + c;
    head_ok[c] = hsub < prm.G && jq < q_len && (!flat || row_in_item < prm.tile_q * gh);
    head[c] = kvh * prm.G + (hsub < prm.G ? hsub : 0);
    // A row that does not exist reads the zero line: the choice is made on the address, so the
    // loads stay in flight next to the tile requests below instead of being waited for here.
    const uint16_t* src = head_ok[c] ? a.q + (((int64_t)(q0 + jq) * a.Hq + head[c]) * D + hh * 8)
                                     : reinterpret_cast<const uint16_t*>(prm.w.zero_line) + hh * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[c][ks] = *reinterpret_cast<const uint4*>(src + ks * 16);
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
    v_src[ii] = ((uint32_t)n * tok_stride + (uint32_t)((pos ^ v_swz<CPR>(row)) * 8)) * 2u;
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
  // K fragment of sub-tile row jrow: chunk 2*ks + hh.  V^T fragment: 16 lanes fetch 4 token rows x
  // 16 dims; tokens 16*ks16 + 4*hh + (lane%16)/4 (+8 for the second read), dims 32*db + ...
  // The swizzles depend on row % 16 only, so fragments of other sub-tiles / k-steps are a
  // constant number of rows further on.
  uint32_t k_off[KS], v_off[DB];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_off[ks] = lds0 + jrow * ROWB + (((2 * ks + hh) ^ k_swz<CPR>(jrow)) * 16);
  {
    const int row = hh * 4 + (lane % 16) / 4;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int chunk = 4 * db + 2 * ((lane / 16) % 2) + (lane % 4) / 2;
      v_off[db] = lds0 + Geo::TENSOR_BYTES + row * ROWB + ((chunk ^ v_swz<CPR>(row)) * 16) + (lane % 2) * 8;
    }
  }

  f32x16_t o[NH][DB];
  float m_run[NH], l_run[NH];
  const float scale = a.scale_log2e;

  // The loop is software-pipelined over 32-token sub-tiles.  Stage s finds the scores of
  // sub-tile s already computed and, in one basic block, gives the matrix cores the scores of
  // sub-tile s+1 and O^T += V^T P^T of sub-tile s-1 while the vector ALU does the softmax of
  // sub-tile s: three independent pieces of work whose instructions interleave, so that the
  // softmax runs in the shadow of the MFMAs.  Scores and probabilities are double-buffered.
  f32x16_t scb[2][NH];
  uint4 pfb[2][NH][2];
  float corr[NH];
  bool any_corr;
  u32x4_t kf[KS];
  u32x2_t vf0[2][DB], vf1[2][DB];          // V^T fragments [k16][db]: tokens +0..3 and +8..11
  // Fragment addresses of the tile being read, K and V separately (the K reads run a tile ahead
  // of the V reads).  They are absolute LDS addresses, and the ring starts at LDS address 0 and
  // has four tile buffers, so stepping to the next buffer (0 -> 1 -> 2 -> 3 -> 0) is an XOR of the
  // two address bits above a tile with 1 or 3: one instruction per address register and tile,
  // where adding a buffer offset at every use cost one per register and sub-tile.  The offset of
  // the sub-tile inside the tile rides in the read instructions.
  static_assert(kRing == 4 && (Geo::TILE_BYTES & (Geo::TILE_BYTES - 1)) == 0, "XOR stepping of the ring");
  uint32_t k_adr[KS], v_adr[DB];
  auto ring_step = [&](int tile) __attribute__((always_inline)) {
    return (uint32_t)((tile & 1) ? 3 * Geo::TILE_BYTES : Geo::TILE_BYTES);
  };
  // K fragments of sub-tile s (its parity given as a constant); after the odd sub-tile the
  // addresses move on to the next tile.
  auto issue_k = [&](int s, auto odd_c) __attribute__((always_inline)) {
    constexpr int ODD = decltype(odd_c)::value;
#pragma unroll
    for (int g4 = 0; g4 < KS; g4 += 4)
      lds_issue4_b128<ODD * 32 * ROWB>(k_adr[g4], k_adr[g4 + 1], k_adr[g4 + 2], k_adr[g4 + 3],
                                       kf[g4], kf[g4 + 1], kf[g4 + 2], kf[g4 + 3]);
    if constexpr (ODD) {
      const uint32_t x = ring_step(s >> 1);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) k_adr[ks] ^= x;
    }
  };
  auto ready_k = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int g4 = 0; g4 < KS; g4 += 4) lds_ready4(kf[g4], kf[g4 + 1], kf[g4 + 2], kf[g4 + 3]);
  };
  auto issue_v = [&](int sv, auto odd_c, auto k16_c) __attribute__((always_inline)) {
    constexpr int ODD = decltype(odd_c)::value;
    constexpr int k16 = decltype(k16_c)::value;
#pragma unroll
    for (int d2 = 0; d2 < DB; d2 += 2)
      lds_issue4_tr<ODD * 32 * ROWB + k16 * 16 * ROWB, 8 * ROWB>(v_adr[d2], v_adr[d2 + 1], vf0[k16][d2], vf1[k16][d2],
                                                                 vf0[k16][d2 + 1], vf1[k16][d2 + 1]);
    if constexpr (ODD && k16 == 1) {
      const uint32_t x = ring_step(sv >> 1);
#pragma unroll
      for (int db = 0; db < DB; ++db) v_adr[db] ^= x;
    }
  };
  auto ready_v = [&](int k16) __attribute__((always_inline)) {
#pragma unroll
    for (int d2 = 0; d2 < DB; d2 += 2) lds_ready4(vf0[k16][d2], vf1[k16][d2], vf0[k16][d2 + 1], vf1[k16][d2 + 1]);
  };
  // S^T = K Q^T from the K fragments in kf.
  auto qk = [&](f32x16_t (&sc)[NH]) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < NH; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[c][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int c = 0; c < NH; ++c)
        sc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[ks]),
                                                        __builtin_bit_cast(bf16x8_t, qf[c][ks]), sc[c], 0, 0, 0);
  };
  // O^T += V^T P^T from the V^T fragments in vf0 / vf1.
  auto pv = [&](const uint4 (&pf)[NH][2], int k16) __attribute__((always_inline)) {
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const u32x4_t vv = {vf0[k16][db][0], vf0[k16][db][1], vf1[k16][db][0], vf1[k16][db][1]};
#pragma unroll
      for (int c = 0; c < NH; ++c)
        o[c][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vv),
                                                           __builtin_bit_cast(bf16x8_t, pf[c][k16]), o[c][db], 0, 0, 0);
    }
  };
  // Softmax of the scores in sc -> bf16 probabilities pf[c][k16] (B operand of V^T P^T), in one
  // of two modes.
  //  fast:   the reference value m of a row is the max of its first sub-tile and never changes,
  //          so there is no per-stage row max and no accumulator rescale: probabilities may
  //          grow far beyond 1, which fp32 sums and bf16 operands (same exponent range) hold
  //          without loss.  If a row sum passes kSumLimit (a later score exceeds the first
  //          sub-tile's max by about 60 in log2 units) or stops being a number, the wave
  //          reports it and the workgroup repeats the tile in robust mode.
  //  robust: the usual running max, except that m only follows the row max when it has grown
  //          by more than kMaxSlack (log2 units), so that the 64-register rescale of the
  //          accumulators is rare; corr[c] is the factor the accumulators of head c must be
  //          multiplied with before these probabilities join them.
  bool overflow = false;
  auto softmax = [&](f32x16_t (&sc)[NH], uint4 (&pf)[NH][2], auto robust_c, auto first_c) __attribute__((always_inline)) {
    constexpr bool robust = decltype(robust_c)::value;
    constexpr bool first = decltype(first_c)::value;
    any_corr = false;
#pragma unroll
    for (int c = 0; c < NH; ++c) {
      corr[c] = 1.0f;
      if constexpr (robust || first) {
        float mx = sc[c][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sc[c][r]);
        mx = other_half_max(mx);
        // (Clamped: a row may see no token of a context partition's first sub-tile, or of the
        // whole partition; its sum and accumulators then stay zero.)
        const float m_cand = fmaxf(mx * scale, kMinusBig);
        const float m_new = (first || m_cand > m_run[c] + kMaxSlack) ? m_cand : m_run[c];
        if constexpr (robust && !first) {
          corr[c] = __builtin_amdgcn_exp2f(m_run[c] - m_new);
          any_corr |= m_new != m_run[c];
        }
        m_run[c] = m_new;
      }
      const float m_ref = m_run[c];
      float t[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) t[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[c][r], scale, -m_ref));
#pragma unroll
      for (int k16 = 0; k16 < 2; ++k16) {
        pf[c][k16].x = pack_bf16(t[8 * k16 + 0], t[8 * k16 + 1]);
        pf[c][k16].y = pack_bf16(t[8 * k16 + 2], t[8 * k16 + 3]);
        pf[c][k16].z = pack_bf16(t[8 * k16 + 4], t[8 * k16 + 5]);
        pf[c][k16].w = pack_bf16(t[8 * k16 + 6], t[8 * k16 + 7]);
      }
      // Row sum over the rounded probabilities (the values V^T P^T really uses), two per
      // instruction: a bf16 dot product with (1, 1).
      float ps = robust ? l_run[c] * corr[c] : l_run[c];
#pragma unroll
      for (int k16 = 0; k16 < 2; ++k16) {
        ps = sum2_bf16(pf[c][k16].x, ps);
        ps = sum2_bf16(pf[c][k16].y, ps);
        ps = sum2_bf16(pf[c][k16].z, ps);
        ps = sum2_bf16(pf[c][k16].w, ps);
      }
      l_run[c] = ps;
      if constexpr (!robust) overflow |= !(ps < kSumLimit);
    }
  };
  auto rescale = [&](const float (&corr)[NH]) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < NH; ++c)
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[c][db][r] *= corr[c];
  };
  // Stage s; CUR = s % 2 selects the buffers.  On entry scb[CUR] holds S^T of sub-tile s,
  // pfb[CUR ^ 1] the probabilities of sub-tile s-1, and the K fragments of sub-tile s+1 are on
  // their way from LDS.  The fragment reads roll along with the MFMAs that consume them: the
  // first half of the V^T fragments is requested before the K Q^T MFMAs, the second half after
  // them, and the K fragments of sub-tile s+2 once their registers are free, so each read has
  // four or eight MFMAs (128-256 cycles) to arrive and no registers are double-buffered.
  // Even stages (s = 2u) hold the barrier of tile u: see next_tile().
  auto stage = [&](int s, auto cur_c, auto with_pv_c, auto robust_c, auto&& tile_sync) __attribute__((always_inline)) {
    constexpr int CUR = decltype(cur_c)::value;
    constexpr bool with_pv = decltype(with_pv_c)::value;
    constexpr bool robust = decltype(robust_c)::value;
    // The two waves of a SIMD (the two halves of the query tile, same head) take turns at the
    // higher issue priority, stage by stage: left to the default arbitration the older wave is
    // served first throughout and then idles at the tile barrier while the other finishes.
    if (flat ? wave / 4 : tg) __builtin_amdgcn_s_setprio(CUR); else __builtin_amdgcn_s_setprio(CUR ^ 1);
    if constexpr (with_pv) {
      issue_v(s - 1, std::integral_constant<int, CUR ^ 1>{}, std::integral_constant<int, 0>{});
      lds_wait<2 * DB>();                // the K fragments (older than these 2*DB reads) are in
    } else {
      lds_wait<0>();
    }
    ready_k();
    // Only sub-tiles that reach past some row's own position need the causal mask (a
    // wave-uniform branch, so the unmasked path pays one scalar compare).
    if (s * 32 + 31 > prefix + j0 + wave_first_tok - pos0) {
#pragma unroll
      for (int c = 0; c < NH; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (s * 32 + (r / 4) * 8 + hh * 4 + (r % 4) > p_j) scb[CUR][c][r] = -INFINITY;
    }
    // Robust mode: the accumulators take the correction found by the previous stage's softmax
    // before that stage's probabilities join them (a rare, wave-uniform branch kept out of the
    // block below).
    if constexpr (with_pv && robust) {
      if (__any(any_corr)) rescale(corr);
    }
    qk(scb[CUR ^ 1]);
    // The asm statements keep their order among themselves, but nothing orders them against
    // the MFMAs except registers: an empty asm that "writes" the last operand an MFMA group
    // reads cannot move above that group, and so anchors what follows it behind the group.
    asm volatile("" : "+v"(kf[KS - 1]));
    if constexpr (with_pv) {
      issue_v(s - 1, std::integral_constant<int, CUR ^ 1>{}, std::integral_constant<int, 1>{});
      lds_wait<2 * DB>();                // first half of V^T in
      ready_v(0);
      pv(pfb[CUR ^ 1], 0);
      asm volatile("" : "+v"(vf1[0][DB - 1]));
    }
    if constexpr (CUR == 0) {
      lds_wait<0>();                     // this wave's last read of tile u-1 is complete
      tile_sync();
      issue_k(s + 2, std::integral_constant<int, CUR>{});
    } else {
      issue_k(s + 2, std::integral_constant<int, CUR>{});
      lds_wait<KS>();                    // second half of V^T in (the K reads may be in flight)
    }
    if constexpr (with_pv) {
      ready_v(1);
      pv(pfb[CUR ^ 1], 1);
    }
    softmax(scb[CUR], pfb[CUR], robust_c, std::integral_constant<bool, !with_pv>{});
    // Ask the scheduler for one MFMA followed by a handful of vector-ALU instructions, repeated:
    // the softmax then runs in the shadow of the matrix-core work of the same wave.
#pragma unroll
    for (int i = 0; i < (with_pv ? 2 * KS : KS); ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                  // MFMA
      __builtin_amdgcn_sched_group_barrier(0x402, with_pv ? (robust ? 6 : 4) : 12, 0);    // VALU or transcendental
    }
    // The probabilities are pinned to this block (an empty asm that "uses" them): otherwise
    // the compiler sinks the exponentials to their first use, past the next stage's branches,
    // where no MFMA is left to hide them.
#pragma unroll
    for (int c = 0; c < NH; ++c)
#pragma unroll
      for (int k16 = 0; k16 < 2; ++k16)
        asm volatile("" ::"v"(pfb[CUR][c][k16].x), "v"(pfb[CUR][c][k16].y), "v"(pfb[CUR][c][k16].z),
                     "v"(pfb[CUR][c][k16].w));
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
    for (int c = 0; c < NH; ++c) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[c][db][r] = 0.f;
      m_run[c] = kMinusBig;
      l_run[c] = 0.f;
    }
    any_corr = false;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_adr[ks] = k_off[ks];
#pragma unroll
    for (int db = 0; db < DB; ++db) v_adr[db] = v_off[db];
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
    for (int c = 0; c < NH; ++c)
  #pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        asm volatile("" : "+v"(qf[c][ks].x), "+v"(qf[c][ks].y), "+v"(qf[c][ks].z), "+v"(qf[c][ks].w));

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
  // Any wave that saw a row sum leave the safe range makes the whole workgroup (the tile
  // requests and barriers are collective) repeat the work item in robust mode.
  if (__any(overflow) && lane == 0) wg_overflow = 1;
  __syncthreads();
  if (wg_overflow) attend(std::true_type{});

  // Output.  A lane holds its query row's values four dims at a time, 32 rows per wave: stored as
  // they are, every store instruction would touch 32 rows with 16 or 32 bytes each.  The values go
  // through LDS instead (the ring is free: every request has landed and every wave is past its
  // last fragment read; 4 KiB per wave), 32 rows x 128 bytes per pass, and come back as eight rows x
  // 128 contiguous bytes per store instruction: whole cache lines.  Staged rows are XOR-swizzled by
  // 16-byte chunk so that neither side has bank conflicts.
  // A cut q-tile writes unnormalised partials (accumulators, and the reference / sum pair per row
  // and head) for the merge kernel; token j of the tile, partition p -> partial
  // first + j * partitions + p.  An uncut one writes the normalised output, fp32 or bf16.
  static_assert(NH == 1 && kWaves * 4096 <= Geo::RING_BYTES, "one head per wave; the staging area fits the ring");
  __syncthreads();
  {
    const float l_tot = other_half_sum(l_run[0]);
    if (!wave_has_rows) return;                                   // (wave-uniform)
    const bool partial = nparts > 1;
    const int first_partial = partial ? prm.w.tile_item0[tile] : -1;
    const float inv = partial ? 1.0f : a.out_scale / l_tot;
    if (partial && head_ok[0] && hh == 0) {
      const int64_t ph = ((int64_t)first_partial + (int64_t)(jq - j0) * nparts + part) * a.Hq + head[0];
      *reinterpret_cast<float2*>(prm.w.part_ml + ph * 2) = make_float2(m_run[0], l_tot);
    }
    const uint32_t stage = lds0 + (uint32_t)wave * 4096u;
    const uint32_t w_row = stage + (uint32_t)jrow * 128u;
    const uint32_t w_swz = (uint32_t)((jrow >> 1) & 7);
    const int rr = lane / 8, ch = lane % 8;               // reading side: chunk ch of rows rr + 8 * pass
    uint32_t r_adr[4];
    int64_t r_dst[4];                                             // element offset of the row in its destination
    bool r_ok[4];
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
      const int row = ps * 8 + rr;
      r_adr[ps] = stage + (uint32_t)row * 128u + (uint32_t)((ch ^ ((row >> 1) & 7)) * 16);
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
      float* const dst = partial ? prm.w.part_acc : reinterpret_cast<float*>(a.out);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
#pragma unroll
        for (int aa = 0; aa < 4; ++aa) {
          const u32x4_t v = {__float_as_uint(o[0][db][aa * 4 + 0] * inv), __float_as_uint(o[0][db][aa * 4 + 1] * inv),
                             __float_as_uint(o[0][db][aa * 4 + 2] * inv), __float_as_uint(o[0][db][aa * 4 + 3] * inv)};
          const uint32_t adr = w_row + (((uint32_t)(aa * 2 + hh) ^ w_swz) * 16u);
          asm volatile("ds_write_b128 %0, %1" ::"v"(adr), "v"(v) : "memory");
        }
        u32x4_t r0, r1, r2, r3;
        lds_issue4_b128<0>(r_adr[0], r_adr[1], r_adr[2], r_adr[3], r0, r1, r2, r3);   // (LDS serves a wave in order)
        lds_wait<0>();
        lds_ready4(r0, r1, r2, r3);
        const u32x4_t rv[4] = {r0, r1, r2, r3};
#pragma unroll
        for (int ps = 0; ps < 4; ++ps)
          if (r_ok[ps]) *reinterpret_cast<u32x4_t*>(dst + r_dst[ps] + db * 32 + ch * 4) = rv[ps];
      }
    } else {
      uint16_t* const dst = reinterpret_cast<uint16_t*>(a.out);
#pragma unroll
      for (int dp = 0; dp < DB; dp += 2) {
#pragma unroll
        for (int dl = 0; dl < 2; ++dl)
#pragma unroll
          for (int aa = 0; aa < 4; ++aa) {
            const int db = dp + dl;
            const u32x2_t v = {pack_bf16(o[0][db][aa * 4 + 0] * inv, o[0][db][aa * 4 + 1] * inv),
                               pack_bf16(o[0][db][aa * 4 + 2] * inv, o[0][db][aa * 4 + 3] * inv)};
            const uint32_t adr = w_row + (((uint32_t)(dl * 4 + aa) ^ w_swz) * 16u) + (uint32_t)hh * 8u;
            asm volatile("ds_write_b64 %0, %1" ::"v"(adr), "v"(v) : "memory");
          }
        u32x4_t r0, r1, r2, r3;
        lds_issue4_b128<0>(r_adr[0], r_adr[1], r_adr[2], r_adr[3], r0, r1, r2, r3);
        lds_wait<0>();
        lds_ready4(r0, r1, r2, r3);
        const u32x4_t rv[4] = {r0, r1, r2, r3};
#pragma unroll
        for (int ps = 0; ps < 4; ++ps)
          if (r_ok[ps]) *reinterpret_cast<u32x4_t*>(dst + r_dst[ps] + dp * 32 + ch * 8) = rv[ps];
      }
    }
  }
}

}  // namespace prefill_impl
}  // namespace dsv
