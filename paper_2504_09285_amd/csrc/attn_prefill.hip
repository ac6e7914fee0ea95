// Attention of long prefill spans on the matrix cores ("tile" work).
//
// A prefill span of a mixed batch is q_len new tokens that resume on ctx_len-q_len cached
// tokens (paper section 3.1, micro-requests) and attend causally over prefix and new tokens
// alike, all read from the paged pool.  This is the compute-bound part of a step (paper
// sections 2.1, 4.2): QK^T and PV are dense contractions and run on bf16 MFMA with fp32
// accumulation and an online softmax.
//
// Work item: (span, 32 consecutive query tokens, KV head).  The four waves of a workgroup take
// the (up to) four query heads that share that KV head, so every K/V tile staged in LDS is used
// by all of them.  K/V tiles of 64 tokens (four 16-token blocks, gathered through the block
// table) are double-buffered in LDS: the global loads of tile i+1 are issued before the math of
// tile i and written to the other buffer after it.
//
// The products are computed transposed, S^T = K Q^T and O^T = V^T P^T, with the 32x32x16 MFMA:
//   - the query row is then the MFMA *column*, so a lane owns one query row for the whole
//     kernel: row max / sum / rescale are per-lane scalars (one cross-lane exchange with the
//     lane that holds the other 16 tokens of the row);
//   - S^T comes out with lane (row j, half h) holding tokens 8a+4h+b (a,b = 0..3) of a 32-token
//     sub-tile, which is exactly a valid B operand for the next MFMA once the contraction index
//     (token) of the A operand V^T is enumerated in the same order.  P never leaves registers.
//   - V^T as A operand needs, per lane, consecutive tokens of one dim, while memory is
//     dim-contiguous: the LDS transpose read (ds_read_b64_tr_b16) delivers that from the
//     natural [token][dim] layout.
// Scores are kept in the log2 domain.  Slots past the span's context (pool garbage) are zeroed
// while V is staged, and masked scores are excluded by select, so NaN/Inf there cannot leak.
#include "attn_internal.h"

namespace dsv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;

constexpr int kTileQ = 32;        // query tokens per work item
constexpr int kTileKV = 64;       // KV tokens per LDS tile
constexpr int kThreads = 256;
constexpr float kMinusBig = -1.0e30f;

struct TilesParams {
  AttnArgs a;
  WorkLists w;
  int32_t num_tiles;
  int32_t G;
};

template <int D>
struct TileGeom {
  static constexpr int KS = D / 16;          // MFMA k-steps of QK^T
  static constexpr int DB = D / 32;          // 32-dim blocks of O^T
  static constexpr int KSTR = D + 8;         // LDS row stride of K (elements): spreads b128 reads over banks
  static constexpr int VSTR = D + 16;        // LDS row stride of V: spreads the 4-row transpose reads
  static constexpr int UPR = D / 8;          // 16-byte units per token row
  static constexpr int UPT = kTileKV * UPR / kThreads;   // units staged per thread per tile
  static constexpr int LDS_BYTES = 2 * kTileKV * (KSTR + VSTR) * 2;
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

// Two fp32 -> packed bf16, round to nearest even (the hardware conversion of gfx950).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <int D>
__global__ __launch_bounds__(kThreads, 2) void prefill_tiles_kernel(TilesParams prm) {
  using Geo = TileGeom<D>;
  constexpr int KS = Geo::KS, DB = Geo::DB, KSTR = Geo::KSTR, VSTR = Geo::VSTR, UPR = Geo::UPR, UPT = Geo::UPT;
  extern __shared__ __align__(16) uint16_t smem[];
  uint16_t* const ksm0 = smem;
  uint16_t* const vsm0 = smem + 2 * kTileKV * KSTR;

  const AttnArgs& a = prm.a;
  const int tid = (int)threadIdx.x;
  const int wave = tid / kWave, lane = tid % kWave;
  const int jrow = lane % 32;            // query row of the tile (MFMA column) / token row of a K sub-tile
  const int hh = lane / 32;

  // Heaviest tiles (late tiles of late spans) first.
  const int tile = prm.num_tiles - 1 - (int)blockIdx.x;
  const int seq = prm.w.tile_seq[tile];
  const int j0 = prm.w.tile_q0[tile];
  const int q0 = a.q_offsets[seq];
  const int q_len = a.q_offsets[seq + 1] - q0;
  const int ctx = a.ctx_lens[seq];
  const int prefix = ctx - q_len;
  const int kvh = blockIdx.y;
  const int hsub = (int)blockIdx.z * 4 + wave;
  const bool head_ok = hsub < prm.G;
  const int head = kvh * prm.G + (head_ok ? hsub : 0);
  const int32_t* table = a.block_tables + (int64_t)seq * a.max_blocks;
  const int nblk = (ctx + kBlockSize - 1) / kBlockSize;
  const int kv_end = min(ctx, prefix + j0 + kTileQ);          // exclusive: last visible token + 1
  const int n_kv_tiles = (kv_end + kTileKV - 1) / kTileKV;

  // Query fragments: B operand of S^T = K Q^T; lane (jrow, hh) holds dims 16*ks + 8*hh .. +8.
  const bool q_ok = head_ok && (j0 + jrow < q_len);
  const int64_t q_row_off = ((int64_t)(q0 + j0 + (q_ok ? jrow : 0)) * a.Hq + head) * D;
  bf16x8_t qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (q_ok) v = *reinterpret_cast<const uint4*>(a.q + q_row_off + ks * 16 + hh * 8);
    qf[ks] = __builtin_bit_cast(bf16x8_t, v);
  }
  const int p_j = prefix + j0 + jrow;    // absolute position of this lane's query row

  // ---- staging: global -> registers -> LDS ----
  uint4 kst[UPT], vst[UPT];
  auto gload = [&](int kt) {
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const int u = tid + kThreads * k;
      const int tok = u / UPR, col = u % UPR;
      const int b = kt * (kTileKV / kBlockSize) + tok / kBlockSize;
      kst[k] = make_uint4(0u, 0u, 0u, 0u);
      vst[k] = make_uint4(0u, 0u, 0u, 0u);
      if (b < nblk) {
        const int64_t off = (((int64_t)table[b] * kBlockSize + tok % kBlockSize) * a.Hkv + kvh) * D + col * 8;
        kst[k] = *reinterpret_cast<const uint4*>(a.k_pool + off);
        if (kt * kTileKV + tok < ctx) vst[k] = *reinterpret_cast<const uint4*>(a.v_pool + off);
      }
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const int u = tid + kThreads * k;
      const int tok = u / UPR, col = u % UPR;
      *reinterpret_cast<uint4*>(ksm0 + buf * kTileKV * KSTR + tok * KSTR + col * 8) = kst[k];
      *reinterpret_cast<uint4*>(vsm0 + buf * kTileKV * VSTR + tok * VSTR + col * 8) = vst[k];
    }
  };

  f32x16_t o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = kMinusBig, l_run = 0.f;
  const float scale = a.scale_log2e;

  gload(0);
  sstore(0);
  __syncthreads();

  for (int kt = 0; kt < n_kv_tiles; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < n_kv_tiles;
    if (more) gload(kt + 1);

    const uint16_t* ksm = ksm0 + cur * kTileKV * KSTR;
    const uint16_t* vsm = vsm0 + cur * kTileKV * VSTR;
    const int T = kt * kTileKV;
    const bool two = T + 32 < kv_end;                 // second 32-token sub-tile has visible tokens
    const bool need_mask = T + kTileKV - 1 > prefix + j0;

    // S^T = K Q^T for the two 32-token sub-tiles.
    f32x16_t s[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
      if (sub == 0 || two) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(ksm + (sub * 32 + jrow) * KSTR + ks * 16 + hh * 8);
          s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[sub], 0, 0, 0);
        }
      }
    }

    // Online softmax; lane owns query row jrow and tokens T + 32*sub + 8a + 4hh + b.
    // The row max is taken on raw scores (softmax_scale > 0), the scale is folded into the
    // exp2 argument: p = 2^(s*scale - m).
    if (need_mask || !two) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int t = T + sub * 32 + (r / 4) * 8 + hh * 4 + (r % 4);
          if (t > p_j || (sub == 1 && !two)) s[sub][r] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sub][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx * scale);
    if (__any(m_new > m_run)) {
      const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= corr;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= corr;
      m_run = m_new;
    }
    float psum = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[sub][r], scale, -m_run));
        s[sub][r] = p;
        psum += p;
      }
    l_run += psum;

    // O^T += V^T P^T, 16 tokens per k-step.
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      if (s4 >= 2 && !two) break;
      const int sub = s4 / 2, a0 = (s4 % 2) * 8;
      uint4 pk;
      pk.x = pack_bf16(s[sub][a0 + 0], s[sub][a0 + 1]);
      pk.y = pack_bf16(s[sub][a0 + 2], s[sub][a0 + 3]);
      pk.z = pack_bf16(s[sub][a0 + 4], s[sub][a0 + 5]);
      pk.w = pack_bf16(s[sub][a0 + 6], s[sub][a0 + 7]);
      const bf16x8_t pf = __builtin_bit_cast(bf16x8_t, pk);
      // transpose reads: 16 lanes fetch 4 token rows x 16 dims; lane gets 4 tokens of its dim
      const int trow = s4 * 16 + hh * 4 + (lane % 16) / 4;
      const int tcol = ((lane / 16) % 2) * 16 + (lane % 4) * 4;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        typedef __attribute__((address_space(3))) s16x4_t* lds_ptr_t;
        const uint16_t* p0 = vsm + trow * VSTR + db * 32 + tcol;
        const s16x4_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p0));
        const s16x4_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p0 + 8 * VSTR));
        const s16x8_t vv = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vv), pf, o[db], 0, 0, 0);
      }
    }

    if (more) sstore(cur ^ 1);
    __syncthreads();
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (!q_ok) return;
  const float inv = 1.0f / l_tot;
  const int64_t o_row = ((int64_t)(q0 + j0 + jrow) * a.Hq + head) * D;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int aa = 0; aa < 4; ++aa) {
      const int dim = db * 32 + aa * 8 + hh * 4;
      const float x0 = o[db][aa * 4 + 0] * inv, x1 = o[db][aa * 4 + 1] * inv;
      const float x2 = o[db][aa * 4 + 2] * inv, x3 = o[db][aa * 4 + 3] * inv;
      if (a.out_bf16) {
        uint2 pk;
        pk.x = pack_bf16(x0, x1);
        pk.y = pack_bf16(x2, x3);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + o_row + dim) = pk;
      } else {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out) + o_row + dim) = make_float4(x0, x1, x2, x3);
      }
    }
}

template <int D>
int launch_t(const TilesParams& prm, dim3 grid, hipStream_t stream) {
  static bool configured = false;       // raising the dynamic-LDS limit is idempotent; races are benign
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_tiles_kernel<D>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, TileGeom<D>::LDS_BYTES) != hipSuccess)
      return DSV_E_LAUNCH;
    configured = true;
  }
  hipLaunchKernelGGL((prefill_tiles_kernel<D>), grid, dim3(kThreads), TileGeom<D>::LDS_BYTES, stream, prm);
  return launch_status();
}

}  // namespace

int launch_prefill_tiles(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg,
                         const PlanCounts& n, hipStream_t stream) {
  if (cfg.tile_tokens != kTileQ) return DSV_E_UNSUPPORTED;
  TilesParams prm{a, w, (int32_t)n.tiles, a.Hq / a.Hkv};
  dim3 grid((unsigned)n.tiles, (unsigned)a.Hkv, (unsigned)ceil_div(prm.G, 4));
  if (a.D == 128) return launch_t<128>(prm, grid, stream);
  if (a.D == 64) return launch_t<64>(prm, grid, stream);
  return DSV_E_UNSUPPORTED;
}

}  // namespace dsv
