// Single-query-token attention over a paged KV cache, split along the context ("row" work).
//
// Serves the decode tokens of a mixed batch - one new token attending to its whole cached
// context, the memory-bound part of a step (paper sections 2.1 and 4.2) - and the tokens of
// prefill spans too short for the MFMA kernel.  A work item is (query token, context
// partition); a workgroup takes one item and gives each of its waves one KV head, so that the
// waves of a workgroup together stream whole 16-token blocks (all heads of a block are
// contiguous in the pool).
//
// Inside a wave a token's head row (D bf16) is spread over D/8 lanes, 16 bytes each, so one
// load instruction covers 64/(D/8) tokens with fully used cache lines.  Each group of lanes
// that shares a token slot keeps its own online-softmax state (running max m, sum l, acc) over
// the tokens it sees; the groups are merged once, at the end of the partition.  All G query
// heads that share the KV head are processed against the same loaded K/V registers.
// Scores live in the log2 domain (scale*log2(e) folded into the dot product, exp2 for exp).
#include "attn_internal.h"

namespace dsv {
namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

constexpr float kMinusBig = -1.0e30f;    // finite stand-in for "no token seen yet"

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL,
                                                               0xf, 0xf, true));
}

// Sum over the LPT (8 or 16) adjacent lanes that hold one token's row; result in every lane.
template <int LPT>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_move<0xB1>(x);     // quad_perm [1,0,3,2]
  x += dpp_move<0x4E>(x);     // quad_perm [2,3,0,1]
  x += dpp_move<0x141>(x);    // row_half_mirror: lane i <-> 7-i
  if (LPT == 16) x += dpp_move<0x140>(x);   // row_mirror: lane i <-> 15-i
  return x;
}

__device__ __forceinline__ float dot8(const uint4& a, const uint4& b, float acc) {
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.x), __builtin_bit_cast(bf16x2_t, b.x), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.y), __builtin_bit_cast(bf16x2_t, b.y), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.z), __builtin_bit_cast(bf16x2_t, b.z), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w), __builtin_bit_cast(bf16x2_t, b.w), acc, false);
  return acc;
}

__device__ __forceinline__ void unpack8(const uint4& u, float (&f)[8]) {
  f[0] = __builtin_bit_cast(float, u.x << 16); f[1] = __builtin_bit_cast(float, u.x & 0xffff0000u);
  f[2] = __builtin_bit_cast(float, u.y << 16); f[3] = __builtin_bit_cast(float, u.y & 0xffff0000u);
  f[4] = __builtin_bit_cast(float, u.z << 16); f[5] = __builtin_bit_cast(float, u.z & 0xffff0000u);
  f[6] = __builtin_bit_cast(float, u.w << 16); f[7] = __builtin_bit_cast(float, u.w & 0xffff0000u);
}

template <int D, int GT>
struct RowState {
  static constexpr int LPT = D / 8;          // lanes per token row
  static constexpr int TPL = kWave / LPT;    // tokens per load instruction
  static constexpr int LPB = kBlockSize / TPL;   // load instructions per block (per K, per V)
  float m[GT], l[GT], acc[GT][8];
};

// One 16-token block.  tok0 = absolute position of the block's slot 0; grp = this lane's token
// sub-slot; MASKED: slots at positions >= ctx are excluded by select (pool garbage, possibly
// NaN/Inf, must not leak: neither through the score nor through 0 * V).
template <int D, int GT, bool MASKED>
__device__ __forceinline__ void process_block(RowState<D, GT>& st, const uint4 (&kreg)[RowState<D, GT>::LPB],
                                              const uint4 (&vreg)[RowState<D, GT>::LPB],
                                              const uint4 (&qreg)[GT], float scale, int tok0, int grp,
                                              int ctx) {
  constexpr int LPT = RowState<D, GT>::LPT, TPL = RowState<D, GT>::TPL, LPB = RowState<D, GT>::LPB;
  float s[LPB][GT];
#pragma unroll
  for (int i = 0; i < LPB; ++i) {
    const bool valid = !MASKED || (tok0 + grp + TPL * i < ctx);
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      const float d = group_sum<LPT>(dot8(qreg[g], kreg[i], 0.f));
      s[i][g] = valid ? d * scale : -INFINITY;
    }
  }
  float corr[GT], p[LPB][GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    float mb = s[0][g];
#pragma unroll
    for (int i = 1; i < LPB; ++i) mb = fmaxf(mb, s[i][g]);
    const float mn = fmaxf(st.m[g], mb);
    corr[g] = exp2f(st.m[g] - mn);
    st.m[g] = mn;
    float ps = 0.f;
#pragma unroll
    for (int i = 0; i < LPB; ++i) {
      p[i][g] = exp2f(s[i][g] - mn);
      ps += p[i][g];
    }
    st.l[g] = st.l[g] * corr[g] + ps;
#pragma unroll
    for (int d = 0; d < 8; ++d) st.acc[g][d] *= corr[g];
  }
#pragma unroll
  for (int i = 0; i < LPB; ++i) {
    uint4 vr = vreg[i];
    if (MASKED && !(tok0 + grp + TPL * i < ctx)) vr = make_uint4(0u, 0u, 0u, 0u);
    float v[8];
    unpack8(vr, v);
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
      for (int d = 0; d < 8; ++d) st.acc[g][d] += p[i][g] * v[d];
  }
}

struct RowsParams {
  AttnArgs a;
  WorkLists w;
  int32_t part_tokens;
  int32_t G;            // query heads per KV head
};

template <int D, int GT>
__global__ __launch_bounds__(512) void rows_kernel(RowsParams prm) {
  using St = RowState<D, GT>;
  constexpr int LPT = St::LPT, TPL = St::TPL, LPB = St::LPB;
  const AttnArgs& a = prm.a;
  const int wave = (int)threadIdx.x / kWave;
  const int lane = (int)threadIdx.x % kWave;
  const int kvh = blockIdx.y * (blockDim.x / kWave) + wave;
  if (kvh >= a.Hkv) return;                      // no workgroup barrier below: safe
  const int h0 = kvh * prm.G + blockIdx.z * GT;  // first query head of this wave
  const int nh = min(GT, prm.G - (int)blockIdx.z * GT);

  const int item = blockIdx.x;
  const int r = prm.w.item_row[item];
  const int part = prm.w.item_part[item];
  const int qtok = prm.w.row_qtok[r];
  const int ctx = prm.w.row_ctx[r];
  const int nparts = prm.w.row_nparts[r];
  const int32_t* table = a.block_tables + (int64_t)prm.w.row_seq[r] * a.max_blocks;

  const int t0 = part * prm.part_tokens;
  const int t1 = min(ctx, t0 + prm.part_tokens);
  const int b0 = t0 / kBlockSize;
  const int b1 = (t1 + kBlockSize - 1) / kBlockSize;

  const int col = lane % LPT;                    // which 8 dims of the row
  const int grp = lane / LPT;                    // which token sub-slot

  uint4 qreg[GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    qreg[g] = make_uint4(0u, 0u, 0u, 0u);
    if (g < nh)
      qreg[g] = *reinterpret_cast<const uint4*>(a.q + ((int64_t)qtok * a.Hq + h0 + g) * D + col * 8);
  }

  St st;
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    st.m[g] = kMinusBig;
    st.l[g] = 0.f;
#pragma unroll
    for (int d = 0; d < 8; ++d) st.acc[g][d] = 0.f;
  }

  const int64_t tok_stride = (int64_t)a.Hkv * D;            // elements between token slots
  const int64_t lane_off = (int64_t)grp * tok_stride + (int64_t)kvh * D + col * 8;
  auto load_block = [&](int b, uint4 (&kr)[LPB], uint4 (&vr)[LPB]) {
    const int64_t base = (int64_t)table[b] * kBlockSize * tok_stride + lane_off;
#pragma unroll
    for (int i = 0; i < LPB; ++i) {
      const int64_t off = base + (int64_t)(TPL * i) * tok_stride;
      kr[i] = *reinterpret_cast<const uint4*>(a.k_pool + off);
      vr[i] = *reinterpret_cast<const uint4*>(a.v_pool + off);
    }
  };
  auto consume = [&](int b, const uint4 (&kr)[LPB], const uint4 (&vr)[LPB]) {
    const int tok0 = b * kBlockSize;
    if (tok0 + kBlockSize <= t1)
      process_block<D, GT, false>(st, kr, vr, qreg, a.scale_log2e, tok0, grp, t1);
    else
      process_block<D, GT, true>(st, kr, vr, qreg, a.scale_log2e, tok0, grp, t1);
  };

  // Two register buffers: the next block's loads are in flight while the current one is used.
  uint4 kA[LPB], vA[LPB], kB[LPB], vB[LPB];
  load_block(b0, kA, vA);
  for (int b = b0; b < b1; b += 2) {
    if (b + 1 < b1) load_block(b + 1, kB, vB);
    consume(b, kA, vA);
    if (b + 1 < b1) {
      if (b + 2 < b1) load_block(b + 2, kA, vA);
      consume(b + 1, kB, vB);
    }
  }

  // Merge the TPL token-slot groups of the wave.
#pragma unroll
  for (int off = LPT; off < kWave; off <<= 1) {
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      const float mo = __shfl_xor(st.m[g], off);
      const float lo = __shfl_xor(st.l[g], off);
      const float mn = fmaxf(st.m[g], mo);
      const float c0 = exp2f(st.m[g] - mn), c1 = exp2f(mo - mn);
      st.l[g] = st.l[g] * c0 + lo * c1;
#pragma unroll
      for (int d = 0; d < 8; ++d) st.acc[g][d] = st.acc[g][d] * c0 + __shfl_xor(st.acc[g][d], off) * c1;
      st.m[g] = mn;
    }
  }

  if (grp != 0) return;
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    if (g >= nh) break;
    const int h = h0 + g;
    if (nparts == 1) {
      const float inv = 1.0f / st.l[g];
      const int64_t o = ((int64_t)qtok * a.Hq + h) * D + col * 8;
      if (a.out_bf16) {
        uint4 pk;
        pk.x = f32_to_bf16_rne(st.acc[g][0] * inv) | ((uint32_t)f32_to_bf16_rne(st.acc[g][1] * inv) << 16);
        pk.y = f32_to_bf16_rne(st.acc[g][2] * inv) | ((uint32_t)f32_to_bf16_rne(st.acc[g][3] * inv) << 16);
        pk.z = f32_to_bf16_rne(st.acc[g][4] * inv) | ((uint32_t)f32_to_bf16_rne(st.acc[g][5] * inv) << 16);
        pk.w = f32_to_bf16_rne(st.acc[g][6] * inv) | ((uint32_t)f32_to_bf16_rne(st.acc[g][7] * inv) << 16);
        *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(a.out) + o) = pk;
      } else {
        float4* op = reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out) + o);
        op[0] = make_float4(st.acc[g][0] * inv, st.acc[g][1] * inv, st.acc[g][2] * inv, st.acc[g][3] * inv);
        op[1] = make_float4(st.acc[g][4] * inv, st.acc[g][5] * inv, st.acc[g][6] * inv, st.acc[g][7] * inv);
      }
    } else {
      const int64_t ph = (int64_t)item * a.Hq + h;
      float4* op = reinterpret_cast<float4*>(prm.w.part_acc + ph * D + col * 8);
      op[0] = make_float4(st.acc[g][0], st.acc[g][1], st.acc[g][2], st.acc[g][3]);
      op[1] = make_float4(st.acc[g][4], st.acc[g][5], st.acc[g][6], st.acc[g][7]);
      if (col == 0) *reinterpret_cast<float2*>(prm.w.part_ml + ph * 2) = make_float2(st.m[g], st.l[g]);
    }
  }
}

template <int D, int GT>
void launch_rows_t(const RowsParams& prm, dim3 grid, int threads, hipStream_t stream) {
  hipLaunchKernelGGL((rows_kernel<D, GT>), grid, dim3(threads), 0, stream, prm);
}

}  // namespace

int launch_rows(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg, const PlanCounts& n,
                hipStream_t stream) {
  RowsParams prm{a, w, cfg.part_tokens, a.Hq / a.Hkv};
  int waves = 1;
  while (waves < a.Hkv && waves < 8) waves <<= 1;
  int gt = 1;
  while (gt < prm.G && gt < 8) gt <<= 1;
  dim3 grid((unsigned)n.items, (unsigned)ceil_div(a.Hkv, waves), (unsigned)ceil_div(prm.G, gt));
  const int threads = waves * kWave;
#define DSV_ROWS_CASE(DD, GG) \
  if (a.D == DD && gt == GG) { launch_rows_t<DD, GG>(prm, grid, threads, stream); return launch_status(); }
  DSV_ROWS_CASE(128, 1) DSV_ROWS_CASE(128, 2) DSV_ROWS_CASE(128, 4) DSV_ROWS_CASE(128, 8)
  DSV_ROWS_CASE(64, 1) DSV_ROWS_CASE(64, 2) DSV_ROWS_CASE(64, 4) DSV_ROWS_CASE(64, 8)
#undef DSV_ROWS_CASE
  return DSV_E_UNSUPPORTED;
}

}  // namespace dsv
