// Launcher of the row kernel (see attn_rows_kernel.h for the kernel itself).
#include "attn_rows_kernel.h"
#include "attn_rows_stream.h"

namespace dsv {
namespace {
using namespace rows_impl;

template <int D, int R, bool KV8>
__global__ __launch_bounds__(512) void rows_kernel(RowsParams prm) {
  extern __shared__ __align__(16) unsigned char smem[];
  int bx, by, bz;
  row_work_item(blockIdx.x, prm.gy, prm.G, bx, by, bz);
  rows_body<D, R, KV8>(prm, bx, by, bz, (int)(blockDim.x / kWave), smem);
}

template <int D, int R, bool KV8>
int launch_rows_t(const RowsParams& prm, dim3 grid, int waves, hipStream_t stream) {
  const int lds = waves * R * RowGeom<D, KV8 ? 1 : 2>::SLOT_BYTES;
  // The dynamic-LDS limit is raised once per instantiation, to the most any geometry can ask for
  // (eight waves' rings), so that no later call - one inside a stream capture, with more KV heads
  // than the first call had - has to touch the kernel's attributes again.
  constexpr int kMaxLds = 8 * R * RowGeom<D, KV8 ? 1 : 2>::SLOT_BYTES <= 160 * 1024
                              ? 8 * R * RowGeom<D, KV8 ? 1 : 2>::SLOT_BYTES
                              : 4 * R * RowGeom<D, KV8 ? 1 : 2>::SLOT_BYTES;
  static OncePerDevice once;     // idempotent; a race between two first calls is benign
  bool* const configured = once.flag();
  if (!configured) return DSV_E_LAUNCH;
  if (lds > kMaxLds) return DSV_E_UNSUPPORTED;
  if (!*configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(rows_kernel<D, R, KV8>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) != hipSuccess)
      return DSV_E_LAUNCH;
    *configured = true;
  }
  hipLaunchKernelGGL((rows_kernel<D, R, KV8>), grid, dim3(waves * kWave), lds, stream, prm);
  return launch_status();
}

// Stream form: one persistent workgroup per run of the row stream, one wave per KV head.
template <int D, bool KV8>
__global__ __launch_bounds__(512) void rows_stream_kernel(RowsParams prm) {
  extern __shared__ __align__(16) unsigned char smem[];
  rows_stream_body<D, KV8>(prm, (int)blockIdx.x, smem);
}

template <int D, bool KV8>
int launch_rows_stream_t(const RowsParams& prm, int wgs, int waves, hipStream_t stream) {
  constexpr int kSlot = RowGeom<D, KV8 ? 1 : 2>::SLOT_BYTES;
  constexpr int kQStage = RowGeom<D, KV8 ? 1 : 2>::KS * 1024;      // per wave: its query fragments
  constexpr int kMaxLds = 8 * (2 * kSlot + kQStage);
  static OncePerDevice once;     // idempotent; a race between two first calls is benign
  bool* const configured = once.flag();
  if (!configured) return DSV_E_LAUNCH;
  if (!*configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(rows_stream_kernel<D, KV8>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) != hipSuccess)
      return DSV_E_LAUNCH;
    *configured = true;
  }
  hipLaunchKernelGGL((rows_stream_kernel<D, KV8>), dim3((unsigned)wgs), dim3(waves * kWave), waves * (2 * kSlot + kQStage), stream, prm);
  return launch_status();
}

}  // namespace

int launch_rows(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg, const PlanCounts& n,
                hipStream_t stream) {
  if (cfg.part_tokens > 64 * kBlockSize) return DSV_E_UNSUPPORTED;   // one table vector per partition
  RowsParams prm{a, w, cfg.part_tokens, a.Hq / a.Hkv, 1};
  if (cfg.stream_wgs > 0) {
    if (a.Hkv > 8 || prm.G > kRowHeads) return DSV_E_UNSUPPORTED;      // the planner does not choose it then
    if (a.D == 128 && !a.kv8) return launch_rows_stream_t<128, false>(prm, cfg.stream_wgs, a.Hkv, stream);
    if (a.D == 128 && a.kv8) return launch_rows_stream_t<128, true>(prm, cfg.stream_wgs, a.Hkv, stream);
    if (a.D == 64 && !a.kv8) return launch_rows_stream_t<64, false>(prm, cfg.stream_wgs, a.Hkv, stream);
    if (a.D == 64 && a.kv8) return launch_rows_stream_t<64, true>(prm, cfg.stream_wgs, a.Hkv, stream);
    return DSV_E_UNSUPPORTED;
  }
  int waves = 1;
  // waves * slots * slot bytes (8 KiB of bf16, 4 KiB of codes) must fit in the 160 KB of LDS
  const int max_waves = cfg.row_nbuf <= (a.kv8 ? 4 : 2) ? 8 : 4;
  int cap = max_waves;
  if (const char* e = getenv("DSV_ROW_WAVES")) cap = min(max_waves, max(1, atoi(e)));
  while (waves < a.Hkv && waves < cap) waves <<= 1;
  prm.gy = ceil_div(a.Hkv, waves);
  const int64_t wgs = n.items * prm.gy * ceil_div(prm.G, kRowHeads);
  if (wgs > 0x7fffffffLL) return DSV_E_UNSUPPORTED;
  dim3 grid((unsigned)wgs);
  const int r = cfg.row_nbuf;
#define DSV_ROWS_CASE(DD, RR, KK) \
  if (a.D == DD && r == RR && (a.kv8 != 0) == KK) return launch_rows_t<DD, RR, KK>(prm, grid, waves, stream);
  DSV_ROWS_CASE(128, 2, false) DSV_ROWS_CASE(128, 3, false) DSV_ROWS_CASE(128, 4, false)
  DSV_ROWS_CASE(64, 2, false) DSV_ROWS_CASE(64, 3, false) DSV_ROWS_CASE(64, 4, false)
  DSV_ROWS_CASE(128, 2, true) DSV_ROWS_CASE(128, 4, true) DSV_ROWS_CASE(128, 8, true)
  DSV_ROWS_CASE(64, 2, true) DSV_ROWS_CASE(64, 4, true) DSV_ROWS_CASE(64, 8, true)
#undef DSV_ROWS_CASE
  return DSV_E_UNSUPPORTED;
}

}  // namespace dsv
