// Launcher of the prefill-tile kernel (see attn_prefill_kernel.h for the kernel itself).
#include <stdlib.h>

#include "attn_prefill_kernel16.h"

namespace dsv {
namespace {
using namespace prefill_impl;

template <int D>
__global__ __launch_bounds__(kThreads, kThreads / 256) void prefill_tiles_kernel(TilesParams prm) {
  extern __shared__ __align__(16) unsigned char smem[];
  int bx, bz;
  tile_work_item(blockIdx.x, prm.a.Hkv, prm.head_groups, bx, bz);
  prefill_tiles_item<D>(prm, bx, bz, smem);
}

template <int D>
__global__ __launch_bounds__(kThreads, kThreads / 256) void prefill_tiles_persistent_kernel(TilesParams prm) {
  extern __shared__ __align__(16) unsigned char smem[];
  // (The parameters are the kernel's only argument: they start the argument segment.)
  prefill_tiles_persistent<D>(prm, (params_ptr)__builtin_amdgcn_kernarg_segment_ptr(), (int)blockIdx.x,
                              (int)gridDim.x, smem);
}

// The same persistent grid on the 16x16x32 MFMA (head_dim 128).
__global__ __launch_bounds__(kThreads, kThreads / 256) void prefill_tiles_persistent16_kernel(TilesParams prm) {
  extern __shared__ __align__(16) unsigned char smem[];
  prefill_tiles_persistent16<128>(prm, (params_ptr)__builtin_amdgcn_kernarg_segment_ptr(), (int)blockIdx.x,
                                  (int)gridDim.x, smem);
}

int launch_persistent16(const TilesParams& prm, int grid, hipStream_t stream) {
  static OncePerDevice once;            // raising the dynamic-LDS limit is idempotent; races are benign
  bool* const configured = once.flag();
  if (!configured) return DSV_E_LAUNCH;
  if (!*configured) {
    hipFuncAttributes fa;               // no static LDS: the ring must start at LDS address 0
    if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(prefill_tiles_persistent16_kernel)) != hipSuccess ||
        fa.sharedSizeBytes != 0)
      return DSV_E_LAUNCH;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_tiles_persistent16_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, TileGeom<128>::LDS_BYTES_PERSISTENT) != hipSuccess)
      return DSV_E_LAUNCH;
    *configured = true;
  }
  hipLaunchKernelGGL(prefill_tiles_persistent16_kernel, dim3((unsigned)grid), dim3(kThreads), TileGeom<128>::LDS_BYTES_PERSISTENT,
                     stream, prm);
  return launch_status();
}

template <int D>
int launch_persistent_t(const TilesParams& prm, int grid, hipStream_t stream) {
  static OncePerDevice once;       // raising the dynamic-LDS limit is idempotent; races are benign
  bool* const configured = once.flag();
  if (!configured) return DSV_E_LAUNCH;
  if (!*configured) {
    hipFuncAttributes fa;               // no static LDS: the ring must start at LDS address 0
    if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(prefill_tiles_persistent_kernel<D>)) != hipSuccess ||
        fa.sharedSizeBytes != 0)
      return DSV_E_LAUNCH;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_tiles_persistent_kernel<D>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, TileGeom<D>::LDS_BYTES_PERSISTENT) != hipSuccess)
      return DSV_E_LAUNCH;
    *configured = true;
  }
  hipLaunchKernelGGL((prefill_tiles_persistent_kernel<D>), dim3((unsigned)grid), dim3(kThreads), TileGeom<D>::LDS_BYTES_PERSISTENT,
                     stream, prm);
  return launch_status();
}

template <int D>
int launch_t(const TilesParams& prm, dim3 grid, hipStream_t stream) {
  static OncePerDevice once;       // raising the dynamic-LDS limit is idempotent; races are benign
  bool* const configured = once.flag();
  if (!configured) return DSV_E_LAUNCH;
  if (!*configured) {
    // The kernel steps through its LDS ring by address bits: the ring must start at LDS
    // address 0, i.e. the kernel must have no static LDS in front of the dynamic part.
    hipFuncAttributes fa;
    if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(prefill_tiles_kernel<D>)) != hipSuccess ||
        fa.sharedSizeBytes != 0)
      return DSV_E_LAUNCH;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_tiles_kernel<D>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, TileGeom<D>::LDS_BYTES) != hipSuccess)
      return DSV_E_LAUNCH;
    *configured = true;
  }
  hipLaunchKernelGGL((prefill_tiles_kernel<D>), grid, dim3(kThreads), TileGeom<D>::LDS_BYTES, stream, prm);
  return launch_status();
}

}  // namespace

int launch_prefill_tiles(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg,
                         const PlanCounts& n, hipStream_t stream) {
  if (cfg.tile_tokens < 32 || cfg.tile_tokens > kTileQ) return DSV_E_UNSUPPORTED;
  const TilesParams prm = make_tiles_params(a, w, cfg, n);
  const int64_t wgs = n.tiles * a.Hkv * cfg.head_groups;
  if (wgs > 0x7fffffffLL) return DSV_E_UNSUPPORTED;
  const char* e = getenv("DSV_TILES_PERSISTENT");
  if (!e || atoi(e) != 0) {
    int cus = cfg.num_cus;
    if (const char* g = getenv("DSV_TILES_WGS")) cus = max(1, min(cus, atoi(g)));     // experiments: fewer workgroups
    const int grid = persistent_grid(cus, a.Hkv, n.tiles * cfg.head_groups);
    if (a.D == 128) return launch_persistent16(prm, grid, stream);
    if (a.D == 64) return launch_persistent_t<64>(prm, grid, stream);
    return DSV_E_UNSUPPORTED;
  }
  dim3 grid((unsigned)wgs);
  if (a.D == 128) return launch_t<128>(prm, grid, stream);
  if (a.D == 64) return launch_t<64>(prm, grid, stream);
  return DSV_E_UNSUPPORTED;
}

}  // namespace dsv
