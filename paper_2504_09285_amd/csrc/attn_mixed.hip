// One launch for a batch that holds both kinds of work: prefill tiles (matrix-core bound) and
// row items (HBM bound).  The paper runs prefill and decode tokens of a step in one hybrid
// launch and observes that mixing them raises utilisation (sections 4.2 and 4.4); here the two
// kernels' workgroups are dealt out in one grid, in alternating groups sized in proportion to
// their counts, so that from the first moment some compute units stream KV for the decodes
// while the others run MFMAs for the prefill spans, instead of one kernel waiting for the
// other's tail.  A workgroup runs exactly one of the two kernel bodies; both are written for
// 512 threads and about 128 KiB of LDS, so a compute unit holds one workgroup of either kind.
//
// Groups are eight consecutive workgroups: the hardware deals consecutive workgroups to the
// eight XCDs in turn, so a group of tile workgroups still puts KV head k on XCD k (see
// attn_prefill_kernel.h), and heaviest-first tile order is kept.
#include "attn_prefill_kernel16.h"
#include "attn_rows_kernel.h"
#include "attn_rows_stream.h"

namespace dsv {
namespace {

constexpr int kGroup = 8;

struct MixParams {
  uint32_t tile_wgs;        // prefill workgroups: tiles * Hkv * ceil(G / 4)
  uint32_t tiles_x;         // tiles * Hkv (the prefill kernel's x extent)
  uint32_t row_wgs;         // row workgroups: items * rows_y * rows_z
  uint32_t rows_x, rows_y;  // the row kernel's x and y extents
  uint32_t tile_groups, total_groups;
  int32_t rows_waves;
};

template <int D, bool KV8>
__global__ __launch_bounds__(512, 2) void mixed_kernel(prefill_impl::TilesParams tp,
                                                       rows_impl::RowsParams rp, MixParams mp) {
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t g = blockIdx.x / kGroup, lane_in_group = blockIdx.x % kGroup;
  // Group g is a tile group iff the running count of tile groups steps at g.
  // (Measured on configs 3 and 4: spreading the tile groups evenly over the whole grid beats
  // packing them towards the front or giving the row groups a head start.)
  const uint32_t t0 = (uint32_t)((uint64_t)g * mp.tile_groups / mp.total_groups);
  const uint32_t t1 = (uint32_t)((uint64_t)(g + 1) * mp.tile_groups / mp.total_groups);
  if (t1 != t0) {
    const uint32_t wg = t0 * kGroup + lane_in_group;
    if (wg >= mp.tile_wgs) return;                               // uniform for the workgroup
    int bx, bz;
    prefill_impl::tile_work_item(wg, tp.a.Hkv, tp.head_groups, bx, bz);
    prefill_impl::prefill_tiles_item<D>(tp, bx, bz, smem);
  } else {
    const uint32_t wg = (g - t0) * kGroup + lane_in_group;
    if (wg >= mp.row_wgs) return;
    int bx, by, bz;
    rows_impl::row_work_item(wg, rp.gy, rp.G, bx, by, bz);
    rows_impl::rows_body<D, 2, KV8>(rp, bx, by, bz, mp.rows_waves, smem);
  }
}

template <int D, bool KV8>
int launch_mixed_t(const prefill_impl::TilesParams& tp, const rows_impl::RowsParams& rp,
                   const MixParams& mp, int lds, hipStream_t stream) {
  // Raised once, to the most either body can ask for (eight row waves with two ring slots each,
  // or the tile ring), so that no later call has to touch the kernel's attributes again.
  constexpr int kRowsMax = 8 * 2 * rows_impl::RowGeom<D, KV8 ? 1 : 2>::SLOT_BYTES;
  constexpr int kMaxLds = kRowsMax > (int)prefill_impl::TileGeom<D>::LDS_BYTES ? kRowsMax
                                                                              : (int)prefill_impl::TileGeom<D>::LDS_BYTES;
  static OncePerDevice once;     // idempotent; a race between two first calls is benign
  bool* const configured = once.flag();
  if (!configured) return DSV_E_LAUNCH;
  if (lds > kMaxLds) return DSV_E_UNSUPPORTED;
  if (!*configured) {
    hipFuncAttributes fa;               // no static LDS: the tile body's ring must start at LDS address 0
    if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(mixed_kernel<D, KV8>)) != hipSuccess ||
        fa.sharedSizeBytes != 0)
      return DSV_E_LAUNCH;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(mixed_kernel<D, KV8>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) != hipSuccess)
      return DSV_E_LAUNCH;
    *configured = true;
  }
  hipLaunchKernelGGL((mixed_kernel<D, KV8>), dim3(mp.total_groups * kGroup), dim3(512), lds, stream, tp, rp, mp);
  return launch_status();
}

// The other way to share the device: the row work as persistent streams (attn_rows_stream.h) on
// the first row_wgs workgroups, which the hardware places first and which keep their compute
// units to the end of the launch, and the tiles' workgroups behind them, one item each, going
// through the remaining compute units as those free up.  Chosen by the planner for batches whose
// row part is large (config 4: 128 decodes next to a 4,096-token prompt); row_wgs is a multiple
// of eight, so a tile workgroup's KV head still falls on XCD (workgroup index mod 8).
// (Measured on config 4, per step: this form 0.65 ms with 144-160 row streams; the interleaved
// groups above 0.70 ms; persistent tile workgroups on the remaining compute units instead of one
// workgroup per item 0.64 ms at their best split and 0.69-0.89 ms when the split is off by a few
// streams, since tiles that stay put cannot take over the compute units of streams that end:
// not kept.)
template <int D, bool KV8>
__global__ __launch_bounds__(512, 2) void mixed_stream_kernel(prefill_impl::TilesParams tp,
                                                              rows_impl::RowsParams rp, uint32_t row_wgs) {
  extern __shared__ __align__(16) unsigned char smem[];
  if (blockIdx.x < row_wgs) {
    rows_impl::rows_stream_body<D, KV8>(rp, (int)blockIdx.x, smem);
  } else {
    int bx, bz;
    prefill_impl::tile_work_item(blockIdx.x - row_wgs, tp.a.Hkv, tp.head_groups, bx, bz);
    prefill_impl::prefill_tiles_item<D>(tp, bx, bz, smem);
  }
}

template <int D, bool KV8>
int launch_mixed_stream_t(const prefill_impl::TilesParams& tp, const rows_impl::RowsParams& rp, uint32_t row_wgs,
                          uint32_t tile_wgs, hipStream_t stream) {
  using RG = rows_impl::RowGeom<D, KV8 ? 1 : 2>;
  constexpr int kRowsLds = 8 * (2 * RG::SLOT_BYTES + RG::KS * 1024);
  constexpr int kTilesLds = (int)prefill_impl::TileGeom<D>::LDS_BYTES;
  constexpr int kLds = kRowsLds > kTilesLds ? kRowsLds : kTilesLds;
  static OncePerDevice once;     // idempotent; a race between two first calls is benign
  bool* const configured = once.flag();
  if (!configured) return DSV_E_LAUNCH;
  if (!*configured) {
    hipFuncAttributes fa;               // no static LDS: the tile body's ring must start at LDS address 0
    if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(mixed_stream_kernel<D, KV8>)) != hipSuccess ||
        fa.sharedSizeBytes != 0)
      return DSV_E_LAUNCH;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(mixed_stream_kernel<D, KV8>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLds) != hipSuccess)
      return DSV_E_LAUNCH;
    *configured = true;
  }
  hipLaunchKernelGGL((mixed_stream_kernel<D, KV8>), dim3(row_wgs + tile_wgs), dim3(512), kLds, stream, tp, rp, row_wgs);
  return launch_status();
}

}  // namespace

bool mixed_launch_supported(const AttnArgs& a, const PlanConfig& cfg, const PlanCounts& n) {
  if (cfg.stream_wgs > 0 && (cfg.stream_wgs % 8 != 0 || a.Hkv > 8 || a.Hq / a.Hkv > rows_impl::kRowHeads)) return false;
  return n.tiles > 0 && n.items > 0 && cfg.row_nbuf == 2 && cfg.tile_tokens >= 32 && cfg.tile_tokens <= prefill_impl::kTileQ &&
         cfg.part_tokens <= 64 * kBlockSize && prefill_impl::kThreads == 512 && (a.D == 128 || a.D == 64);
}

int launch_mixed(const AttnArgs& a, const WorkLists& w, const PlanConfig& cfg, const PlanCounts& n,
                 hipStream_t stream) {
  if (!mixed_launch_supported(a, cfg, n)) return DSV_E_UNSUPPORTED;
  const int G = a.Hq / a.Hkv;
  const prefill_impl::TilesParams tp = prefill_impl::make_tiles_params(a, w, cfg, n);
  rows_impl::RowsParams rp{a, w, cfg.part_tokens, G, 1};
  if (cfg.stream_wgs > 0) {
    const int64_t tile_wgs = n.tiles * a.Hkv * cfg.head_groups;
    if (tile_wgs + cfg.stream_wgs > 0x7fffffffLL) return DSV_E_UNSUPPORTED;
    const uint32_t rw = (uint32_t)cfg.stream_wgs, tw = (uint32_t)tile_wgs;
    if (a.D == 128) return a.kv8 ? launch_mixed_stream_t<128, true>(tp, rp, rw, tw, stream)
                                 : launch_mixed_stream_t<128, false>(tp, rp, rw, tw, stream);
    return a.kv8 ? launch_mixed_stream_t<64, true>(tp, rp, rw, tw, stream)
                 : launch_mixed_stream_t<64, false>(tp, rp, rw, tw, stream);
  }
  int waves = 1;
  while (waves < a.Hkv && waves < 8) waves <<= 1;
  MixParams mp;
  mp.tiles_x = (uint32_t)(n.tiles * a.Hkv);
  const int64_t tile_wgs = (int64_t)mp.tiles_x * cfg.head_groups;
  mp.rows_x = (uint32_t)n.items;
  mp.rows_y = (uint32_t)ceil_div(a.Hkv, waves);
  rp.gy = (int32_t)mp.rows_y;
  const int64_t row_wgs = (int64_t)n.items * mp.rows_y * ceil_div(G, rows_impl::kRowHeads);
  const int64_t tg = ceil_div(tile_wgs, (int64_t)kGroup), rg = ceil_div(row_wgs, (int64_t)kGroup);
  if ((tg + rg) * kGroup > 0x7fffffffLL) return DSV_E_UNSUPPORTED;
  mp.tile_wgs = (uint32_t)tile_wgs;
  mp.row_wgs = (uint32_t)row_wgs;
  mp.tile_groups = (uint32_t)tg;
  mp.total_groups = (uint32_t)(tg + rg);
  mp.rows_waves = waves;
  const int slot = a.D == 128 ? (a.kv8 ? rows_impl::RowGeom<128, 1>::SLOT_BYTES : rows_impl::RowGeom<128, 2>::SLOT_BYTES)
                              : (a.kv8 ? rows_impl::RowGeom<64, 1>::SLOT_BYTES : rows_impl::RowGeom<64, 2>::SLOT_BYTES);
  const int rows_lds = waves * 2 * slot;
  if (a.D == 128) {
    const int lds = max(rows_lds, (int)prefill_impl::TileGeom<128>::LDS_BYTES);
    return a.kv8 ? launch_mixed_t<128, true>(tp, rp, mp, lds, stream) : launch_mixed_t<128, false>(tp, rp, mp, lds, stream);
  }
  const int lds = max(rows_lds, (int)prefill_impl::TileGeom<64>::LDS_BYTES);
  return a.kv8 ? launch_mixed_t<64, true>(tp, rp, mp, lds, stream) : launch_mixed_t<64, false>(tp, rp, mp, lds, stream);
}

}  // namespace dsv
