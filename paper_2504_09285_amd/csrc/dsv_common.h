// Internal helpers shared by the HIP translation units of libdsv_attn (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "dsv_attn.h"

namespace dsv {

constexpr int kBlockSize = 16;          // tokens per KV block (the only size supported)
constexpr int kWave = 64;               // CDNA wavefront width

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Validates pool geometry common to all entry points.
inline int check_pool(const dsv_kv_pool* p) {
  if (!p || !p->k_base || !p->v_base) return DSV_E_INVALID;
  if (p->num_layers < 1 || p->num_blocks < 1 || p->num_kv_heads < 1) return DSV_E_INVALID;
  if (p->num_layers > 1 && p->layer_stride < 0) return DSV_E_INVALID;
  if (p->block_size != kBlockSize) return DSV_E_UNSUPPORTED;
  if (p->head_dim != 64 && p->head_dim != 128) return DSV_E_UNSUPPORTED;
  return DSV_OK;
}

// fp32 -> bf16 bits, round to nearest even (NaN stays a quiet NaN).
__host__ __device__ inline uint16_t f32_to_bf16_rne(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Called by every entry point before its first launch: an error that an earlier HIP call of this
// host thread left behind (the caller's, or another library's) must not be taken for a failed
// launch of ours by launch_status() below.
inline void begin_gpu_work() { (void)hipGetLastError(); }

inline int launch_status() {
  return hipGetLastError() == hipSuccess ? DSV_OK : DSV_E_LAUNCH;
}

// Set-up that HIP keeps per device (a kernel's dynamic-LDS limit) is done once per device: a
// launcher owns one of these as a function-local static and asks it for the current device's
// flag.  Setting the same limit twice is harmless, so two first calls that race are too.
constexpr int kMaxDevices = 64;
struct OncePerDevice {
  bool done[kMaxDevices] = {};
  // The current device's flag, or nullptr when HIP names no device (or one beyond kMaxDevices).
  bool* flag() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
      (void)hipGetLastError();
      return nullptr;
    }
    return &done[dev];
  }
};

}  // namespace dsv
