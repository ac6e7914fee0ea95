// Calibration kernels: what this GPU delivers on the plainest possible HBM streaming and
// matrix-core loops, measured with the same launch shapes and memory hints the product kernels
// use.  A benchmark reports them next to the nominal peaks (HBM 8 TB/s, bf16 MFMA 2.5 PFLOP/s),
// so that a kernel's distance from what the hardware can reach is visible beside its distance
// from the data-sheet number.  Nothing on the hot path calls these.
#include "dsv_common.h"

namespace dsv {
namespace {

typedef uint32_t unit_t __attribute__((ext_vector_type(4)));
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int kThreads = 256;
constexpr int kUnits = kThreads * 4;          // 16 KiB per workgroup, one round: as kv_copy_kernel

// MODE 0: read only (the values are folded into a word that is never stored unless it takes an
// impossible value), 1: write only, 2: copy.  Nontemporal loads and stores, as in kv_copy_kernel.
template <int MODE>
__global__ __launch_bounds__(kThreads) void hbm_kernel(const unit_t* __restrict__ src, unit_t* __restrict__ dst,
                                                       uint64_t units) {
  const uint64_t u0 = (uint64_t)blockIdx.x * kUnits + threadIdx.x;
  unit_t v[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint64_t u = u0 + (uint64_t)k * kThreads;
    if (MODE != 1) v[k] = u < units ? __builtin_nontemporal_load(&src[u]) : unit_t{0u, 0u, 0u, 0u};
    else v[k] = unit_t{(uint32_t)u, 1u, 2u, 3u};
  }
  if (MODE == 0) {
    const unit_t x = v[0] ^ v[1] ^ v[2] ^ v[3];
    if (x.x == 0x9e3779b9u && x.y == 0x7f4a7c15u && x.z == 0x85ebca6bu && x.w == 0xc2b2ae35u) dst[0] = x;
    return;
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint64_t u = u0 + (uint64_t)k * kThreads;
    if (u < units) __builtin_nontemporal_store(v[k], &dst[u]);
  }
}

// Register-resident MFMA loop: every wave keeps eight independent 32x32 accumulators and issues
// bf16 32x32x16 MFMAs on them back to back; 512 threads per workgroup = two waves per SIMD, the
// occupancy of the prefill kernel.  Operands are made from the lane id so nothing is constant-folded.
constexpr int kMfmaPerIter = 8;
__global__ __launch_bounds__(512, 2) void mfma_kernel(float* sink, int iters) {
  f32x16_t acc[kMfmaPerIter];
#pragma unroll
  for (int i = 0; i < kMfmaPerIter; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8_t a, b;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    a[r] = (__bf16)(float)((threadIdx.x + r) & 3);
    b[r] = (__bf16)(float)((threadIdx.x * 3 + r) & 1);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kMfmaPerIter; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kMfmaPerIter; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (s == -1.0f) sink[0] = s;                   // never true: sums of non-negative products
}

// The same loop on operands that change from one MFMA to the next, as they do in a real product:
// every lane loads eight A and eight B fragments (16 bytes each) from a buffer of bf16 values the
// caller filled, and MFMA (i, j) of an unrolled group multiplies A[(i + j) % 8] with B[j] into
// accumulator i.  What the matrix cores draw depends on how many operand bits toggle, so this loop,
// not the one above, shows what the chip sustains within its power limit on data like the
// attention kernel's.  SHAPE 0: 32x32x16 MFMAs on eight accumulators; 1: 16x16x32 on sixteen
// (the same flops per iteration and per launch).
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
template <int SHAPE>
__global__ __launch_bounds__(512, 2) void mfma_data_kernel(const uint4* __restrict__ operands, uint32_t frags,
                                                           float* sink, int iters) {
  uint4 a[8], b[8];
  const uint32_t first = (blockIdx.x * 512u + threadIdx.x) * 16u;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = operands[(first + (uint32_t)i) % frags];
    b[i] = operands[(first + 8u + (uint32_t)i) % frags];
  }
  float s = 0.f;
  if constexpr (SHAPE == 0) {
    f32x16_t acc[kMfmaPerIter];
#pragma unroll
    for (int i = 0; i < kMfmaPerIter; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; it += 8) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int i = 0; i < kMfmaPerIter; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a[(i + j) % 8]),
                                                           __builtin_bit_cast(bf16x8_t, b[j]), acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < kMfmaPerIter; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[i][r];
  } else {
    f32x4_t acc[2 * kMfmaPerIter];
#pragma unroll
    for (int i = 0; i < 2 * kMfmaPerIter; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; it += 8) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int i = 0; i < 2 * kMfmaPerIter; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a[(i + j) % 8]),
                                                           __builtin_bit_cast(bf16x8_t, b[j]), acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 2 * kMfmaPerIter; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) s += acc[i][r];
  }
  if (s == 1.2345678e-30f) sink[0] = s;          // practically never: keeps the accumulators alive
}

// The row kernel's access shape with nothing else: both buffers are read as pools of 32 KiB
// blocks ([16 tokens][8 heads][256 bytes]) visited in a scattered order; a workgroup of eight
// waves streams 64 blocks, wave w fetching the 256-byte pieces of head w of every token, 16 bytes
// per lane, global->LDS, into a ring of two 8 KiB slots of its own (K piece, V piece), one block
// ahead of the one it waits for.  Block i of the sweep is pool block (i * 40503 + 977) mod blocks
// (blocks is a power of two, so the map is a permutation).
constexpr int kPagedBlock = 32768;
constexpr int kPagedPerItem = 64;
constexpr int kCalibStreamOnce = 2;     // cache-policy bits of the load: nontemporal, as the row kernel streams K/V
__global__ __launch_bounds__(512) void paged_read_kernel(const unsigned char* __restrict__ kbuf,
                                                         const unsigned char* __restrict__ vbuf, uint32_t blocks,
                                                         unsigned* sink) {
  extern __shared__ __align__(16) unsigned char smem[];
  typedef __attribute__((address_space(3))) void* lds_void_t;
  typedef const __attribute__((address_space(1))) void* gbl_void_t;
  const int wave = (int)threadIdx.x / 64, lane = (int)threadIdx.x % 64;
  unsigned char* ring = smem + wave * 16384;
  uint32_t off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) off[i] = (uint32_t)((i * 4 + lane / 16) * 2048 + wave * 256 + (lane % 16) * 16);
  const uint32_t first = blockIdx.x * kPagedPerItem;
  auto issue = [&](uint32_t i, int slot) {
    const size_t base = (size_t)((i * 40503u + 977u) & (blocks - 1)) * kPagedBlock;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      __builtin_amdgcn_global_load_lds((gbl_void_t)(kbuf + base + off[r]), (lds_void_t)(ring + slot * 8192 + r * 1024), 16, 0, kCalibStreamOnce);
      __builtin_amdgcn_global_load_lds((gbl_void_t)(vbuf + base + off[r]), (lds_void_t)(ring + slot * 8192 + 4096 + r * 1024), 16, 0, kCalibStreamOnce);
    }
  };
  unsigned acc = 0;
  issue(first, 0);
  for (int b = 0; b < kPagedPerItem; ++b) {
    const int slot = b & 1;
    if (b + 1 < kPagedPerItem) {
      issue(first + b + 1, slot ^ 1);
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    unsigned x;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                 : "=v"(x)
                 : "v"((uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)(ring + slot * 8192 + lane * 16))
                 : "memory");
    acc ^= x;
  }
  if (acc == 0x9e3779b9u && blocks == 3u) sink[0] = acc;       // never true: blocks is a power of two
}

}  // namespace
}  // namespace dsv

extern "C" int dsv_calib_paged_read(const void* k, const void* v, size_t bytes_each, void* sink, double* bytes_out,
                                    void* hip_stream) {
  using namespace dsv;
  if (!k || !v || !sink || (reinterpret_cast<uintptr_t>(k) & 15) || (reinterpret_cast<uintptr_t>(v) & 15)) return DSV_E_INVALID;
  const uint64_t blocks = bytes_each / kPagedBlock;
  if (blocks < (uint64_t)kPagedPerItem || (blocks & (blocks - 1)) || blocks * kPagedBlock != bytes_each) return DSV_E_INVALID;
  if (blocks > 0x40000000ull) return DSV_E_UNSUPPORTED;
  static OncePerDevice once;       // raising the dynamic-LDS limit is idempotent; races are benign
  bool* const configured = once.flag();
  if (!configured) return DSV_E_LAUNCH;
  if (!*configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(paged_read_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            128 * 1024) != hipSuccess)
      return DSV_E_LAUNCH;
    *configured = true;
  }
  if (bytes_out) *bytes_out = 2.0 * (double)bytes_each;
  begin_gpu_work();
  hipLaunchKernelGGL(paged_read_kernel, dim3((unsigned)(blocks / kPagedPerItem)), dim3(512), 128 * 1024,
                     static_cast<hipStream_t>(hip_stream), static_cast<const unsigned char*>(k),
                     static_cast<const unsigned char*>(v), (uint32_t)blocks, static_cast<unsigned*>(sink));
  return launch_status();
}

extern "C" int dsv_calib_hbm(int32_t mode, void* dst, const void* src, size_t bytes, void* hip_stream) {
  using namespace dsv;
  if (mode < 0 || mode > 2 || !dst || (mode != 1 && !src) || bytes == 0 || (bytes & 15)) return DSV_E_INVALID;
  if ((reinterpret_cast<uintptr_t>(dst) & 15) || (reinterpret_cast<uintptr_t>(src) & 15)) return DSV_E_INVALID;
  const uint64_t units = bytes / 16;
  const uint64_t grid = (units + kUnits - 1) / kUnits;
  if (grid > 0x7fffffffull) return DSV_E_UNSUPPORTED;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const unit_t* s = static_cast<const unit_t*>(src);
  unit_t* d = static_cast<unit_t*>(dst);
  begin_gpu_work();
  if (mode == 0) hipLaunchKernelGGL(hbm_kernel<0>, dim3((unsigned)grid), dim3(kThreads), 0, stream, s, d, units);
  else if (mode == 1) hipLaunchKernelGGL(hbm_kernel<1>, dim3((unsigned)grid), dim3(kThreads), 0, stream, s, d, units);
  else hipLaunchKernelGGL(hbm_kernel<2>, dim3((unsigned)grid), dim3(kThreads), 0, stream, s, d, units);
  return launch_status();
}

extern "C" int dsv_calib_mfma_data(int32_t shape, int32_t iters, const void* operands, size_t operand_bytes, void* sink,
                                   double* flops_out, void* hip_stream) {
  using namespace dsv;
  if (shape < 0 || shape > 1 || iters < 8 || (iters & 7) || !sink || !operands || operand_bytes < 256 || (operand_bytes & 15) ||
      operand_bytes > 0x40000000ull || (reinterpret_cast<uintptr_t>(operands) & 15))
    return DSV_E_INVALID;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
    (void)hipGetLastError();
    return DSV_E_LAUNCH;
  }
  const int grid = cus * 4;
  if (flops_out) *flops_out = (double)grid * 8 /*waves*/ * iters * kMfmaPerIter * (2.0 * 32 * 32 * 16);
  begin_gpu_work();
  if (shape == 0)
    hipLaunchKernelGGL(mfma_data_kernel<0>, dim3((unsigned)grid), dim3(512), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const uint4*>(operands), (uint32_t)(operand_bytes / 16), static_cast<float*>(sink), iters);
  else
    hipLaunchKernelGGL(mfma_data_kernel<1>, dim3((unsigned)grid), dim3(512), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const uint4*>(operands), (uint32_t)(operand_bytes / 16), static_cast<float*>(sink), iters);
  return launch_status();
}

extern "C" int dsv_calib_mfma(int32_t iters, void* sink, double* flops_out, void* hip_stream) {
  using namespace dsv;
  if (iters < 1 || !sink) return DSV_E_INVALID;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
    (void)hipGetLastError();
    return DSV_E_LAUNCH;
  }
  const int grid = cus * 4;                      // four rounds of one workgroup per compute unit
  if (flops_out) *flops_out = (double)grid * 8 /*waves*/ * iters * kMfmaPerIter * (2.0 * 32 * 32 * 16);
  begin_gpu_work();
  hipLaunchKernelGGL(mfma_kernel, dim3((unsigned)grid), dim3(512), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<float*>(sink), iters);
  return launch_status();
}
