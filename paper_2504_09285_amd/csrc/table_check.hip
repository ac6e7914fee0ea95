// dsv_check_block_tables: opt-in validation of block-table entries.
//
// Every other entry point trusts the table: token t of a request lives in pool block
// table[t / 16] (paper sections 2.1 and 4.3: the KV cache is block-granular and the receiver of a
// hand-off chooses the placement), and an entry outside [0, num_blocks) makes a kernel read or
// write outside the pool.  Checking costs a pass over the table, so it is a call of its own that a
// caller makes when it wants the guarantee (after building a table, in debug runs), not a part of
// the hot path.  The result stays on the device; the host reads it when it chooses to.
#include "dsv_common.h"

namespace dsv {
namespace {

constexpr int kCheckThreads = 256;

__global__ void check_init_kernel(int32_t* result) {
  result[0] = 0;
  result[1] = 0x7fffffff;
}

// grid (ceil(max_blocks / 256), num_seqs): row blockIdx.y, entries blockIdx.x * 256 + thread.
__global__ __launch_bounds__(kCheckThreads) void check_tables_kernel(const int32_t* __restrict__ tables,
                                                                     int32_t max_blocks,
                                                                     const int32_t* __restrict__ tokens,
                                                                     int32_t num_blocks, int32_t* result) {
  const int row = blockIdx.y;
  const int col = (int)blockIdx.x * kCheckThreads + (int)threadIdx.x;
  const int ntok = tokens[row];
  const int64_t needed = ntok > 0 ? ((int64_t)ntok + kBlockSize - 1) / kBlockSize : 0;
  const int64_t flat = (int64_t)row * max_blocks + col;
  bool bad = false;
  if (col < max_blocks && col < needed) {
    const int32_t e = tables[flat];
    bad = e < 0 || e >= num_blocks;
  }
  // A row that needs more entries than the table is wide is reported once, at its first entry.
  if (col == 0 && (ntok < 0 || needed > max_blocks)) bad = true;
  const unsigned long long m = __ballot(bad);
  if (m == 0ull) return;                                        // uniform for the wave
  const int lane = (int)threadIdx.x & 63;
  if (lane == __ffsll((long long)m) - 1) {
    atomicAdd(&result[0], __popcll(m));
    // flat indices rise with the lane, so the wave's first offender has its smallest one
    atomicMin(&result[1], (int32_t)(flat > 0x7ffffffeLL ? 0x7ffffffeLL : flat));
  }
}

}  // namespace
}  // namespace dsv

extern "C" int dsv_check_block_tables(const int32_t* block_tables, int32_t max_blocks_per_seq,
                                      const int32_t* tokens_per_seq, int32_t num_seqs, int32_t num_blocks,
                                      int32_t* result, void* hip_stream) {
  using namespace dsv;
  if (num_seqs < 0 || max_blocks_per_seq < 1 || num_blocks < 1 || !result) return DSV_E_INVALID;
  if (num_seqs > 0 && (!block_tables || !tokens_per_seq)) return DSV_E_INVALID;
  if (num_seqs > 65535) return DSV_E_UNSUPPORTED;              // one grid row per table row
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  begin_gpu_work();
  hipLaunchKernelGGL(check_init_kernel, dim3(1), dim3(1), 0, stream, result);
  if (launch_status()) return DSV_E_LAUNCH;
  if (num_seqs == 0) return DSV_OK;
  dim3 grid((unsigned)ceil_div(max_blocks_per_seq, kCheckThreads), (unsigned)num_seqs);
  hipLaunchKernelGGL(check_tables_kernel, grid, dim3(kCheckThreads), 0, stream, block_tables,
                     max_blocks_per_seq, tokens_per_seq, num_blocks, result);
  return launch_status();
}
