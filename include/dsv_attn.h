/*
 * dsv_attn.h - C ABI of the MI355X (gfx950) library for the per-step hot path under
 * micro-request execution: attention of one mixed prefill+decode batch over a paged KV
 * cache, and the chunked KV pack/unpack that hands a split request's cache between
 * instances.
 *
 * Conventions for every entry point
 *   - Plain C, no exceptions, thread-compatible.  State the library keeps between calls, all
 *     of it host-side and none of it derived from a caller's buffers, per device (up to 64
 *     devices in a process): the compute-unit count, one flag per kernel saying that its
 *     dynamic-LDS limit has been raised on that device, and the address of the fixed array of
 *     attn_mixed_batch_static; and, per host thread, the event handles set with
 *     dsv_profile_events (until cleared).
 *   - "device" pointers are HIP device memory on the current device; "host" pointers are
 *     ordinary host memory.  All buffers are caller-owned; the library allocates no device
 *     memory and keeps no pointer after the call returns.
 *   - All GPU work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).  Calls never synchronise.  Host arrays are consumed before return.
 *   - Stream capture: a call made while `hip_stream` is being captured into a HIP graph
 *     records kernel launches only (no allocation, no synchronisation, no memset node; the
 *     work lists are cleared by the library's own kernels), so it may be captured and
 *     replayed.  A replay reads every device buffer afresh; what the host derived from the
 *     host-side arrays (grid sizes, workspace layout) is frozen, so a graph is valid for
 *     batches with the same host-side arrays.  Make one call of the same entry point, with the
 *     same head geometry and cache element size, on the same device, outside the capture first: the
 *     first launch of each kernel variant on a device raises that kernel's dynamic-LDS limit (once, to the largest value any
 *     batch can need), which is not a capturable operation.
 *   - A call that enqueues work first clears the calling thread's HIP last-error state
 *     (hipGetLastError), so that an error left by an earlier, unrelated HIP call is not
 *     reported as DSV_E_LAUNCH.
 *   - Return value: DSV_OK (0) or a negative DSV_E_* code.  Arguments are checked before any
 *     GPU work: with DSV_E_INVALID, DSV_E_UNSUPPORTED or DSV_E_WORKSPACE nothing has been
 *     enqueued.  DSV_E_LAUNCH means HIP refused a launch part-way; outputs are then undefined.
 *   - bf16 = upper 16 bits of IEEE-754 binary32, stored as uint16.
 *   - Block-table entries are trusted (not range-checked against num_blocks);
 *     dsv_check_block_tables() checks a table on request.
 */
#ifndef DSV_ATTN_H
#define DSV_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DSV_OK              0
#define DSV_E_INVALID      -1   /* null pointer, bad length, chunk outside its table, ...   */
#define DSV_E_UNSUPPORTED  -2   /* head_dim not 64/128, block_size not 16, counts past 2^31 */
#define DSV_E_WORKSPACE    -3   /* workspace smaller than attn_mixed_batch_workspace_bytes() */
#define DSV_E_LAUNCH       -4   /* HIP reported an error while enqueueing                    */

#define DSV_OUT_F32 0
#define DSV_OUT_BF16 1

/*
 * A paged KV pool (paper sections 2.1 and 4.3: the KV cache is kept in GPU memory in
 * fixed-size blocks and is append-only).  K and V have identical geometry:
 *   layer l, block b, slot s, kv head g, dim d  ->
 *   base[l*layer_stride + ((b*block_size + s)*num_kv_heads + g)*head_dim + d]   (bf16 elements)
 * Token t of a request lives in block block_table[t / block_size], slot t % block_size.
 */
typedef struct {
  void*   k_base;        /* device */
  void*   v_base;        /* device */
  int64_t layer_stride;  /* elements between consecutive layers; ignored when num_layers == 1 */
  int32_t num_layers;
  int32_t num_blocks;
  int32_t block_size;    /* must be 16 */
  int32_t num_kv_heads;
  int32_t head_dim;      /* 64 or 128 */
} dsv_kv_pool;

/*
 * One contiguous chunk of a request's KV = one transfer unit (paper section 4.3: a
 * micro-request's KV is shipped in equal-sized chunks regardless of token type; the last
 * chunk of a range may be shorter and is stored short).
 * Chunk layout inside chunk_buf, starting at element chunk_offset:
 *   [layer][K=0|V=1][num_tokens][num_kv_heads][head_dim]  bf16, tight.
 */
typedef struct {
  int32_t seq;           /* row of the block table                                  */
  int32_t token_begin;   /* first token position of the chunk (need not be a multiple of 16) */
  int32_t num_tokens;    /* > 0                                                     */
  int32_t reserved;      /* must be 0                                               */
  int64_t chunk_offset;  /* element offset of the chunk in chunk_buf; multiple of 8 */
} dsv_chunk_desc;

/*
 * Bytes of device workspace attn_mixed_batch needs for this batch: the work lists of the batch
 * plan (paper section 4.2, Alg. 2: a batch is formed on the host before each iteration; its
 * decode tokens and prefill spans become the kernels' work items) and the partial results of
 * contexts split across workgroups.  Arguments as in attn_mixed_batch; host pointers only, no GPU
 * call.  Returns 0 if the batch is invalid.
 */
size_t attn_mixed_batch_workspace_bytes(int32_t num_seqs, const int32_t* q_offsets_host,
                                        const int32_t* ctx_lens_host, int32_t num_q_heads,
                                        int32_t num_kv_heads, int32_t head_dim);

/*
 * How the library would cut this batch into GPU work (paper section 4.2, Alg. 2: the batch is
 * known on the host before the step; the cut depends on nothing else, apart from the tuning
 * knobs in the environment).  Host only, no GPU call; for tests, benchmarks and logs.
 *   kv_elem_bytes  2 (bf16 cache) or 1 (8-bit cache)
 *   info           host, int32[8], filled on success:
 *     [0] row streams: 0 = the row work (decodes and the smallest spans) is cut into items of
 *         info[1] tokens of context, one workgroup each; n > 0 = it runs as n persistent
 *         workgroups that each stream an equal share of all rows' KV blocks
 *     [1] tokens per context partition of a row item (0 with row streams)
 *     [2] query tokens on the row path   [3] row work items (with streams: an upper bound)
 *     [4] work items of the prefill-span (matrix-core) path, per KV head and head group
 *     [5] KV tiles per partition of a query tile cut along the context, 0 = not cut
 *     [6] 1 if row work and prefill tiles go out in one launch   [7] query tokens per tile
 * Returns DSV_OK, DSV_E_INVALID or DSV_E_UNSUPPORTED as attn_mixed_batch would.
 */
int attn_mixed_batch_plan_info(int32_t num_seqs, const int32_t* q_offsets_host,
                               const int32_t* ctx_lens_host, int32_t num_q_heads,
                               int32_t num_kv_heads, int32_t head_dim, int32_t kv_elem_bytes,
                               int32_t* info);

/*
 * Attention of one mixed batch (paper section 3.1 "Unified execution instances", section 4.2
 * and Alg. 2: each step runs one token-level batch holding all decode tokens plus prefill
 * spans; section 3.1 "Micro-request abstraction": a span is any contiguous token range of a
 * request and resumes on the earlier tokens as cached prefix; section 2.1: attention is
 * autoregressive over the KV cache).
 *
 * Segment i has q_len_i = q_offsets[i+1]-q_offsets[i] >= 1 new tokens and ctx_lens[i] >=
 * q_len_i KV tokens in total, its own new tokens included (their K/V must already be in the
 * pool).  New token j sits at position p = ctx_lens[i]-q_len_i+j and attends to tokens 0..p
 * of the segment's block-table row.  Query head h reads KV head h / (num_q_heads/num_kv_heads).
 *   out[q_offsets[i]+j][h][:] = sum_t softmax_t(softmax_scale * <q, K[t]>) * V[t],  t = 0..p
 * Segments with q_len 1 (decodes) and longer ones (prefill spans) may come in any order.
 *
 *   q            device, bf16 [total_q][num_q_heads][head_dim]
 *   out          device, [total_q][num_q_heads][head_dim], fp32 (DSV_OUT_F32) or bf16
 *                (DSV_OUT_BF16: round-to-nearest-even of the fp32 result)
 *   pool, layer  the pool and the layer attended (0 <= layer < num_layers)
 *   block_tables device, int32 [num_seqs][max_blocks_per_seq]; row i needs
 *                ceil(ctx_lens[i]/16) valid entries, the rest is never read
 *   q_offsets, ctx_lens            device, int32 [num_seqs+1] and [num_seqs]
 *   q_offsets_host, ctx_lens_host  host copies of the same (the batch was composed on the host)
 *   softmax_scale  finite and >= 0 (1/sqrt(head_dim) in the usual case)
 *   workspace    device, 256-byte aligned, at least attn_mixed_batch_workspace_bytes(); may be
 *                reused once the stream has passed this call
 * Accumulation is fp32; probabilities entering the PV product of prefill spans are rounded to
 * bf16.  num_seqs == 0 is a no-op.
 */
int attn_mixed_batch(const void* q, void* out, const dsv_kv_pool* pool, int32_t layer,
                     const int32_t* block_tables, int32_t max_blocks_per_seq,
                     const int32_t* q_offsets, const int32_t* ctx_lens,
                     const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                     int32_t num_seqs, int32_t num_q_heads, float softmax_scale,
                     int32_t out_dtype, void* workspace, size_t workspace_bytes,
                     void* hip_stream);

/*
 * Gather token ranges of requests from a paged pool into contiguous chunks, all layers
 * (paper section 4.3: the sender's side of chunk-based KV transfer).  Byte-exact copy.
 *   descs       device array of num_chunks descriptors;  descs_host: host copy of the same
 *   chunk_buf   device, 16-byte aligned; chunk c is written at chunk_offset_c
 * Chunks must not overlap in chunk_buf.  num_chunks == 0 is a no-op.
 */
int kv_pack_chunks(const dsv_kv_pool* src, const int32_t* block_tables,
                   int32_t max_blocks_per_seq, const dsv_chunk_desc* descs,
                   const dsv_chunk_desc* descs_host, int32_t num_chunks, void* chunk_buf,
                   void* hip_stream);

/*
 * Scatter contiguous chunks into a paged pool through the receiver's own block table (paper
 * section 4.3: placement is chosen on the receiver side).  Only the covered token slots are
 * written; every other byte of the destination pool is left as it was.  Byte-exact copy.
 */
int kv_unpack_chunks(const void* chunk_buf, const dsv_chunk_desc* descs,
                     const dsv_chunk_desc* descs_host, int32_t num_chunks,
                     const dsv_kv_pool* dst, const int32_t* dst_block_tables,
                     int32_t max_blocks_per_seq, void* hip_stream);

/*
 * kv_unpack_chunks with the destination written in ascending block order (paper section 4.3: the
 * receiver places the chunks; a receiver that took most of a pool's blocks for a hand-off gets
 * them filled at the rate of a sequential copy, whatever the order of its table).  Same arguments,
 * same result byte for byte, plus a workspace for the inverse of the block table:
 *   workspace   device, 8-byte aligned, at least kv_unpack_chunks_ordered_workspace_bytes(
 *               dst->num_blocks) = 8 bytes per pool block; overwritten by every call
 * The ordered sweep is used when every chunk starts on a block boundary (token_begin % 16 == 0)
 * and the chunks cover at least half of the pool's blocks; any other hand-off runs exactly as
 * kv_unpack_chunks does.  Two rows of the table must not name the same block for tokens of the
 * hand-off (with kv_unpack_chunks the later writer would win; here the result is undefined).
 * Errors as for kv_unpack_chunks, DSV_E_WORKSPACE for a workspace too small.
 */
size_t kv_unpack_chunks_ordered_workspace_bytes(int32_t num_blocks);
int kv_unpack_chunks_ordered(const void* chunk_buf, const dsv_chunk_desc* descs,
                             const dsv_chunk_desc* descs_host, int32_t num_chunks,
                             const dsv_kv_pool* dst, const int32_t* dst_block_tables,
                             int32_t max_blocks_per_seq, void* workspace, size_t workspace_bytes,
                             void* hip_stream);

/*
 * Write the keys/values of the batch's new tokens into layer `layer` of the paged pool, at the
 * positions they occupy (paper section 2.1: prefill populates the KV cache and every decode
 * step appends to it, before attention reads it).  For segment i and its j-th new token the
 * destination is token position ctx_len_i - q_len_i + j of row i of the block table.
 *   k_new, v_new   device, bf16 [total_q][num_kv_heads][head_dim], 16-byte aligned
 *   block_tables, q_offsets, ctx_lens, the host mirrors, num_seqs: as for attn_mixed_batch
 * Byte-exact copy; every other byte of the pool is left as it was.  Two new tokens must not
 * map to the same pool slot (the result for that slot would be either one).  Enqueues one
 * kernel on hip_stream; an attn_mixed_batch call on the same stream afterwards sees the rows.
 * num_seqs == 0 is a no-op.  Errors as for attn_mixed_batch (no workspace is needed).
 */
int kv_append(const void* k_new, const void* v_new, const dsv_kv_pool* pool, int32_t layer,
              const int32_t* block_tables, int32_t max_blocks_per_seq,
              const int32_t* q_offsets, const int32_t* ctx_lens,
              const int32_t* q_offsets_host, const int32_t* ctx_lens_host, int32_t num_seqs,
              void* hip_stream);

/*
 * ---- 8-bit KV cache variant --------------------------------------------------------------
 * The paper (sections 2.1, 3.1, 4.3) treats a token's KV as a payload whose size sets both the
 * bytes a decode step streams and the bytes a hand-off ships, and leaves its number format
 * open.  The entry points below are the same operations on a cache stored as one byte per
 * element: codes of the OCP 8-bit floating point format E4M3 (1 sign, 4 exponent bits with bias
 * 7, 3 mantissa bits; subnormals; no infinities; 0x7f/0xff = NaN; largest finite 448), with one
 * positive finite fp32 scale per tensor:  value = scale * decode(code).
 * The pool descriptor is the same struct; its elements are then bytes (layer_stride in bytes,
 * a multiple of 16), and the chunk layout is the same with 1-byte elements (chunk_offset in
 * bytes, a multiple of 16).
 */

/*
 * attn_mixed_batch on a cache of E4M3 codes:
 *   out[q_offsets[i]+j][h][:] = sum_t softmax_t(softmax_scale * <q, k_scale*K8[t]>) * v_scale*V8[t]
 * Every argument as for attn_mixed_batch; k_scale, v_scale: the dequantisation scales of the
 * layer (positive, finite, else DSV_E_INVALID).  The workspace is larger: prefill spans of 16
 * and more tokens are computed from a bf16 copy of their whole contexts, made inside the call
 * (exact: every code is a bf16 value), of 4 * head_dim * num_kv_heads bytes per cached token.
 * Codes of cached tokens must not be NaN.
 */
size_t attn_mixed_batch_fp8kv_workspace_bytes(int32_t num_seqs, const int32_t* q_offsets_host,
                                              const int32_t* ctx_lens_host, int32_t num_q_heads,
                                              int32_t num_kv_heads, int32_t head_dim);
int attn_mixed_batch_fp8kv(const void* q, void* out, const dsv_kv_pool* pool, int32_t layer,
                           const int32_t* block_tables, int32_t max_blocks_per_seq,
                           const int32_t* q_offsets, const int32_t* ctx_lens,
                           const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                           int32_t num_seqs, int32_t num_q_heads, float softmax_scale,
                           float k_scale, float v_scale, int32_t out_dtype, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

/*
 * kv_append for a cache of E4M3 codes: the new tokens' bf16 keys/values are quantised on the
 * way in.  The code of an input x is decided in fp32: y = fp32(x) / scale (one IEEE division),
 * then the E4M3 value nearest to y, ties to the even mantissa; |y| >= 448 (infinities
 * included) gives +-448; a NaN input gives a NaN code; the sign of zero is kept.
 * Arguments as for kv_append; k_scale, v_scale positive and finite.
 */
int kv_append_fp8(const void* k_new, const void* v_new, const dsv_kv_pool* pool, int32_t layer,
                  const int32_t* block_tables, int32_t max_blocks_per_seq,
                  const int32_t* q_offsets, const int32_t* ctx_lens,
                  const int32_t* q_offsets_host, const int32_t* ctx_lens_host, int32_t num_seqs,
                  float k_scale, float v_scale, void* hip_stream);

/*
 * kv_pack_chunks / kv_unpack_chunks for a cache of 1-byte elements (paper section 4.3: the
 * chunk is the unit of transfer whatever the payload).  Byte-exact copies; a chunk is half the
 * size of its bf16 counterpart.  Arguments as for the bf16 calls, offsets in bytes.
 */
int kv_pack_chunks_fp8(const dsv_kv_pool* src, const int32_t* block_tables,
                       int32_t max_blocks_per_seq, const dsv_chunk_desc* descs,
                       const dsv_chunk_desc* descs_host, int32_t num_chunks, void* chunk_buf,
                       void* hip_stream);
int kv_unpack_chunks_fp8(const void* chunk_buf, const dsv_chunk_desc* descs,
                         const dsv_chunk_desc* descs_host, int32_t num_chunks,
                         const dsv_kv_pool* dst, const int32_t* dst_block_tables,
                         int32_t max_blocks_per_seq, void* hip_stream);

/*
 * ---- One plan for all layers of a step ---------------------------------------------------
 * A serving iteration runs the same batch through every layer of the model (paper sections
 * 2.1 and 4.2: a batch is formed once per iteration), and the work lists attn_mixed_batch
 * derives from the batch (which span takes which path, context partitions, tile order) do not
 * depend on the layer.  attn_mixed_batch_plan builds them once into `workspace`;
 * attn_mixed_batch_planned / attn_mixed_batch_fp8kv_planned then run the step of one layer on
 * those lists: the same result as attn_mixed_batch, without its list-building kernel.
 *
 *   plan      host memory, caller-owned, written by attn_mixed_batch_plan, read by the planned
 *             calls.  It records what the lists depend on; a planned call whose arguments differ
 *             (host arrays by content; workspace, block_tables, q_offsets, ctx_lens by address;
 *             sequence and head counts, head_dim, max_blocks_per_seq, element size, the tuning
 *             knobs of the environment) returns DSV_E_INVALID and enqueues nothing.
 *   kv_elem_bytes  2 for a bf16 cache (planned calls: attn_mixed_batch_planned), 1 for E4M3 codes
 *             (attn_mixed_batch_fp8kv_planned); workspace size as for the respective full call.
 *   The planned calls must be enqueued after the plan call on the same stream (or ordered
 *   behind it by the caller).  Between them nothing else may write the workspace, and the
 *   contents of block_tables, q_offsets and ctx_lens must not change.  The calls of successive
 *   layers share the partial-result area of the workspace, so they must not overlap in time
 *   (one stream, or ordered by the caller).  All other arguments, the result and the error
 *   codes are those of attn_mixed_batch / attn_mixed_batch_fp8kv.  num_seqs == 0: no work.
 */
typedef struct { uint64_t opaque[16]; } dsv_attn_plan;
int attn_mixed_batch_plan(dsv_attn_plan* plan, const int32_t* block_tables,
                          int32_t max_blocks_per_seq, const int32_t* q_offsets,
                          const int32_t* ctx_lens, const int32_t* q_offsets_host,
                          const int32_t* ctx_lens_host, int32_t num_seqs, int32_t num_q_heads,
                          int32_t num_kv_heads, int32_t head_dim, int32_t kv_elem_bytes,
                          void* workspace, size_t workspace_bytes, void* hip_stream);
int attn_mixed_batch_planned(const dsv_attn_plan* plan, const void* q, void* out,
                             const dsv_kv_pool* pool, int32_t layer, const int32_t* block_tables,
                             int32_t max_blocks_per_seq, const int32_t* q_offsets,
                             const int32_t* ctx_lens, const int32_t* q_offsets_host,
                             const int32_t* ctx_lens_host, int32_t num_seqs, int32_t num_q_heads,
                             float softmax_scale, int32_t out_dtype, void* workspace,
                             size_t workspace_bytes, void* hip_stream);
int attn_mixed_batch_fp8kv_planned(const dsv_attn_plan* plan, const void* q, void* out,
                                   const dsv_kv_pool* pool, int32_t layer,
                                   const int32_t* block_tables, int32_t max_blocks_per_seq,
                                   const int32_t* q_offsets, const int32_t* ctx_lens,
                                   const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                                   int32_t num_seqs, int32_t num_q_heads, float softmax_scale,
                                   float k_scale, float v_scale, int32_t out_dtype, void* workspace,
                                   size_t workspace_bytes, void* hip_stream);

/*
 * ---- attn_mixed_batch without a workspace argument -------------------------------------------
 * For callers that cannot allocate device memory or bring a workspace: code that runs under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same computation and
 * the same kernels as attn_mixed_batch (same arguments, result and error codes, minus the two
 * workspace arguments); the work lists and split-context partials live in a fixed array of
 * DSV_STATIC_SCRATCH_BYTES in device memory that the library itself owns (part of its code object:
 * every GPU the library is used on holds one copy until the process ends).  The call allocates
 * nothing, frees nothing and calls no allocating routine.
 *   - A batch whose attn_mixed_batch_workspace_bytes() exceeds DSV_STATIC_SCRATCH_BYTES is
 *     refused with DSV_E_WORKSPACE before anything is enqueued (64 MiB hold each of the five
 *     benchmark configurations; the largest, 64 decodes on 16K-128K contexts, needs 56 MiB).
 *   - All calls on one GPU share that GPU's array, and the array keeps the previous call's
 *     contents (nothing in it needs to start at zero: every call rewrites what it reads).  Calls
 *     that overlap in time on one GPU - two streams, two host threads - race on it and give
 *     undefined results; calls on one stream, or ordered by the caller, are safe.
 *   - The first call on a device looks the array's address up (no allocation); make it outside
 *     stream capture, as for every entry point.
 * attn_mixed_batch_static_max_bytes() returns DSV_STATIC_SCRATCH_BYTES as built.
 */
#define DSV_STATIC_SCRATCH_BYTES (64u << 20)
size_t attn_mixed_batch_static_max_bytes(void);
int attn_mixed_batch_static(const void* q, void* out, const dsv_kv_pool* pool, int32_t layer,
                            const int32_t* block_tables, int32_t max_blocks_per_seq,
                            const int32_t* q_offsets, const int32_t* ctx_lens,
                            const int32_t* q_offsets_host, const int32_t* ctx_lens_host,
                            int32_t num_seqs, int32_t num_q_heads, float softmax_scale,
                            int32_t out_dtype, void* hip_stream);

/*
 * Opt-in check of block-table entries.  Every other entry point trusts the table (paper sections
 * 2.1 and 4.3: KV lives in blocks, and the receiver of a hand-off chooses their placement): an
 * entry outside [0, num_blocks) makes a kernel read or write outside the pool.  This call checks,
 * on the device, the entries a batch or a hand-off will use: for row i the first
 * ceil(tokens_per_seq[i] / 16) entries.  A row that needs more entries than max_blocks_per_seq,
 * or has a negative token count, counts as one offence at its first entry.
 *   block_tables    device, int32 [num_seqs][max_blocks_per_seq]
 *   tokens_per_seq  device, int32 [num_seqs]: ctx_lens of attn_mixed_batch / kv_append, or the
 *                   number of tokens a hand-off touches in each row
 *   num_blocks      blocks in the pool (dsv_kv_pool.num_blocks)
 *   result          device, int32[2], written by the call: [0] = number of offending entries
 *                   (0: the table is safe to use), [1] = smallest flat index
 *                   row * max_blocks_per_seq + column among them, 0x7fffffff if there is none
 * Enqueues two small kernels on hip_stream and returns; the host reads `result` when it wants
 * to (after synchronising with the stream).  No workspace, no allocation, capturable.
 * num_seqs == 0 writes {0, 0x7fffffff}.  More than 65535 rows: DSV_E_UNSUPPORTED.
 */
int dsv_check_block_tables(const int32_t* block_tables, int32_t max_blocks_per_seq,
                           const int32_t* tokens_per_seq, int32_t num_seqs, int32_t num_blocks,
                           int32_t* result, void* hip_stream);

/*
 * Profiling aid for benchmarks (not needed for correct use).  Until cleared with NULLs, every
 * later attn_mixed_batch call made by the calling host thread records `start_event` on its
 * stream immediately before, and `stop_event` immediately after, the launch of the named
 * kernel (both hipEvent_t, created by the caller with timing enabled).  If that kernel is not
 * launched for a batch the events are not recorded.  Returns DSV_E_INVALID for an unknown id.
 */
#define DSV_KERNEL_PLAN   0   /* work-list construction                                   */
#define DSV_KERNEL_ROWS   1   /* single-token attention split along the context (decodes) */
#define DSV_KERNEL_TILES  2   /* MFMA attention of long prefill spans                     */
#define DSV_KERNEL_MERGE  3   /* combination of context partitions                        */
#define DSV_KERNEL_MIXED  4   /* rows and tiles in one launch: what a batch holding both  */
                              /* kinds of work runs instead of ids 1 and 2 (environment    */
                              /* DSV_MIXED_LAUNCH=0 keeps them in launches of their own)   */
#define DSV_KERNEL_STAGE  5   /* bf16 copy of the prefill spans' contexts (8-bit cache only)  */
int dsv_profile_events(int32_t kernel_id, void* start_event, void* stop_event);

/*
 * Calibration aids for benchmarks (nothing on the hot path calls them): what this GPU delivers on
 * the plainest HBM streaming and matrix-core loops, with the launch shape and memory hints of the
 * product kernels, to be reported next to the nominal peaks.
 *   dsv_calib_hbm   mode 0: read `bytes` from src (dst: any valid 16 bytes, normally untouched);
 *                   mode 1: write `bytes` to dst (src ignored); mode 2: copy src -> dst.
 *                   One workgroup of 256 threads per 16 KiB, four 16-byte nontemporal accesses per
 *                   thread in one round: kv_copy_kernel without the block table.  Device pointers,
 *                   16-byte aligned; bytes a positive multiple of 16.
 *   dsv_calib_mfma  a register-resident loop of bf16 32x32x16 MFMAs, eight independent
 *                   accumulators per wave, two waves per SIMD (the prefill kernel's occupancy),
 *                   four workgroups per compute unit; *flops_out (host, may be NULL) receives the
 *                   floating-point operations one launch performs.  sink: device, 4 bytes.
 *   dsv_calib_mfma_data  the same loop on operands that change from one MFMA to the next: every
 *                   lane loads sixteen 16-byte fragments from operands (device, operand_bytes bytes
 *                   of bf16 values the caller chose, 256 .. 2^30, a multiple of 16) and cycles
 *                   through them.  The power the matrix cores draw follows the operand bits that
 *                   toggle, so on random data this loop, not dsv_calib_mfma's fixed operands, shows
 *                   what the chip sustains within its power limit.  shape 0: 32x32x16 MFMAs,
 *                   1: 16x16x32 (what the head_dim-128 prefill kernels use; the same flops per
 *                   launch).  iters: a multiple of 8.
 *   dsv_calib_paged_read  the row kernel's access shape with nothing else: k and v (device,
 *                   bytes_each bytes each, a power-of-two number of 32 KiB blocks, at least 64) are
 *                   read as pools of [16 tokens][8 heads][256 bytes] blocks visited in a scattered
 *                   order, by workgroups of eight waves that stream 64 blocks each, every wave
 *                   fetching one head's 256-byte pieces global->LDS into a ring of two 8 KiB slots,
 *                   one block ahead.  *bytes_out (host, may be NULL) receives the bytes one launch
 *                   reads.  sink: device, 4 bytes.
 * Each enqueues one kernel on hip_stream and returns; errors as for the other entry points.
 */
int dsv_calib_hbm(int32_t mode, void* dst, const void* src, size_t bytes, void* hip_stream);
int dsv_calib_mfma_data(int32_t shape, int32_t iters, const void* operands, size_t operand_bytes, void* sink,
                        double* flops_out, void* hip_stream);
int dsv_calib_paged_read(const void* k, const void* v, size_t bytes_each, void* sink, double* bytes_out,
                         void* hip_stream);
int dsv_calib_mfma(int32_t iters, void* sink, double* flops_out, void* hip_stream);

/* Library build identification: a static string, e.g. "dsv_attn gfx950 <date>". */
const char* dsv_build_info(void);

#ifdef __cplusplus
}
#endif
#endif /* DSV_ATTN_H */
