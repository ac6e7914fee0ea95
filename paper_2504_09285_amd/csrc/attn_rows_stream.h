// Row work as one stream per workgroup.
//
// The arithmetic, the LDS ring, the fragment layouts and the load shapes are those of
// attn_rows_kernel.h (read that header first).  What changes is how the work is cut.  There a
// work item is (query token, context partition of a fixed size) and a workgroup takes one item;
// on long contexts (decode over tens of thousands of cached tokens, the memory-bound part of a
// step: paper sections 2.1 and 4.2) that costs in three ways: the launch ends on a round in
// which only some compute units still have an item, every item pays its own start-up, and every
// item writes 16 KiB of partials whose stores, trickling into a memory system that is busy
// reading, slow the K/V stream far more than their size suggests.
//
// Here all rows' blocks form one sequence, which the planner cuts into as many equal runs as
// there are workgroups; a workgroup streams its run from end to end.  A row that straddles a cut
// is partitioned there, so there are at most (rows + workgroups - 1) items, only the rows that
// were cut write partials, every workgroup ends at the same time, and the K/V requests of a
// workgroup never stop between items: the first block of the next item is requested while the
// last block of the current one is consumed, its query rows right behind it.
#pragma once
#include "attn_rows_kernel.h"

namespace dsv {
namespace rows_impl {

template <int D, bool KV8>
__device__ __forceinline__ void rows_stream_body(const RowsParams& prm, int wg, unsigned char* smem) {
  constexpr int EB = KV8 ? 1 : 2;
  constexpr int R = 2;                                   // ring slots per wave
  using Geo = RowGeom<D, EB>;
  constexpr int ROWB = Geo::ROWB, CPR = Geo::CPR, TPI = Geo::TPI, IPB = Geo::IPB, KS = Geo::KS, DB = Geo::DB;
  constexpr int LPB = Geo::LOADS_PER_BLOCK;

  const AttnArgs& a = prm.a;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
  const int lane = (int)threadIdx.x % kWave;
  const int kvh = wave;                                  // one KV head per wave, no head groups
  if (kvh >= a.Hkv) return;                              // no workgroup barrier below: safe
  const int h0 = kvh * prm.G;
  const int nh = prm.G;                                  // <= kRowHeads
  const int qcol = lane % 16, jj = lane / 16;

  // (Everything about an item is the same for all lanes; the values are pinned to scalar
  // registers so that the records and block ids are fetched by scalar loads, which the count of
  // vector loads in flight does not see.)
  auto uni = [](int v) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(v); };
  int it = uni(prm.w.wg_first[wg]);
  const int it_end = uni(prm.w.wg_first[wg + 1]);
  if (it >= it_end) return;

  // ---- items ----
  struct Item {
    int qtok, b1, t1, nparts, blk0;
    const __attribute__((address_space(4))) int32_t* table;
  };
  // Constant address space: read by scalar loads (none of this changes while the kernel runs).
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const const_i32_ptr recs = (const_i32_ptr)(uintptr_t)prm.w.item_rec;
  const const_i32_ptr spans = (const_i32_ptr)(uintptr_t)prm.w.item_span;
  auto load_item = [&](int i, int& b0_out) __attribute__((always_inline)) -> Item {
    i = uni(i);
    const const_i32_ptr rp = recs + 4 * (int64_t)i;      // {seq, qtok, ctx, part | nparts << 16}
    const const_i32_ptr sp = spans + 4 * (int64_t)i;     // {first block, end block, id of the first block, run}
    const int seq = rp[0], qtok = rp[1], ctx = rp[2], pw = rp[3];
    const int b0 = sp[0], b1 = sp[1], blk0 = sp[2];
    Item x;
    x.qtok = qtok;
    x.b1 = b1;
    x.t1 = min(ctx, b1 * kBlockSize);
    x.nparts = (int)((uint32_t)pw >> 16);
    x.blk0 = blk0;
    x.table = (const_i32_ptr)(uintptr_t)(a.block_tables + (int64_t)seq * a.max_blocks);
    b0_out = b0;
    return x;
  };
  auto block_id = [&](const_i32_ptr table, int b) __attribute__((always_inline)) -> int { return table[uni(b)]; };
  // Query rows travel through LDS like the K/V blocks: each lane requests its own fragments into
  // a 16-byte cell of its own (global->LDS, no destination registers, so nothing but the count
  // of loads in flight orders them) and reads them back once they are known to have landed.
  unsigned char* const q_stage = smem + (size_t)a.Hkv * R * Geo::SLOT_BYTES + (size_t)wave * KS * 1024;
  const uint32_t q_stage_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)q_stage;
  auto request_q = [&](int qtok) __attribute__((always_inline)) {
    const int col = qcol < nh ? qcol : 0;                // padding columns: a valid row, zeroed after the read
    const uint16_t* qp = a.q + ((int64_t)qtok * a.Hq + h0 + col) * D + jj * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      __builtin_amdgcn_global_load_lds((gbl_void_t)(qp + ks * 32), (lds_void_t)(q_stage + ks * 1024), 16, 0, 0);
  };
  auto read_q = [&](bf16x8_t (&dst)[KS]) __attribute__((always_inline)) {
    const uint32_t cell = q_stage_lds + (uint32_t)lane * 16u;
    uint4 v[KS];
    if constexpr (KS == 4) {
      asm volatile(
          "ds_read_b128 %0, %4\n\t"
          "ds_read_b128 %1, %4 offset:1024\n\t"
          "ds_read_b128 %2, %4 offset:2048\n\t"
          "ds_read_b128 %3, %4 offset:3072\n\t"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
          : "v"(cell)
          : "memory");
    } else {
      asm volatile(
          "ds_read_b128 %0, %2\n\t"
          "ds_read_b128 %1, %2 offset:1024\n\t"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(v[0]), "=&v"(v[1])
          : "v"(cell)
          : "memory");
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      dst[ks] = __builtin_bit_cast(bf16x8_t, qcol < nh ? v[ks] : make_uint4(0u, 0u, 0u, 0u));
  };

  // ---- loader (as in rows_body) ----
  unsigned char* const ring = smem + (size_t)wave * R * Geo::SLOT_BYTES;
  const int ld_row = lane / CPR, ld_pos = lane % CPR;
  const uint32_t tok_stride = (uint32_t)a.Hkv * ROWB;
  const int64_t blk_bytes = (int64_t)kBlockSize * tok_stride;
  const unsigned char* const k_bytes = reinterpret_cast<const unsigned char*>(a.k_pool);
  const unsigned char* const v_bytes = reinterpret_cast<const unsigned char*>(a.v_pool);
  const unsigned char* const zero_line = reinterpret_cast<const unsigned char*>(prm.w.zero_line);
  auto issue_block = [&](int bid, int b, int t1, int slot) __attribute__((always_inline)) {
    const unsigned char* kb = k_bytes + (int64_t)bid * blk_bytes + (uint32_t)kvh * ROWB;
    const unsigned char* vb = v_bytes + (int64_t)bid * blk_bytes + (uint32_t)kvh * ROWB;
    unsigned char* ks_base = ring + slot * Geo::SLOT_BYTES;
    unsigned char* vs_base = ks_base + Geo::TENSOR_BYTES;
#pragma unroll
    for (int i = 0; i < IPB; ++i) {
      const int n = i * TPI + ld_row;
      const unsigned char* kp = kb + (uint32_t)n * tok_stride + ((ld_pos ^ k_swz<D, EB>(n)) * 16);
      const unsigned char* vp = vb + (uint32_t)n * tok_stride + ((ld_pos ^ v_swz<D, EB>(n)) * 16);
      if (b * kBlockSize + n >= t1) vp = zero_line + ld_pos * 16;    // beyond the item's tokens: V := 0
      __builtin_amdgcn_global_load_lds((gbl_void_t)kp, (lds_void_t)(ks_base + i * 1024), 16, 0, kStreamOnce);
      __builtin_amdgcn_global_load_lds((gbl_void_t)vp, (lds_void_t)(vs_base + i * 1024), 16, 0, kStreamOnce);
    }
  };

  // ---- fragment offsets inside a slot (as in rows_body) ----
  int k_off[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    if constexpr (KV8)
      k_off[ks] = qcol * ROWB + (((ks * 2 + jj / 2) ^ k_swz<D, EB>(qcol)) * 16) + (jj % 2) * 8;
    else
      k_off[ks] = qcol * ROWB + (((ks * 4 + jj) ^ k_swz<D, EB>(qcol)) * 16);
  }
  constexpr int VT = KV8 ? DB / 2 : DB;
  const int v_row = jj * 4 + (lane % 16) / 4;
  const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring;
  uint32_t v_off[VT];
#pragma unroll
  for (int db = 0; db < VT; ++db)
    v_off[db] = Geo::TENSOR_BYTES + v_row * ROWB + (((2 * db + (lane % 4) / 2) ^ v_swz<D, EB>(v_row)) * 16) + (lane % 2) * 8;

  // ---- per-item state ----
  f32x4_t o[DB];
  float m_run, l_run;
  auto reset = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int db = 0; db < DB; ++db) o[db] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    m_run = kMinusBig;
    l_run = 0.f;
  };
  const float scale = a.scale_log2e;

  // Output of an item: the row itself if it has one partition, else its partial for the merge
  // kernel (nontemporal: written once, read once; see rows_body).  The stores are what an item
  // costs beyond its blocks (measured: 1,024 rows of 352 tokens 244 us against 226 for 256 rows of
  // 1,408; without the partials 235 and 221, without any store 221 and 220), and it is their
  // number that costs, not where in the run they are issued: with finished items' results held in
  // registers and stored at the end of the run the times were the same.  The planner prices a
  // row's start at two blocks for them.
  auto finish = [&](const Item& x, int item) __attribute__((always_inline)) {
    const float l_tot = cross16_sum(l_run);
    if (qcol >= nh) return;
    const int h = h0 + qcol;
    if (x.nparts == 1) {
      const float inv = a.out_scale / l_tot;
      if constexpr (KV8) {
        const int64_t ob = ((int64_t)x.qtok * a.Hq + h) * D + jj * 8;
#pragma unroll
        for (int j = 0; j < DB / 2; ++j) {
          float y[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) { y[2 * e] = o[2 * j][e] * inv; y[2 * e + 1] = o[2 * j + 1][e] * inv; }
          if (a.out_bf16) {
            uint4 pk;
            pk.x = (uint32_t)f32_to_bf16_rne(y[0]) | ((uint32_t)f32_to_bf16_rne(y[1]) << 16);
            pk.y = (uint32_t)f32_to_bf16_rne(y[2]) | ((uint32_t)f32_to_bf16_rne(y[3]) << 16);
            pk.z = (uint32_t)f32_to_bf16_rne(y[4]) | ((uint32_t)f32_to_bf16_rne(y[5]) << 16);
            pk.w = (uint32_t)f32_to_bf16_rne(y[6]) | ((uint32_t)f32_to_bf16_rne(y[7]) << 16);
            *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(a.out) + ob + j * 32) = pk;
          } else {
            float* dst = reinterpret_cast<float*>(a.out) + ob + j * 32;
            *reinterpret_cast<float4*>(dst) = make_float4(y[0], y[1], y[2], y[3]);
            *reinterpret_cast<float4*>(dst + 4) = make_float4(y[4], y[5], y[6], y[7]);
          }
        }
      } else {
        const int64_t ob = ((int64_t)x.qtok * a.Hq + h) * D + jj * 4;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const float x0 = o[db][0] * inv, x1 = o[db][1] * inv, x2 = o[db][2] * inv, x3 = o[db][3] * inv;
          if (a.out_bf16) {
            uint2 pk;
            pk.x = (uint32_t)f32_to_bf16_rne(x0) | ((uint32_t)f32_to_bf16_rne(x1) << 16);
            pk.y = (uint32_t)f32_to_bf16_rne(x2) | ((uint32_t)f32_to_bf16_rne(x3) << 16);
            // (plain stores: with the nontemporal hint, which helps the partials, a row's output
            // costs the run more - 1,024 rows of 352 tokens 255 us against 244)
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + ob + db * 16) = pk;
          } else {
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out) + ob + db * 16) = make_float4(x0, x1, x2, x3);
          }
        }
      }
    } else {
      const int64_t ph = (int64_t)item * a.Hq + h;
      if constexpr (KV8) {
        f32x4_t* pa = reinterpret_cast<f32x4_t*>(prm.w.part_acc + ph * D + jj * 8);
#pragma unroll
        for (int j = 0; j < DB / 2; ++j) {
          __builtin_nontemporal_store(f32x4_t{o[2 * j][0], o[2 * j + 1][0], o[2 * j][1], o[2 * j + 1][1]}, pa + j * 8);
          __builtin_nontemporal_store(f32x4_t{o[2 * j][2], o[2 * j + 1][2], o[2 * j][3], o[2 * j + 1][3]}, pa + j * 8 + 1);
        }
      } else {
        f32x4_t* pa = reinterpret_cast<f32x4_t*>(prm.w.part_acc + ph * D + jj * 4);
#pragma unroll
        for (int db = 0; db < DB; ++db) __builtin_nontemporal_store(o[db], pa + db * 4);
      }
      if (jj == 0) *reinterpret_cast<float2*>(prm.w.part_ml + ph * 2) = make_float2(m_run, l_tot);
    }
  };

  // ---- the stream ----
  // `cur` is the item being consumed, block c_blk of it next; `nxt` the item after it and `nn` the
  // one after that (records are read two items early, query rows one item early).  The K/V
  // requests are exactly one block ahead of the consuming side: every step requests the block
  // after the one it consumes - the next block of cur, or the first block of nxt - and asks for
  // the id of the block after that (a scalar load) so that it is there one step later.
  //
  // What orders everything is the count of vector-memory operations in flight, which complete in
  // the order they were issued.  A step waits until only the block it has just requested (LPB
  // loads) may still be in flight, plus `extra`: the operations issued between the previous
  // step's request and this one's (an item's output stores, the next item's query rows), which
  // are younger than the block this step consumes and need not have completed.  Of an item's
  // stores only half are allowed for (DB / 2: the fewest any output form issues), the rest of
  // them, its oldest, are simply waited for.
  constexpr int kStoresAllowed = DB / 2;
  auto wait_block = [&](int extra) __attribute__((always_inline)) {
    if (extra == 0) wait_vmcnt<LPB>();
    else if (extra == KS) wait_vmcnt<LPB + KS>();
    else if (extra == kStoresAllowed) wait_vmcnt<LPB + kStoresAllowed>();
    else wait_vmcnt<LPB + kStoresAllowed + KS>();
  };
  int c_blk, nb0 = 0, nnb0 = 0;
  Item cur = load_item(it, c_blk), nxt = cur, nn = cur;
  bool has_nxt = it + 1 < it_end, has_nn = it + 2 < it_end;
  if (has_nxt) nxt = load_item(it + 1, nb0);
  if (has_nn) nn = load_item(it + 2, nnb0);
  bf16x8_t qf[KS];
  request_q(cur.qtok);
  issue_block(cur.blk0, c_blk, cur.t1, 0);
  int bid_next = 0;
  bool bid_next_valid = c_blk + 1 < cur.b1;
  if (bid_next_valid) bid_next = block_id(cur.table, c_blk + 1);
  reset();
  wait_vmcnt<LPB>();                                     // the first item's query rows are in
  read_q(qf);
  int extra = 0;
  if (has_nxt) { request_q(nxt.qtok); extra = KS; }

  for (int step = 0;; ++step) {
    const int slot = step & 1;
    const bool in_cur = c_blk + 1 < cur.b1;              // (all of this is uniform)
    const bool cross = !in_cur && has_nxt;
    // (The id of the block after the one requested here is asked for before the wait, which is
    // where a step spends its time: the scalar load returns under it.)
    if (in_cur) {
      const int bid = bid_next_valid ? bid_next : block_id(cur.table, c_blk + 1);
      issue_block(bid, c_blk + 1, cur.t1, slot ^ 1);
      bid_next_valid = c_blk + 2 < cur.b1;
      if (bid_next_valid) bid_next = block_id(cur.table, c_blk + 2);
      wait_block(extra);
    } else if (cross) {
      issue_block(nxt.blk0, nb0, nxt.t1, slot ^ 1);
      bid_next_valid = nb0 + 1 < nxt.b1;
      if (bid_next_valid) bid_next = block_id(nxt.table, nb0 + 1);
      wait_block(extra);
    } else {
      bid_next_valid = false;
      wait_vmcnt<0>();                                   // the run's last block
    }
    extra = 0;
    row_block_step<D, KV8>(ring_lds + (uint32_t)slot * Geo::SLOT_BYTES, k_off, v_off, qf, c_blk * kBlockSize + jj * 4,
                           cur.t1, scale, o, m_run, l_run);
    ++c_blk;
    if (c_blk < cur.b1) continue;
    // The item is done.  The next item's query rows were requested before its first block (which
    // this step requested): with only that block's loads left in flight they have landed, and the
    // query registers are free to take them before the output leaves.
    if (has_nxt) {
      wait_vmcnt<LPB>();
      read_q(qf);
    }
    finish(cur, it);
    if (!has_nxt) break;
    ++it;
    cur = nxt;
    c_blk = nb0;
    reset();
    nxt = nn;
    nb0 = nnb0;
    has_nxt = has_nn;
    has_nn = it + 2 < it_end;
    if (has_nn) nn = load_item(it + 2, nnb0);
    extra = kStoresAllowed;
    if (has_nxt) { request_q(nxt.qtok); extra += KS; }
  }
  wait_vmcnt<0>();
}

}  // namespace rows_impl
}  // namespace dsv
