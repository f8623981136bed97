// Zero optimisation steps (iters = 0): outlier isolation followed by round-to-nearest at the
// initial range (Algorithm 1 without its second step), group size 128.
//
// A workgroup takes one batch of rows at a time through statistics, outlier compaction
// (eq_rowbatch.h) and code emission; the 128-bit loads of its next batch start as soon as the
// registers that held this one are free.  Emission is the unit-per-lane scheme of
// eq_fused128.h (the transposition through the padded LDS slots makes both the HBM reads and
// the code writes fully coalesced), one round per batch, nothing carried over.
#pragma once

#include "eq_fused128.h"

namespace eq {

// NT threads (256, two workgroups per compute unit; 512 for rows longer than 8192, one per compute
// unit); K = 16-byte chunks of a row per thread (cols <= 8 * K * NT); a batch is 16 / K rows,
// i.e. at most NT units, which one round of the NT lanes emits.
template <int DT, int NT, int K>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void quantize_rtn128(
    const MatDesc* __restrict__ mats, const WorkItem* __restrict__ items, KParams kp) {
  constexpr int RB = 16 / K;
  typedef BatchScratch<RB, NT / kWave> Scratch;
  static_assert(sizeof(Scratch) <= kLdsHeader, "staging scratch must fit the LDS header");
  extern __shared__ __align__(16) unsigned char smem[];
  Scratch* sc = reinterpret_cast<Scratch*>(smem);
  unsigned char* pool = smem + kLdsHeader;
  const WorkItem it = items[blockIdx.x];
  const MatDesc md = mats[it.mat];
  const uint32_t upr = (uint32_t)md.upr;
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int64_t row_end = (int64_t)it.row0 + it.nrows;

  auto rows_at = [&](int64_t row) { return (int)max((int64_t)0, min((int64_t)RB, row_end - row)); };

  uint4 v[RB][K];
  int nb = rows_at(it.row0);
  batch_issue_loads<NT, RB, K>(md, it.row0, nb, v);
  for (int64_t row0 = it.row0; row0 < row_end; row0 += RB) {
    // the next batch's loads start half-way through this one (past the end: zero-sized buffers,
    // no traffic), so that they fly under the compaction and the emission
    const int nb_next = rows_at(row0 + RB);
    stage_loaded_rows<DT, NT, RB, K, Padded128Layout>(md, kp, row0, nb, pool, 0u, sc, v, [&] {
      batch_issue_loads<NT, RB, K>(md, row0 + RB, nb_next, v);
    });
    const uint32_t take = (uint32_t)nb * upr;              // <= NT
    const bool valid = tid < take;
    unsigned char* slot = pool + (size_t)(valid ? tid : 0u) * kSlotBytes;
    float vmin, vmax;
    slot_min_max<DT>(slot, vmin, vmax);
    float r0;
    int z;
    const bool active = init_unit(kp, vmin, vmax, r0, z);
    float s32, inv;
    scale_of(kp, active ? r0 : kp.D, s32, inv);            // an all-zero unit keeps s = 1
    if (valid) {
      emit_codes_to_slot<DT>(kp, slot, inv, z);
      const int64_t gu = row0 * (int64_t)upr + tid;
      md.scales[gu] = s32;
      md.zps[gu] = (unsigned char)z;
    }
    __syncthreads();
    copy_wave_codes(kp, md, pool, row0 * (int64_t)upr, wave * kWave, take, lane);
    __syncthreads();                                       // the pool is refilled by the next batch
    nb = nb_next;
  }
}

}  // namespace eq
