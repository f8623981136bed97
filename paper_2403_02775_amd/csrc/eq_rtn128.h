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

// NT threads per workgroup; K = 16-byte chunks of a row per thread (cols <= 8 * K * NT); a batch
// is 16 / K rows, i.e. at most NT segments of 128 elements, which one round of the NT lanes emits.
// PER_ROW: one range per row (the paper's per-channel setting) instead of one per segment: the
// lanes of a row combine their extremes through LDS and all use the row's scale and zero-point.
template <int DT, int NT, int K, bool PER_ROW>
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
  const uint32_t upr = (uint32_t)md.cols >> 7;            // 128-element segments per row
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
    if (PER_ROW && tid < (uint32_t)RB) {                  // published by the barriers of the staging
      sc->rowmax_bits[tid] = 0;
      sc->rownegmin_bits[tid] = 0;
    }
    stage_loaded_rows<DT, NT, RB, K, Padded128Layout>(md, kp, row0, nb, pool, 0u, sc, v, [&] {
      batch_issue_loads<NT, RB, K>(md, row0 + RB, nb_next, v);
    });
    const uint32_t take = (uint32_t)nb * upr;              // <= NT
    const bool valid = tid < take;
    unsigned char* slot = pool + (size_t)(valid ? tid : 0u) * kSlotBytes;
    float vmin, vmax;
    slot_min_max<DT>(slot, vmin, vmax);
    const uint32_t my_row = valid ? tid / upr : 0u;        // row of the batch this lane's segment belongs to
    if (PER_ROW) {
      if (valid) {                                         // non-negative floats order like their bit patterns
        atomicMax(&sc->rowmax_bits[my_row], __float_as_uint(vmax));
        atomicMax(&sc->rownegmin_bits[my_row], __float_as_uint(0.0f - vmin));
      }
      __syncthreads();
      vmax = __uint_as_float(sc->rowmax_bits[my_row]);
      vmin = -__uint_as_float(sc->rownegmin_bits[my_row]);
    }
    float r0;
    int z;
    const bool active = init_unit(kp, vmin, vmax, r0, z);
    float s32, inv;
    scale_of(kp, active ? r0 : kp.D, s32, inv);            // an all-zero unit keeps s = 1
    if (valid) {
      emit_codes_to_slot<DT>(kp, slot, inv, z);
      if (!PER_ROW) {
        const int64_t gu = row0 * (int64_t)upr + tid;
        md.scales[gu] = s32;
        md.zps[gu] = (unsigned char)z;
      } else if (tid == my_row * upr) {
        md.scales[row0 + my_row] = s32;
        md.zps[row0 + my_row] = (unsigned char)z;
      }
    }
    __syncthreads();
    copy_wave_codes(kp, md, pool, row0 * (int64_t)upr, wave * kWave, take, lane);
    __syncthreads();                                       // the pool is refilled by the next batch
    nb = nb_next;
  }
}

}  // namespace eq
