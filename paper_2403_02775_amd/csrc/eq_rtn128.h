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
// LDS in front of the pool: the staging scratch, rounded up to whole 256 bytes.
template <int NT, int K>
constexpr size_t rtn_header_bytes() {
  return (sizeof(BatchScratch<16 / K, NT / kWave>) + 255u) & ~(size_t)255u;
}

// Wavefronts per SIMD the kernel is compiled for (256 registers).  Three per SIMD (168 registers)
// would let three three-wavefront workgroups share a compute unit instead of two, but the compiler
// then spills some 85 registers and rows of 22016 take 11.5 ms per 65B-shaped set instead of 9.1.
template <int NT>
constexpr int rtn_waves_per_simd() { return 2; }

template <int DT, int NT, int K, bool PER_ROW>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(rtn_waves_per_simd<NT>(), rtn_waves_per_simd<NT>()))) void quantize_rtn128(
    const MatDesc* __restrict__ mats, const WorkItem* __restrict__ items, KParams kp) {
  constexpr int RB = 16 / K;
  // one row per batch over several wavefronts: every wavefront looks after a contiguous part of the
  // row (whole units), from the loads to the code stores (eq_rowbatch.h)
  constexpr bool WM = RB == 1 && NT > kWave;
  typedef BatchScratch<RB, NT / kWave> Scratch;
  extern __shared__ __align__(16) unsigned char smem[];
  Scratch* sc = reinterpret_cast<Scratch*>(smem);
  unsigned char* pool = smem + rtn_header_bytes<NT, K>();
  const WorkItem it = items[blockIdx.x];
  const MatDesc md = mats[it.mat];
  const uint32_t upr = (uint32_t)md.cols >> 7;            // 128-element segments per row
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int64_t row_end = (int64_t)it.row0 + it.nrows;
  uint32_t part_c0, part_c1;
  wave_part<NT, WM>((uint32_t)md.cols >> 3, part_c0, part_c1);
  // the unit this lane emits: unit `lane` of its wavefront's part, or unit `tid` of the batch
  const uint32_t w_first = WM ? part_c0 >> 4 : wave * kWave;

  auto rows_at = [&](int64_t row) { return (int)max((int64_t)0, min((int64_t)RB, row_end - row)); };

  uint4 v[RB][K];
  int nb = rows_at(it.row0);
  batch_issue_loads<NT, RB, K, WM>(md, it.row0, nb, v);
  const int64_t step = it.stride ? it.stride : RB;        // rows from one batch of this workgroup to its next
  for (int64_t row0 = it.row0; row0 < row_end; row0 += step) {
    // the next batch's loads start half-way through this one (past the end: zero-sized buffers,
    // no traffic), so that they fly under the outlier writes and the emission
    const int nb_next = rows_at(row0 + step);
    if (PER_ROW && tid < (uint32_t)RB) {                  // published by the barriers of the staging
      sc->rowmax_bits[tid] = 0;
      sc->rownegmin_bits[tid] = 0;
    }
    stage_loaded_rows<DT, NT, RB, K, Padded128Layout, WM>(md, kp, row0, nb, pool, 0u, nullptr, sc, v, [&] {
      batch_issue_loads<NT, RB, K, WM>(md, row0 + step, nb_next, v);
    });
    const uint32_t take = WM ? part_c1 >> 4 : (uint32_t)nb * upr;   // end of the units this wavefront emits
    const uint32_t slot_i = w_first + lane;
    const bool valid = slot_i < take;
    unsigned char* slot = pool + (size_t)(valid ? slot_i : 0u) * kSlotBytes;
    float vmin, vmax;
    slot_min_max<DT>(slot, vmin, vmax);
    const uint32_t my_row = (RB > 1 && valid) ? slot_i / upr : 0u;   // row of the batch this lane's segment belongs to
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
    // the range: the initial one (an all-zero unit keeps s = 1), or the one an optimisation that ran
    // before this kernel left for the row
    const bool given = PER_ROW && kp.range_given;
    scale_of(kp, given ? md.range[row0 + my_row] : active ? r0 : kp.D, s32, inv);
    if (valid) {
      // symmetric mode at the initial range: |x| <= r0, so no level leaves [-D, D] and Eq. 1's clamp
      // is the identity (uniform branch)
      if (kp.mode == EQ_SYMMETRIC && !given) emit_codes_to_slot<DT, true>(kp, slot, inv, z);
      else emit_codes_to_slot<DT, false>(kp, slot, inv, z);
      if (!PER_ROW) {
        const int64_t gu = row0 * (int64_t)upr + slot_i;
        md.scales[gu] = s32;
        md.zps[gu] = (unsigned char)z;
      } else if (slot_i == my_row * upr) {
        md.scales[row0 + my_row] = s32;
        md.zps[row0 + my_row] = (unsigned char)z;
      }
    }
    // the wavefront copies the codes of its own 64 units: only its own lanes have to be done
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
    copy_wave_codes(kp, md, pool, row0 * (int64_t)upr, w_first, take, lane);
    // The pool is refilled by the next batch.  Interleaved chunks: by every wavefront everywhere, so
    // all wait for the copies; wavefront-major: each part by its own wavefront.  (With one range
    // per row the extremes are reset by the next batch while another wavefront may still read them.)
    if (!WM || PER_ROW) __syncthreads();
    nb = nb_next;
  }
}

}  // namespace eq
