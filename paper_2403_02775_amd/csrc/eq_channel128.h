// Per-channel rows (one range per output channel, the setting of the paper's main tables;
// Sec. 5, Setup) on the lane-per-128-elements machinery of eq_fused128.h.
//
// A row of `cols` = 128 * segs elements is spread over segs consecutive lanes; a workgroup of
// 256 lanes takes floor(256 / segs) rows per round.  Every lane holds the fixed-point planes of
// its segment in registers and evaluates its share of the two exact sums of Eq. 2 exactly as
// the group kernel does; the shares are integers in a fixed-point format common to the row
// (one exponent from the row's largest magnitude), so the row totals are formed with integer
// LDS atomics: exact, hence independent of the order in which lanes arrive.  After one barrier
// per evaluation every lane of the row reads the totals and takes the same Adam step
// (Sec. 4.2 / Algorithm 1), redundantly, in binary64.
//
// Rotation of the accumulators: evaluation p adds into set p mod 3; after its barrier one lane
// per row clears set (p + 2) mod 3, which was last read before that barrier and is next
// written after the following one, so one barrier per evaluation suffices.
//
// A row whose values are not all multiples of 2^-q (possible for bf16) is evaluated with
// binary64 partial sums combined in lane order (the whole round then repeats the optimisation
// that way: the branch has to be uniform for the barriers).
#pragma once

#include "eq_fused128.h"

namespace eq {

constexpr int kChanThreads = 256;
constexpr int kChanMaxRows = 16;     // rows per round (rows shorter than 2048 go to the general kernel)
constexpr int kChanHeader = 7168;    // LDS in front of the pool: staging scratch, then ChanScratch
constexpr int kChanScratchOff = 4096;

struct RowAcc {
  uint32_t max_bits, negmin_bits;    // bit patterns of max(x, 0) and max(-x, 0) over the row
  uint32_t cc[3];                    // sum c^2, three rotating sets
  uint32_t pad_;
  unsigned long long xc[3];          // sum (x 2^q) c as a two's-complement 64-bit integer
};
struct ChanScratch {
  RowAcc acc[kChanMaxRows];
  uint32_t inexact;                  // some row of the round cannot use the fixed-point form
  uint32_t keep_bf16;                // some segment of the round has no exact fp16 form (slot_fits_f16)
  uint32_t pad_[2];
  double part[kChanThreads];         // binary64 shares of the lanes (slow path only)
};
static_assert(kChanScratchOff + sizeof(ChanScratch) <= kChanHeader, "LDS header too small");

// Sums over aligned groups of lanes with data-parallel-primitive adds (no LDS): after the four
// row_shr steps lane 15 of every 16-lane row holds the row's sum; WIDE adds row 0 into row 1
// and row 2 into row 3 (row_bcast:15), so that lanes 31 and 63 hold the sums of their 32-lane
// halves.  Other lanes hold partial sums.  32-bit wrap-around cannot occur for the callers:
// |level| <= 15 and 16-bit plane values over 32 * 128 elements stay below 2^31.
template <bool WIDE>
__device__ __forceinline__ int group_sum_dpp(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);   // row_shr:8
  if (WIDE) v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, true);   // row_bcast:15 into rows 1 and 3
  return v;
}

// K = 16-byte chunks of a row per thread (cols <= 8 * K * 256); rows are staged 16 / K at a time.
// FULL: cols == 8 * K * 256 exactly, i.e. rows of 2048, 4096 or 8192 elements over 16, 32 or 64 lanes:
// the lane count is then a compile-time constant and the in-wavefront combination is the only path.
template <int DT, int K, bool FULL>
__global__ __launch_bounds__(kChanThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void quantize_channels128(
    const MatDesc* __restrict__ mats, const WorkItem* __restrict__ items, KParams kp) {
  constexpr int NT = kChanThreads;
  constexpr int RB = 16 / K;
  typedef BatchScratch<RB, NT / kWave> Scratch;
  static_assert(sizeof(Scratch) <= kChanScratchOff, "staging scratch overlaps the row accumulators");
  extern __shared__ __align__(16) unsigned char smem[];
  Scratch* sc = reinterpret_cast<Scratch*>(smem);
  ChanScratch* cs = reinterpret_cast<ChanScratch*>(smem + kChanScratchOff);
  unsigned char* pool = smem + kChanHeader;
  const WorkItem it = items[blockIdx.x];
  const MatDesc md = mats[it.mat];
  static_assert(!FULL || K <= 4, "in-wavefront sums serve rows of up to 64 lanes");
  const uint32_t segs = FULL ? 16u * K : (uint32_t)md.cols >> 7;   // lanes per row
  const uint32_t R = min((uint32_t)NT / segs, (uint32_t)kChanMaxRows);
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const uint32_t my_row = tid / segs, seg = tid - my_row * segs;
  const int64_t row_end = (int64_t)it.row0 + it.nrows;

  for (int64_t row0 = it.row0; row0 < row_end; row0 += R) {
    const uint32_t nr = (uint32_t)min((int64_t)R, row_end - row0);
    if (tid < (uint32_t)kChanMaxRows) {
      RowAcc z0;
      z0.max_bits = z0.negmin_bits = z0.pad_ = 0;
      z0.cc[0] = z0.cc[1] = z0.cc[2] = 0;
      z0.xc[0] = z0.xc[1] = z0.xc[2] = 0;
      cs->acc[tid] = z0;
    }
    if (tid == 0) {
      cs->inexact = 0;
      cs->keep_bf16 = 0;
    }
    for (uint32_t b = 0; b < nr; b += RB) {     // ends with a barrier, which also publishes the clears above
      uint32_t ch0 = b * segs * 16u;
      // opaque on purpose: with a compile-time lane count the compiler would otherwise keep every
      // thread's 16 pool addresses alive across the whole kernel, in scratch memory
      asm volatile("" : "+s"(ch0));
      stage_rows_batch<DT, NT, RB, K, Padded128Layout>(md, kp, row0 + b, (int)min((uint32_t)RB, nr - b), pool, ch0, nullptr, sc);
    }

    const bool valid = my_row < nr;
    unsigned char* slot = pool + (size_t)(valid ? tid : 0u) * kSlotBytes;
    RowAcc* ra = &cs->acc[valid ? my_row : 0u];

    // ---- range and zero-point of the row; the row's fixed-point exponent ----
    {
      float vmin, vmax;
      slot_min_max<DT>(slot, vmin, vmax);
      if (valid) {                               // non-negative floats order like their bit patterns
        atomicMax(&ra->max_bits, __float_as_uint(vmax));
        atomicMax(&ra->negmin_bits, __float_as_uint(0.0f - vmin));
      }
    }
    __syncthreads();
    const float vmax = __uint_as_float(ra->max_bits), vmin = -__uint_as_float(ra->negmin_bits);
    float r0;
    int z;
    const bool active = init_unit(kp, vmin, vmax, r0, z);
    const float clo = (float)(-z), chi = (float)(kp.L - z);
    const float mlo = clo + kMagic, mhi = chi + kMagic;
    const float r_start = active ? r0 : kp.D;
    int E = 0;
    (void)frexpf(fmaxf(-vmin, vmax), &E);
    const int q = 30 - E;
    // bf16 rows take the fp16 form of their values when every segment of the round has one
    // (see slot_fits_f16; the shift comes from the row's largest magnitude).  The choice is
    // uniform over the workgroup because the code below synchronises.
    const int shift_f16 = 15 - E;
    bool as_f16 = false;
    if (DT == EQ_BF16) {
      if (valid && !slot_fits_f16(slot, shift_f16)) cs->keep_bf16 = 1u;     // benign race: every writer stores 1
      __syncthreads();
      as_f16 = cs->keep_bf16 == 0;
      if (as_f16 && valid) slot_bf16_to_f16(slot, shift_f16);
    }
    auto rest = [&](auto dx, const int shift) {
      constexpr int DX = decltype(dx)::value;
      const float unshift = ldexpf(1.0f, -shift);            // exact power of two
      uint32_t H[kPairs], Lo[kPairs];
      uint32_t frac_bits = 0;
      const bool need_test = !(DX == EQ_F16 && __all(q - shift >= 24));
      if (need_test) build_planes<DX, true>(slot, q - shift, H, Lo, frac_bits);
      else build_planes<DX, false>(slot, q - shift, H, Lo, frac_bits);
      if (valid && (frac_bits << 1) != 0) cs->inexact = 1u;      // benign race: every writer stores 1

      // How the lanes of a row combine their shares (all three choices give the same exact sums):
      //  * a row that lies inside one wavefront in an aligned group of 16, 32 or 64 lanes needs no
      //    LDS and no barrier: group sums by lane shifts, then every lane fetches its group's sums;
      //  * otherwise the shares go to the row's LDS accumulators, one barrier per evaluation;
      //    a wavefront whose 32-lane halves each hold lanes of one row only adds the two half sums
      //    instead of 64 single shares (64 atomics on one address serialise).
      // The 32-bit group sums need |level| <= 15, i.e. at most 4 bits.
      const bool small_levels = kp.bits <= 4;
      // uniform over the grid (FULL kernels are launched for code widths of at most 4 bits only)
      const bool in_wave = FULL || (small_levels && (segs == 16u || segs == 32u || segs == 64u));
      const uint32_t half_row = (uint32_t)__shfl((int)my_row, (int)(lane & 32u));
      const bool half_valid = __shfl((int)valid, (int)(lane & 32u)) != 0;
      const bool halves_uniform = small_levels && __all(!valid || my_row == half_row);      // uniform over the wavefront
      RowAcc* ha = &cs->acc[half_valid ? half_row : 0u];

      uint32_t pass = 0;                           // evaluations so far in this round (selects the accumulator set)
      float r_sel = optimise_range(kp, r_start, [&](float inv, double& A, double& B) {
        int cc, hc, lc;
        eval_sums<DX>(slot, H, Lo, inv * unshift, mlo, mhi, cc, hc, lc);
        if (in_wave) {
          if (!valid) cc = hc = lc = 0;
          int tc, th, tl;
          long long xq;
          if (segs == 16u) {
            cc = group_sum_dpp<false>(cc);
            hc = group_sum_dpp<false>(hc);
            lc = group_sum_dpp<false>(lc);
            const int src = (int)(lane | 15u);
            tc = __shfl(cc, src);
            th = __shfl(hc, src);
            tl = __shfl(lc, src);
            xq = (long long)th * 65536 + (long long)tl;
          } else {
            cc = group_sum_dpp<true>(cc);
            hc = group_sum_dpp<true>(hc);
            lc = group_sum_dpp<true>(lc);
            const int c0 = __builtin_amdgcn_readlane(cc, 31), c1 = __builtin_amdgcn_readlane(cc, 63);
            const long long x0 = (long long)__builtin_amdgcn_readlane(hc, 31) * 65536 + (long long)__builtin_amdgcn_readlane(lc, 31);
            const long long x1 = (long long)__builtin_amdgcn_readlane(hc, 63) * 65536 + (long long)__builtin_amdgcn_readlane(lc, 63);
            if (segs == 64u) {
              tc = c0 + c1;
              xq = x0 + x1;
            } else {
              tc = lane < 32u ? c0 : c1;
              xq = lane < 32u ? x0 : x1;
            }
          }
          A = (double)tc;
          B = ldexp((double)xq, -q);
          return;
        }
        const uint32_t set = pass % 3u;
        if (halves_uniform) {
          if (!valid) cc = hc = lc = 0;
          cc = group_sum_dpp<true>(cc);
          hc = group_sum_dpp<true>(hc);
          lc = group_sum_dpp<true>(lc);
          if ((lane & 31u) == 31u && half_valid) {
            atomicAdd(&ha->cc[set], (uint32_t)cc);
            atomicAdd(&ha->xc[set], (unsigned long long)((long long)hc * 65536 + (long long)lc));
          }
        } else if (valid) {
          atomicAdd(&ra->cc[set], (uint32_t)cc);
          atomicAdd(&ra->xc[set], (unsigned long long)((long long)hc * 65536 + (long long)lc));
        }
        __syncthreads();
        A = (double)ra->cc[set];
        B = ldexp((double)(long long)ra->xc[set], -q);            // the integer is exact; one rounding at most
        if (valid && seg == 0) {
          const uint32_t clr = (pass + 2u) % 3u;
          ra->cc[clr] = 0;
          ra->xc[clr] = 0;
        }
        ++pass;
      });
      __syncthreads();                             // the flag is complete (no evaluation ran when iters == 0)
      if (cs->inexact) {
        r_sel = optimise_range(kp, r_start, [&](float inv, double& A, double& B) {
          double a_lane, b_lane;
          eval_slot<DX>(slot, inv * unshift, clo, chi, a_lane, b_lane);
          b_lane = ldexp(b_lane, -shift);
          const uint32_t set = pass % 3u;
          cs->part[tid] = valid ? b_lane : 0.0;
          if (valid) atomicAdd(&ra->cc[set], (uint32_t)a_lane);
          __syncthreads();
          A = (double)ra->cc[set];
          double b = 0.0;
          const uint32_t first = (valid ? my_row : 0u) * segs;
          for (uint32_t j = 0; j < segs; ++j) b += cs->part[first + j];
          B = b;
          if (valid && seg == 0) ra->cc[(pass + 2u) % 3u] = 0;
          ++pass;
          __syncthreads();                         // part[] is rewritten by the next evaluation
        });
      }

      // ---- emit (Algorithm 1, third step) ----
      float s32, inv;
      scale_of(kp, r_sel, s32, inv);
      __syncthreads();
      if (valid) {
        emit_codes_to_slot<DX>(kp, slot, inv * unshift, z);
        if (seg == 0) {
          md.scales[row0 + my_row] = s32;
          md.zps[row0 + my_row] = (unsigned char)z;
        }
      }
    };
    if (DT == EQ_BF16 && as_f16) rest(std::integral_constant<int, EQ_F16>{}, shift_f16);
    else rest(std::integral_constant<int, DT>{}, 0);
    __syncthreads();
    copy_wave_codes(kp, md, pool, row0 * (int64_t)segs, wave * kWave, nr * segs, lane);
    __syncthreads();                             // the pool is overwritten by the next round's staging
  }
}

}  // namespace eq
