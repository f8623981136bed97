// Per-channel rows whose 128-element segments do not fill a workgroup: 11008, 13824, 17920 and
// 22016 columns, the MLP down-projections of the LLaMA shapes.  eq_channel128.h gives such a row
// one lane per 128 elements, i.e. 172 of 256 lanes for 22016 columns, with the other 84 idling
// through every evaluation.  Here a row is cut into LPR equal pieces of 2 P elements instead
// (22016 = 256 * 86, 11008 = 128 * 86, 13824 = 256 * 54, 17920 = 256 * 70), one per lane, so
// every lane of the workgroup works.  A piece is no
// longer a whole number of 16-byte chunks, so the row is staged linearly (eq_rowbatch.h) and each
// lane copies its P packed pairs into registers once, where they stay for all evaluations
// together with the two fixed-point planes: no LDS reads per pass.  The sums,
// their exact combination over the row (integer LDS atomics on rotating sets, 32-lane half sums
// first) and the Adam step are those of eq_channel128.h.
//
// 4-bit codes only (a pair of codes is then one byte of the row's stream, so the lanes' P-byte
// pieces need no bit shifting); other widths keep the 128-element kernel.  bf16 rows are served as
// they are (the values sit widened in registers either way); one whose values span more than the
// fixed-point planes hold takes the binary64 sums.
#pragma once

#include "eq_channel128.h"

namespace eq {

template <int DT, int P, int LPR>
__global__ __launch_bounds__(kChanThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void quantize_channels_split(
    const MatDesc* __restrict__ mats, const WorkItem* __restrict__ items, KParams kp) {
  constexpr int NT = kChanThreads;
  constexpr int R = NT / LPR;                  // rows per round
  constexpr int EPL = 2 * P;                   // elements per lane
  constexpr int K = (EPL * LPR / 8 + NT - 1) / NT <= 8 ? 8 : 16;   // staging chunks per thread and row
  constexpr int RB = 16 / K;
  static_assert(RB >= R, "a round is staged as one batch");
  static_assert(LPR % 64 == 0, "a wavefront holds lanes of one row only");
  typedef BatchScratch<RB, NT / kWave> Scratch;
  static_assert(sizeof(Scratch) <= kChanScratchOff, "staging scratch overlaps the row accumulators");
  extern __shared__ __align__(16) unsigned char smem[];
  Scratch* sc = reinterpret_cast<Scratch*>(smem);
  ChanScratch* cs = reinterpret_cast<ChanScratch*>(smem + kChanScratchOff);
  unsigned char* pool = smem + kChanHeader;    // R rows of values; later R rows of packed codes
  const WorkItem it = items[blockIdx.x];
  const MatDesc md = mats[it.mat];
  constexpr uint32_t cols = (uint32_t)EPL * LPR;                 // checked by the host
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
  const uint32_t my_row = tid / LPR, seg = tid % LPR;
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
    if (tid == 0) cs->inexact = 0;
    // ends with a barrier, which also publishes the clears above
    // (the outlier-mask bytes of the staging, one per 16-byte chunk, sit behind the R rows)
    stage_rows_batch<DT, NT, RB, K, LinearLayout>(md, kp, row0, (int)nr, pool, 0u, pool + (size_t)R * cols * 2u, sc);

    const bool valid = my_row < nr;
    RowAcc* ra = &cs->acc[valid ? my_row : 0u];

    // ---- the lane's piece, for good; its extremes ----
    uint32_t x[P];
    {
      const uint32_t* src = reinterpret_cast<const uint32_t*>(pool + ((size_t)(valid ? my_row : 0u) * cols + (size_t)seg * EPL) * 2u);
      float lmin = 0.0f, lmax = 0.0f;
      if (DT == EQ_F16) {
        uint32_t mnb = 0u, mxb = 0u;
#pragma unroll
        for (int j = 0; j < P; ++j) {
          x[j] = src[j];
          mnb = pk_min_f16(mnb, x[j]);
          mxb = pk_max_f16(mxb, x[j]);
        }
        const half2_t mn = __builtin_bit_cast(half2_t, mnb), mx = __builtin_bit_cast(half2_t, mxb);
        lmin = fminf((float)mn.x, (float)mn.y);
        lmax = fmaxf((float)mx.x, (float)mx.y);
      } else {
#pragma unroll
        for (int j = 0; j < P; ++j) {
          x[j] = src[j];
          const float x0 = widen16<DT>(x[j] & 0xFFFFu), x1 = widen16<DT>(x[j] >> 16);
          lmin = fminf(lmin, fminf(x0, x1));
          lmax = fmaxf(lmax, fmaxf(x0, x1));
        }
      }
      if (valid) {                               // non-negative floats order like their bit patterns
        atomicMax(&ra->max_bits, __float_as_uint(lmax));
        atomicMax(&ra->negmin_bits, __float_as_uint(0.0f - lmin));
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

    // ---- fixed-point planes of the piece: xi = x 2^q = 65536 H + L (see eq_fused128.h) ----
    uint32_t H[P], Lo[P];
    {
      uint32_t frac_bits = 0;
#pragma unroll
      for (int j = 0; j < P; ++j) {
        const float y0 = ldexpf(widen16<DT>(x[j] & 0xFFFFu), q), y1 = ldexpf(widen16<DT>(x[j] >> 16), q);
        const int i0 = (int)y0, i1 = (int)y1;
        frac_bits |= __float_as_uint(y0 - (float)i0) | __float_as_uint(y1 - (float)i1);
        Lo[j] = __builtin_amdgcn_perm((uint32_t)i1, (uint32_t)i0, 0x05040100u);
        H[j] = __builtin_amdgcn_perm((uint32_t)(i1 + 0x8000), (uint32_t)(i0 + 0x8000), 0x07060302u);
        asm volatile("" : "+v"(frac_bits));      // keep the running flag: no long-lived temporaries
      }
      if (valid && (frac_bits << 1) != 0) cs->inexact = 1u;      // benign race: every writer stores 1
    }

    uint32_t pass = 0;                           // evaluations so far in this round (selects the accumulator set)
    float r_sel = optimise_range(kp, r_start, [&](float inv, double& A, double& B) {
      int cc = 0, hc = 0, lc = 0;                // one accumulator per sum, taking turns (see eval_sums)
#pragma unroll
      for (int j = 0; j < P; ++j) {
        const float x0 = widen16<DT>(x[j] & 0xFFFFu), x1 = widen16<DT>(x[j] >> 16);
        const float t0 = __builtin_amdgcn_fmed3f(__builtin_fmaf(x0, inv, kMagic), mlo, mhi);
        const float t1 = __builtin_amdgcn_fmed3f(__builtin_fmaf(x1, inv, kMagic), mlo, mhi);
        const short2_t c = __builtin_bit_cast(short2_t, __builtin_amdgcn_perm(__float_as_uint(t1), __float_as_uint(t0), 0x05040100u));
        cc = __builtin_amdgcn_sdot2(c, c, cc, false);
        hc = __builtin_amdgcn_sdot2(__builtin_bit_cast(short2_t, H[j]), c, hc, false);
        lc = __builtin_amdgcn_sdot2(__builtin_bit_cast(short2_t, Lo[j]), c, lc, false);
      }
      if (!valid) cc = hc = lc = 0;
      // 32-lane half sums (no 32-bit wrap-around: 32 * 2 P elements, |level| <= 15, 16-bit planes)
      cc = group_sum_dpp<true>(cc);
      hc = group_sum_dpp<true>(hc);
      lc = group_sum_dpp<true>(lc);
      const uint32_t set = pass % 3u;
      if ((lane & 31u) == 31u && valid) {
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
      // a row with values that are not multiples of 2^-q: binary64 shares combined in lane order
      r_sel = optimise_range(kp, r_start, [&](float inv, double& A, double& B) {
        int a_lane = 0;
        double b_lane = 0.0;
#pragma unroll
        for (int j = 0; j < P; ++j) {        // unrolled: the piece lives in registers
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const float xv = widen16<DT>((x[j] >> (16 * h)) & 0xFFFFu);
            const float c = level_of(xv, inv, clo, chi);
            a_lane += (int)c * (int)c;
            b_lane += (double)(xv * c);
          }
        }
        const uint32_t set = pass % 3u;
        cs->part[tid] = valid ? b_lane : 0.0;
        if (valid) atomicAdd(&ra->cc[set], (uint32_t)a_lane);
        __syncthreads();
        A = (double)ra->cc[set];
        double b = 0.0;
        const uint32_t first = (valid ? my_row : 0u) * LPR;
#pragma unroll 4
        for (uint32_t j = 0; j < (uint32_t)LPR; ++j) b += cs->part[first + j];
        B = b;
        if (valid && seg == 0) ra->cc[(pass + 2u) % 3u] = 0;
        ++pass;
        __syncthreads();                         // part[] is rewritten by the next evaluation
      });
    }

    // ---- emit (Algorithm 1, third step): a pair of 4-bit codes is one byte of the row's stream ----
    float s32, inv;
    scale_of(kp, r_sel, s32, inv);
    __syncthreads();                             // the pool now takes the codes
    if (valid) {
      // the zero-point rides in the rounding constant, an odd one as z + 1 (see emit_codes_to_slot)
      const int zodd = z & 1;
      const float mz = kMagic + (float)(z + zodd), ulo = kMagic + (float)zodd, uhi = kMagic + (float)(kp.L + zodd);
      unsigned char* dst = pool + (size_t)my_row * (cols / 2u) + (size_t)seg * P;
#pragma unroll
      for (int j = 0; j < P; ++j) {
        const float x0 = widen16<DT>(x[j] & 0xFFFFu), x1 = widen16<DT>(x[j] >> 16);
        const uint32_t f0 = __float_as_uint(__builtin_amdgcn_fmed3f(__builtin_fmaf(x0, inv, mz), ulo, uhi)) - (uint32_t)zodd;
        const uint32_t f1 = __float_as_uint(__builtin_amdgcn_fmed3f(__builtin_fmaf(x1, inv, mz), ulo, uhi)) - (uint32_t)zodd;
        dst[j] = (unsigned char)((f0 & 0xFu) | ((f1 & 0xFu) << 4));
      }
      if (seg == 0) {
        md.scales[row0 + my_row] = s32;
        md.zps[row0 + my_row] = (unsigned char)z;
      }
    }
    __syncthreads();
    {
      // the round's rows are contiguous in the code array: coalesced 128-bit stores
      const uint32_t n16 = nr * (cols / 32u);
      EQ_GLOBAL uint32_t* gdst = md.codes + row0 * (int64_t)md.words_per_row;
      for (uint32_t i = tid; i < n16; i += NT)
        global_store128(gdst + 4 * (size_t)i, *reinterpret_cast<const uint4*>(pool + (size_t)i * 16u));
    }
    __syncthreads();                             // the pool is overwritten by the next round's staging
  }
}

}  // namespace eq
