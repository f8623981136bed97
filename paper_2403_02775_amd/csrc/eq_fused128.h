// Fast path for group_size 128: one LANE owns one unit.
//
// A workgroup walks a range of rows.  Rows are staged into an LDS pool (eq_rowstage.h: one
// coalesced HBM read, statistics, outlier compaction); whenever the pool holds 256 units
// every lane takes one, pulls its 128 values into registers and runs ALL range-optimisation
// iterations there (Sec. 4.2 / Algorithm 1, second step) with no memory traffic at all:
// no cross-lane reduction, and the scalar Adam step is paid once per 128 elements.  Units
// left over (< 256) are carried to the next fill, so lanes idle only at the end of a range.
//
// Exact sums without binary64 in the inner loop: x is held as a block fixed-point integer
// xi = x * 2^q (|xi| < 2^30, q from the unit's largest magnitude), split into two signed
// 16-bit planes xi = 65536 H + L.  Codes c are small integers, so
//      A = sum c^2,   B * 2^q = 65536 sum H c + sum L c
// are three packed 16-bit integer dot products per element pair (v_dot2_i32_i16) that
// cannot overflow 32 bits (|H| <= 2^14, |L| <= 2^15, |c| <= 255, 128 terms).  A unit whose
// values are not all multiples of 2^-q (possible for bf16, or fp16 beyond 64) is evaluated
// by a plain binary64 loop instead; the result is the same exact sum either way.
#pragma once

#include "eq_common.h"
#include "eq_rowstage.h"

namespace eq {

constexpr int kG = 128;               // elements per unit
constexpr int kPairs = kG / 2;
constexpr int kSlotBytes = 272;       // 256 B of data + 16 B of padding (bank spread)
constexpr int kSlotChunks = 17;
constexpr int kCodeOff = 128;         // packed codes are assembled in the upper half of the slot
constexpr float kMagic = 12582912.0f; // 1.5 * 2^23: (t + kMagic) rounds t to an integer, ties to even

struct WorkItem {
  int32_t mat, row0, nrows, pad_;
};

typedef short short2_t __attribute__((ext_vector_type(2)));

// Bit patterns of (clamp(x * inv) + kMagic) for the two elements of a packed pair.  The low
// 16 bits of each pattern are the signed level c in two's complement.
template <int DT>
__device__ __forceinline__ void pair_levels(uint32_t w, float inv, float clo, float chi, uint32_t& f0, uint32_t& f1) {
  float t0, t1;
  if (DT == EQ_F16) {
    // fma(x, inv, 0) == x * inv (one rounding); written as fma so that the half -> float
    // widening folds into the instruction (v_fma_mix_f32)
    t0 = __builtin_fmaf(__half2float(__ushort_as_half((unsigned short)(w & 0xFFFFu))), inv, 0.0f);
    t1 = __builtin_fmaf(__half2float(__ushort_as_half((unsigned short)(w >> 16))), inv, 0.0f);
  } else {
    t0 = __uint_as_float(w << 16) * inv;
    t1 = __uint_as_float(w & 0xFFFF0000u) * inv;
  }
  f0 = __float_as_uint(__builtin_amdgcn_fmed3f(t0, clo, chi) + kMagic);
  f1 = __float_as_uint(__builtin_amdgcn_fmed3f(t1, clo, chi) + kMagic);
}

// One evaluation of Eq. 1 / Eq. 2 for the unit held in registers.
template <int DT>
__device__ __forceinline__ void eval_regs(const uint32_t (&xr)[kPairs], const uint32_t (&H)[kPairs],
                                          const uint32_t (&Lo)[kPairs], float inv, float clo, float chi, int q,
                                          double& A, double& B) {
  int a = 0, bh = 0, bl = 0;
#pragma unroll
  for (int k = 0; k < kPairs; ++k) {
    uint32_t f0, f1;
    // The packed pair is passed through an empty asm so that the optimiser treats it as new
    // in every evaluation: otherwise it hoists the 128 widenings out of the iteration loop
    // and the unit no longer fits the register file.
    uint32_t w = xr[k];
    asm volatile("" : "+v"(w));
    pair_levels<DT>(w, inv, clo, chi, f0, f1);
    const short2_t c = __builtin_bit_cast(short2_t, __builtin_amdgcn_perm(f1, f0, 0x05040100u));
    a = __builtin_amdgcn_sdot2(c, c, a, false);
    bh = __builtin_amdgcn_sdot2(__builtin_bit_cast(short2_t, H[k]), c, bh, false);
    bl = __builtin_amdgcn_sdot2(__builtin_bit_cast(short2_t, Lo[k]), c, bl, false);
  }
  A = (double)a;
  B = ldexp((double)bh * 65536.0 + (double)bl, -q);     // exact: |.| < 2^47
}

// The same from the LDS slot with a binary64 accumulation (units the fixed-point form cannot hold).
template <int DT>
__device__ __forceinline__ void eval_slot(const unsigned char* slot, float inv, float clo, float chi, double& A, double& B) {
  int a = 0;
  double b = 0.0;
  for (int ch = 0; ch < 16; ++ch) {
    const uint4 v = *reinterpret_cast<const uint4*>(slot + ch * 16);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float xv = widen16<DT>((w[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
      const float c = rintf(fminf(fmaxf(xv * inv, clo), chi));
      const int ci = (int)c;
      a += ci * ci;
      b += (double)(xv * c);
    }
  }
  A = (double)a;
  B = b;
}

// Adam on the range of one unit (per lane); `ev(inv, A, B)` evaluates the exact sums.
template <class Eval>
__device__ __forceinline__ float optimise_range(const KParams& kp, float r0, Eval&& ev) {
  float r32 = r0, r_sel = r0;
  double J_best = __builtin_inf();
  const double floor_r = (double)r0 * 0.0009765625;
  Adam ad;
  ad.init();
  for (int t = 0; t < kp.iters; ++t) {
    const float s32 = r32 / kp.D;
    const float inv = 1.0f / s32;
    double A, B, J, g;
    ev(inv, A, B);
    loss_and_grad(s32, A, B, kp.D, J, g);
    if (J < J_best) {
      J_best = J;
      r_sel = r32;
    }
    r32 = ad.step(kp, r32, g, floor_r);
  }
  if (kp.select == EQ_SELECT_LAST) return r32;
  if (kp.iters > 0) {
    const float s32 = r32 / kp.D;
    const float inv = 1.0f / s32;
    double A, B, J, g;
    ev(inv, A, B);
    loss_and_grad(s32, A, B, kp.D, J, g);
    if (J < J_best) r_sel = r32;
  }
  return r_sel;
}

template <int DT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void quantize_units128(const MatDesc* __restrict__ mats,
                                                              const WorkItem* __restrict__ items, KParams kp,
                                                              uint32_t pool_slots) {
  extern __shared__ __align__(16) unsigned char smem[];
  StageScratch* sc = reinterpret_cast<StageScratch*>(smem);
  unsigned char* pool = smem + 256;
  unsigned char* maskb = pool + (size_t)pool_slots * kSlotBytes;
  const WorkItem it = items[blockIdx.x];
  const MatDesc md = mats[it.mat];
  const uint32_t upr = (uint32_t)md.upr;
  const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const uint32_t code_words = 4u * (uint32_t)kp.bits;      // packed words per unit
  int64_t next_row = it.row0;
  const int64_t row_end = (int64_t)it.row0 + it.nrows;
  int64_t unit_base = (int64_t)it.row0 * upr;               // matrix-wide index of the unit in slot 0
  uint32_t pool_units = 0;

  while (true) {
    // ---- fill: stage rows until a full round of units is available ----
    while (next_row < row_end && pool_units < (uint32_t)kThreads && pool_units + upr <= pool_slots) {
      stage_row<DT, Padded128Layout>(md, kp, next_row, pool, pool_units * 16u, maskb, sc);
      pool_units += upr;
      ++next_row;
    }
    if (pool_units == 0) break;
    const bool last = next_row >= row_end;
    const uint32_t take = last ? pool_units : (pool_units / kThreads) * kThreads;
    if (take == 0) break;                                    // cannot happen with pool_slots >= 255 + upr

    for (uint32_t base = 0; base < take; base += kThreads) {
      const uint32_t slot_i = base + threadIdx.x;
      const bool valid = slot_i < take;
      unsigned char* slot = pool + (size_t)(valid ? slot_i : base) * kSlotBytes;

      // ---- the unit's values: LDS -> registers ----
      uint32_t xr[kPairs];
#pragma unroll
      for (int ch = 0; ch < 16; ++ch) {
        const uint4 v = *reinterpret_cast<const uint4*>(slot + ch * 16);
        xr[4 * ch + 0] = v.x; xr[4 * ch + 1] = v.y; xr[4 * ch + 2] = v.z; xr[4 * ch + 3] = v.w;
      }
      float vmin = 0.0f, vmax = 0.0f;
#pragma unroll
      for (int k = 0; k < kPairs; ++k) {
        const float x0 = widen16<DT>(xr[k] & 0xFFFFu), x1 = widen16<DT>(xr[k] >> 16);
        vmin = fminf(vmin, fminf(x0, x1));
        vmax = fmaxf(vmax, fmaxf(x0, x1));
      }
      float r0;
      int z;
      const bool active = init_unit(kp, vmin, vmax, r0, z);
      const float clo = (float)(-z), chi = (float)(kp.L - z);
      const float r_start = active ? r0 : kp.D;              // an all-zero unit keeps s = 1

      // ---- block fixed point: xi = x * 2^q, |xi| < 2^30, split into 16-bit planes ----
      int E = 0;
      (void)frexpf(fmaxf(-vmin, vmax), &E);                  // max |x| < 2^E
      const int q = 30 - E;
      uint32_t H[kPairs], Lo[kPairs];
      bool exact = true;
#pragma unroll
      for (int k = 0; k < kPairs; ++k) {
        const float y0 = ldexpf(widen16<DT>(xr[k] & 0xFFFFu), q);
        const float y1 = ldexpf(widen16<DT>(xr[k] >> 16), q);
        const int i0 = (int)y0, i1 = (int)y1;
        exact = exact && ((float)i0 == y0) && ((float)i1 == y1);
        Lo[k] = __builtin_amdgcn_perm((uint32_t)i1, (uint32_t)i0, 0x05040100u);
        H[k] = __builtin_amdgcn_perm((uint32_t)(i1 + 0x8000), (uint32_t)(i0 + 0x8000), 0x07060302u);
      }

      float r_sel = optimise_range(kp, r_start, [&](float inv, double& A, double& B) {
        eval_regs<DT>(xr, H, Lo, inv, clo, chi, q, A, B);
      });
      if (!exact) {
        r_sel = optimise_range(kp, r_start, [&](float inv, double& A, double& B) {
          eval_slot<DT>(slot, inv, clo, chi, A, B);
        });
      }

      // ---- emit (Algorithm 1, third step) ----
      const float s32 = r_sel / kp.D;
      const float inv = 1.0f / s32;
      __syncthreads();              // every lane has finished reading slots that are not its own
      if (valid) {
        if (kp.bits == 4) {
          uint32_t* dst = reinterpret_cast<uint32_t*>(slot + kCodeOff);
#pragma unroll
          for (int wd = 0; wd < 16; wd += 4) {
            uint32_t o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              uint32_t word = 0;
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                uint32_t f0, f1;
                pair_levels<DT>(xr[(wd + j) * 4 + k], inv, clo, chi, f0, f1);
                word |= ((f0 + (uint32_t)z) & 0xFu) << (8 * k);
                word |= ((f1 + (uint32_t)z) & 0xFu) << (8 * k + 4);
              }
              o[j] = word;
            }
            *reinterpret_cast<uint4*>(dst + wd) = make_uint4(o[0], o[1], o[2], o[3]);
          }
        } else {
          // unsigned codes as bytes in the lower half of the slot, then a bit-stream pack
          uint32_t* bytes = reinterpret_cast<uint32_t*>(slot);
#pragma unroll
          for (int k = 0; k < kPairs; k += 2) {
            uint32_t f0, f1, f2, f3;
            pair_levels<DT>(xr[k], inv, clo, chi, f0, f1);
            pair_levels<DT>(xr[k + 1], inv, clo, chi, f2, f3);
            bytes[k >> 1] = ((f0 + (uint32_t)z) & 0xFFu) | (((f1 + (uint32_t)z) & 0xFFu) << 8) |
                            (((f2 + (uint32_t)z) & 0xFFu) << 16) | (((f3 + (uint32_t)z) & 0xFFu) << 24);
          }
          const unsigned char* ub = slot;
          uint32_t* dst = reinterpret_cast<uint32_t*>(slot + kCodeOff);
          unsigned long long acc = 0;
          int nb = 0, wi = 0;
          for (int e = 0; e < kG; ++e) {
            acc |= (unsigned long long)ub[e] << nb;
            nb += kp.bits;
            if (nb >= 32) {
              dst[wi++] = (uint32_t)acc;
              acc >>= 32;
              nb -= 32;
            }
          }
        }
        const int64_t gu = unit_base + slot_i;
        md.scales[gu] = s32;
        md.zps[gu] = (unsigned char)z;
      }
      __syncthreads();
      // ---- the wavefront's 64 units' codes are contiguous in HBM: coalesced 128-bit stores ----
      {
        const uint32_t w_first = base + wave * kWave;
        const uint32_t nvalid = w_first < take ? min((uint32_t)kWave, take - w_first) : 0u;
        const uint32_t nchunk = nvalid * (uint32_t)kp.bits;   // 16-byte chunks
        uint4* gdst = reinterpret_cast<uint4*>(md.codes + (unit_base + w_first) * (int64_t)code_words);
        for (uint32_t j = lane; j < nchunk; j += kWave) {
          const uint32_t un = j / (uint32_t)kp.bits, part = j - un * (uint32_t)kp.bits;
          gdst[j] = *reinterpret_cast<const uint4*>(pool + (size_t)(w_first + un) * kSlotBytes + kCodeOff + part * 16u);
        }
      }
    }
    __syncthreads();
    // ---- carry the units that did not fill a round to the front of the pool ----
    const uint32_t left = pool_units - take;
    if (left) {
      const uint32_t nch = left * kSlotChunks, shift = take * kSlotChunks;
      for (uint32_t c0 = 0; c0 < nch; c0 += kThreads) {
        const uint32_t ch = c0 + threadIdx.x;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (ch < nch) v = *reinterpret_cast<const uint4*>(pool + (size_t)(ch + shift) * 16u);
        __syncthreads();
        if (ch < nch) *reinterpret_cast<uint4*>(pool + (size_t)ch * 16u) = v;
      }
      __syncthreads();
    }
    pool_units = left;
    unit_base += take;
  }
}

}  // namespace eq
