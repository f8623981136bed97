// Fast path for group_size 128: one LANE owns one unit.
//
// A workgroup walks a range of rows.  Rows are staged into an LDS pool (eq_rowbatch.h: one
// coalesced HBM read, statistics, outlier compaction); whenever the pool holds a round of
// units (one per lane) every lane takes one and runs ALL range-optimisation iterations on it (Sec. 4.2 /
// Algorithm 1, second step) without touching HBM: the unit's fixed-point planes live in
// registers, its 16-bit values are re-read from the lane's own LDS slot in each iteration
// (conflict-free 128-bit reads, ~3 % of the instruction stream), there is no cross-lane
// reduction, and the scalar Adam step is paid once per 128 elements.  Units left over
// (less than a round) are carried to the next fill, so lanes idle only at the end of a range.
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

#include <type_traits>

#include "eq_common.h"
#include "eq_rowbatch.h"
#include "eq_rowstage.h"

namespace eq {

constexpr int kG = 128;               // elements per unit
constexpr int kPairs = kG / 2;
constexpr int kSlotBytes = 272;       // 256 B of data + 16 B of padding (bank spread)
constexpr int kSlotChunks = 17;
constexpr int kCodeOff = 128;         // packed codes are assembled in the upper half of the slot
constexpr int kLdsHeader = 6144;      // scratch of the row staging, in front of the pool

// What one workgroup does: rows [row0, row0 + nrows) of matrix `mat`, either all of them
// (stride == 0) or, in steps of `stride` rows, only the first batch of rows of every step
// (the kernel without optimisation steps: neighbouring workgroups then read neighbouring rows at
// about the same time, and the whole chip moves through a matrix as one front).
struct WorkItem {
  int32_t mat, row0, nrows, stride;
};

typedef short short2_t __attribute__((ext_vector_type(2)));

// Levels of the 8 elements of one 16-byte chunk as four packed int16 pairs: the low 16 bits of the
// bit pattern of kMagic + level (see level_of) are the signed level in two's complement; mlo / mhi
// are the level bounds plus kMagic; for fp16 the widening folds into the multiply-add
// (v_fma_mix_f32).  Written stage by
// stage (8 multiply-adds, 8 clamps, 4 packs) so that neighbouring instructions are independent:
// a dependent instruction cannot issue back to back, and only two wavefronts share a SIMD.
template <int DT>
__device__ __forceinline__ void chunk_levels(const uint4 v, float inv, float mlo, float mhi, short2_t (&c)[4]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  float t[8];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float x0, x1;
    if (DT == EQ_F16) {
      x0 = __half2float(__ushort_as_half((unsigned short)(w[j] & 0xFFFFu)));
      x1 = __half2float(__ushort_as_half((unsigned short)(w[j] >> 16)));
    } else {
      x0 = __uint_as_float(w[j] << 16);
      x1 = __uint_as_float(w[j] & 0xFFFF0000u);
    }
    t[2 * j] = __builtin_fmaf(x0, inv, kMagic);
    t[2 * j + 1] = __builtin_fmaf(x1, inv, kMagic);
  }
  __builtin_amdgcn_sched_barrier(0);       // keep the stages apart: the scheduler would re-serialise them
#pragma unroll
  for (int j = 0; j < 8; ++j) t[j] = __builtin_amdgcn_fmed3f(t[j], mlo, mhi);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < 4; ++j)
    c[j] = __builtin_bit_cast(short2_t, __builtin_amdgcn_perm(__float_as_uint(t[2 * j + 1]), __float_as_uint(t[2 * j]), 0x05040100u));
  __builtin_amdgcn_sched_barrier(0);
}

// Block fixed-point planes of the lane's unit: xi = x * 2^q (|xi| < 2^30) as 65536 H + L with
// signed 16-bit halves, two elements per register.  TEST also ORs the bit patterns of
// y - trunc(y) into frac_bits (zero iff every x * 2^q is an integer).
template <int DT, bool TEST>
__device__ __forceinline__ void build_planes(const unsigned char* slot, int q, uint32_t (&H)[kPairs], uint32_t (&Lo)[kPairs],
                                             uint32_t& frac_bits) {
#pragma unroll
  for (int ch = 0; ch < 16; ++ch) {
    const uint4 v = *reinterpret_cast<const uint4*>(slot + ch * 16);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = 4 * ch + j;
      const float y0 = ldexpf(widen16<DT>(w[j] & 0xFFFFu), q);
      const float y1 = ldexpf(widen16<DT>(w[j] >> 16), q);
      const int i0 = (int)y0, i1 = (int)y1;
      if (TEST) frac_bits |= __float_as_uint(y0 - (float)i0) | __float_as_uint(y1 - (float)i1);
      Lo[k] = __builtin_amdgcn_perm((uint32_t)i1, (uint32_t)i0, 0x05040100u);
      H[k] = __builtin_amdgcn_perm((uint32_t)(i1 + 0x8000), (uint32_t)(i0 + 0x8000), 0x07060302u);
    }
    // pin the running flag here: otherwise the OR tree is rebalanced, every y and trunc(y) stays
    // live to the end of the unit, and 256 values are spilled to scratch memory
    if (TEST) asm volatile("" : "+v"(frac_bits));
    else __builtin_amdgcn_sched_barrier(0);
  }
}

// One evaluation of Eq. 1 / Eq. 2 for the lane's unit: values from its LDS slot (read one
// chunk ahead of use), planes from registers.  The compiler barrier keeps the reads inside
// the iteration loop (hoisted, they would pin 64 more registers).
template <int DT>
__device__ __forceinline__ void eval_sums(const unsigned char* slot, const uint32_t (&H)[kPairs],
                                          const uint32_t (&Lo)[kPairs], float inv, float mlo, float mhi,
                                          int& sum_cc, int& sum_hc, int& sum_lc) {
  asm volatile("" ::: "memory");
  // one accumulator per sum, the three sums taking turns: a dependent dot product is then three
  // instructions away, and there is nothing to clear or to add up beyond the three registers
  int a = 0, bh = 0, bl = 0;
  uint4 nxt = *reinterpret_cast<const uint4*>(slot);
#pragma unroll
  for (int ch = 0; ch < 16; ++ch) {
    const uint4 cur = nxt;
    if (ch + 1 < 16) nxt = *reinterpret_cast<const uint4*>(slot + (ch + 1) * 16);
    short2_t c[4];
    chunk_levels<DT>(cur, inv, mlo, mhi, c);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      a = __builtin_amdgcn_sdot2(c[j], c[j], a, false);
      bh = __builtin_amdgcn_sdot2(__builtin_bit_cast(short2_t, H[4 * ch + j]), c[j], bh, false);
      bl = __builtin_amdgcn_sdot2(__builtin_bit_cast(short2_t, Lo[4 * ch + j]), c[j], bl, false);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  sum_cc = a;
  sum_hc = bh;
  sum_lc = bl;
}
template <int DT>
__device__ __forceinline__ void eval_regs(const unsigned char* slot, const uint32_t (&H)[kPairs],
                                          const uint32_t (&Lo)[kPairs], float inv, float mlo, float mhi, int q,
                                          double& A, double& B) {
  int cc, hc, lc;
  eval_sums<DT>(slot, H, Lo, inv, mlo, mhi, cc, hc, lc);
  A = (double)cc;
  B = ldexp((double)hc * 65536.0 + (double)lc, -q);  // exact: |.| < 2^47
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
      const float c = level_of(xv, inv, clo, chi);
      const int ci = (int)c;
      a += ci * ci;
      b += (double)(xv * c);
    }
  }
  A = (double)a;
  B = b;
}

// Smallest and largest value of the unit in `slot`, 0 included.
template <int DT>
__device__ __forceinline__ void slot_min_max(const unsigned char* slot, float& vmin, float& vmax) {
  vmin = 0.0f;
  vmax = 0.0f;
  if (DT == EQ_F16) {
    // packed fp16 min / max over the pairs (exact: they only select), widened once at the end
    uint32_t mnb = 0u, mxb = 0u;
#pragma unroll
    for (int ch = 0; ch < 16; ++ch) {
      const uint4 v = *reinterpret_cast<const uint4*>(slot + ch * 16);
      mnb = pk_min3_f16(pk_min3_f16(mnb, v.x, v.y), v.z, v.w);
      mxb = pk_max3_f16(pk_max3_f16(mxb, v.x, v.y), v.z, v.w);
    }
    typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
    const half2_t mn = __builtin_bit_cast(half2_t, mnb), mx = __builtin_bit_cast(half2_t, mxb);
    vmin = fminf((float)mn.x, (float)mn.y);
    vmax = fmaxf((float)mx.x, (float)mx.y);
  } else {
#pragma unroll
    for (int ch = 0; ch < 16; ++ch) {
      const uint4 v = *reinterpret_cast<const uint4*>(slot + ch * 16);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float x0 = widen16<DT>(w[j] & 0xFFFFu), x1 = widen16<DT>(w[j] >> 16);
        vmin = fminf(vmin, fminf(x0, x1));
        vmax = fmaxf(vmax, fmaxf(x0, x1));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// Code widths other than 4: the unit's 128 codes as a bit stream (code e at bits [BITS e,
// BITS e + BITS), least significant first) of 4 BITS words, built in registers with constant
// shifts and written over the upper part of the slot once every value has been read.  A chunk
// of 8 values yields BITS whole bytes.  The zero-point rides in the rounding constant as in the
// 4-bit form (an odd one as z + 1 so that exact ties still go to the even level; the 1 comes
// off the gathered bytes, or off each pattern for 8 bits, where code + 1 can reach 256).
template <int DT, int BITS, bool NOCLAMP>
__device__ __forceinline__ void emit_codes_bits(const KParams& kp, unsigned char* slot, float inv, int z) {
  const int zodd = z & 1;
  const uint32_t unfold = zodd ? 0x01010101u : 0u;
  const float mz = kMagic + (float)(z + zodd), ulo = kMagic + (float)zodd, uhi = kMagic + (float)(kp.L + zodd);
  constexpr int NWORDS = 4 * BITS;
  constexpr uint32_t kPairMask = (((1u << BITS) - 1u) << BITS) * 0x00010001u;
  uint32_t o[NWORDS];
#pragma unroll
  for (int i = 0; i < NWORDS; ++i) o[i] = 0u;
#pragma unroll
  for (int ch = 0; ch < 16; ++ch) {
    const uint4 v = *reinterpret_cast<const uint4*>(slot + ch * 16);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t f[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float x0, x1;
      if (DT == EQ_F16) {
        x0 = __half2float(__ushort_as_half((unsigned short)(w[j] & 0xFFFFu)));
        x1 = __half2float(__ushort_as_half((unsigned short)(w[j] >> 16)));
      } else {
        x0 = __uint_as_float(w[j] << 16);
        x1 = __uint_as_float(w[j] & 0xFFFF0000u);
      }
      f[2 * j] = __float_as_uint(NOCLAMP ? __builtin_fmaf(x0, inv, mz) : __builtin_amdgcn_fmed3f(__builtin_fmaf(x0, inv, mz), ulo, uhi));
      f[2 * j + 1] = __float_as_uint(NOCLAMP ? __builtin_fmaf(x1, inv, mz) : __builtin_amdgcn_fmed3f(__builtin_fmaf(x1, inv, mz), ulo, uhi));
      if (BITS == 8) {
        f[2 * j] -= (uint32_t)zodd;
        f[2 * j + 1] -= (uint32_t)zodd;
      }
    }
    // the low bytes of four patterns, in element order
    uint32_t b[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      b[h] = __builtin_amdgcn_perm(f[4 * h + 1], f[4 * h], 0x0C0C0400u) | __builtin_amdgcn_perm(f[4 * h + 3], f[4 * h + 2], 0x04000C0Cu);
      if (BITS != 8) b[h] -= unfold;
      // four bytes -> two fields of 2 BITS bits -> one of 4 BITS bits
      const uint32_t pr = (b[h] & 0x00FF00FFu) | ((b[h] >> (8 - BITS)) & kPairMask);
      b[h] = (pr & 0xFFFFu) | ((pr >> 16) << (2 * BITS));
    }
    const unsigned long long r = (unsigned long long)b[0] | ((unsigned long long)b[1] << (4 * BITS));
    const uint32_t lo = (uint32_t)r, hi = (uint32_t)(r >> 32);
    constexpr int kChunkBits = 8 * BITS;
    const int off = ch * kChunkBits, wd = off >> 5, sh = off & 31;
    o[wd] |= lo << sh;
    if (sh) {
      if (wd + 1 < NWORDS) o[wd + 1] |= (lo >> (32 - sh)) | (hi << sh);
      if (kChunkBits + sh > 64 && wd + 2 < NWORDS) o[wd + 2] |= hi >> (32 - sh);
    } else if (kChunkBits > 32) {
      if (wd + 1 < NWORDS) o[wd + 1] |= hi;
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  uint4* dst = reinterpret_cast<uint4*>(slot + kCodeOff);
#pragma unroll
  for (int wd = 0; wd < BITS; ++wd) dst[wd] = make_uint4(o[4 * wd], o[4 * wd + 1], o[4 * wd + 2], o[4 * wd + 3]);
}

// Packed codes of the unit in `slot` at reciprocal scale `inv` (Eq. 1), assembled in the upper
// half of the slot (the values in the lower half stay intact for 4-bit codes only).
// NOCLAMP: the caller knows that no level can leave [l_min, l_max] (symmetric mode at the initial
// range: |x| <= r0 gives |x / s| <= D (1 + 2^-22)), so the clamp of Eq. 1 is left out.
template <int DT, bool NOCLAMP = false>
__device__ __forceinline__ void emit_codes_to_slot(const KParams& kp, unsigned char* slot, float inv, int z) {
  if (kp.bits == 4) {
    // all 16 words first (they overwrite the upper half of the values), then one store burst
    // The zero-point goes into the magic constant, so the low byte of each pattern is the
    // unsigned code itself; even and odd elements are gathered into bytes and merged.
    // Ties go to the even value of the whole sum, so the constant added must stay even for
    // them to go to the even level: an odd zero-point is folded in as z + 1, and the 1 is
    // taken off the gathered bytes (every byte is then >= 1: no borrow between bytes).
    const int zodd = z & 1;
    const uint32_t unfold = zodd ? 0x01010101u : 0u;
    const float mz = kMagic + (float)(z + zodd), ulo = kMagic + (float)zodd, uhi = kMagic + (float)(kp.L + zodd);
    uint32_t o[16];
#pragma unroll
    for (int ch = 0; ch < 16; ++ch) {
      const uint4 v = *reinterpret_cast<const uint4*>(slot + ch * 16);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
      uint32_t f[8];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float x0, x1;
        if (DT == EQ_F16) {
          x0 = __half2float(__ushort_as_half((unsigned short)(w[j] & 0xFFFFu)));
          x1 = __half2float(__ushort_as_half((unsigned short)(w[j] >> 16)));
        } else {
          x0 = __uint_as_float(w[j] << 16);
          x1 = __uint_as_float(w[j] & 0xFFFF0000u);
        }
        f[2 * j] = __float_as_uint(NOCLAMP ? __builtin_fmaf(x0, inv, mz) : __builtin_amdgcn_fmed3f(__builtin_fmaf(x0, inv, mz), ulo, uhi));
        f[2 * j + 1] = __float_as_uint(NOCLAMP ? __builtin_fmaf(x1, inv, mz) : __builtin_amdgcn_fmed3f(__builtin_fmaf(x1, inv, mz), ulo, uhi));
      }
      const uint32_t even = __builtin_amdgcn_perm(f[2], f[0], 0x0C0C0400u) | __builtin_amdgcn_perm(f[6], f[4], 0x04000C0Cu);
      const uint32_t odd = __builtin_amdgcn_perm(f[3], f[1], 0x0C0C0400u) | __builtin_amdgcn_perm(f[7], f[5], 0x04000C0Cu);
      o[ch] = ((odd - unfold) << 4) | (even - unfold);
      __builtin_amdgcn_sched_barrier(0);
    }
    uint4* dst = reinterpret_cast<uint4*>(slot + kCodeOff);
#pragma unroll
    for (int wd = 0; wd < 4; ++wd) dst[wd] = make_uint4(o[4 * wd], o[4 * wd + 1], o[4 * wd + 2], o[4 * wd + 3]);
  } else {
    switch (kp.bits) {
      case 2: emit_codes_bits<DT, 2, NOCLAMP>(kp, slot, inv, z); break;
      case 3: emit_codes_bits<DT, 3, NOCLAMP>(kp, slot, inv, z); break;
      case 5: emit_codes_bits<DT, 5, NOCLAMP>(kp, slot, inv, z); break;
      case 6: emit_codes_bits<DT, 6, NOCLAMP>(kp, slot, inv, z); break;
      case 7: emit_codes_bits<DT, 7, NOCLAMP>(kp, slot, inv, z); break;
      default: emit_codes_bits<DT, 8, NOCLAMP>(kp, slot, inv, z); break;
    }
  }
}

// The codes of the wavefront's 64 units (slots w_first ..) are contiguous in HBM: coalesced
// 128-bit stores.  `take` = number of valid slots in the pool, unit_base = matrix-wide index of
// the unit in slot 0.
__device__ __forceinline__ void copy_wave_codes(const KParams& kp, const MatDesc& md, const unsigned char* pool,
                                                int64_t unit_base, uint32_t w_first, uint32_t take, uint32_t lane) {
  const uint32_t code_words = 4u * (uint32_t)kp.bits;
  const uint32_t nvalid = w_first < take ? min((uint32_t)kWave, take - w_first) : 0u;
  const uint32_t nchunk = nvalid * (uint32_t)kp.bits;   // 16-byte chunks
  EQ_GLOBAL uint32_t* gdst = md.codes + (unit_base + w_first) * (int64_t)code_words;
  for (uint32_t j = lane; j < nchunk; j += kWave) {
    const uint32_t un = j / (uint32_t)kp.bits, part = j - un * (uint32_t)kp.bits;
    global_store_stream128(gdst + 4 * (size_t)j, *reinterpret_cast<const uint4*>(pool + (size_t)(w_first + un) * kSlotBytes + kCodeOff + part * 16u));
  }
}

// A bf16 unit as fp16: x' = x * 2^k is exactly representable in fp16 for every x of the unit
// unless the unit spans more than ~2^38 in magnitude (k puts the largest magnitude just below
// 2^15; fp16 then reaches down to multiples of 2^-24).  Levels and sums are unchanged when the
// reciprocal scale is multiplied by 2^-k (both exact), and the fp16 forms of the inner loop are
// a quarter cheaper: the widening folds into the multiply-add, which bf16 has no instruction for.
__device__ __forceinline__ bool slot_fits_f16(const unsigned char* slot, int k) {
  uint32_t bad = 0;
#pragma unroll
  for (int ch = 0; ch < 16; ++ch) {
    const uint4 v = *reinterpret_cast<const uint4*>(slot + ch * 16);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float y0 = ldexpf(widen16<EQ_BF16>(w[j] & 0xFFFFu), k), y1 = ldexpf(widen16<EQ_BF16>(w[j] >> 16), k);
      bad |= (__half2float(__float2half_rn(y0)) != y0 ? 1u : 0u) | (__half2float(__float2half_rn(y1)) != y1 ? 1u : 0u);
    }
    asm volatile("" : "+v"(bad));       // keep the running flag: no long-lived temporaries
  }
  return bad == 0;
}
__device__ __forceinline__ void slot_bf16_to_f16(unsigned char* slot, int k) {
#pragma unroll
  for (int ch = 0; ch < 16; ++ch) {
    const uint4 v = *reinterpret_cast<const uint4*>(slot + ch * 16);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float y0 = ldexpf(widen16<EQ_BF16>(w[j] & 0xFFFFu), k), y1 = ldexpf(widen16<EQ_BF16>(w[j] >> 16), k);
      o[j] = (uint32_t)__half_as_ushort(__float2half_rn(y0)) | ((uint32_t)__half_as_ushort(__float2half_rn(y1)) << 16);
    }
    *reinterpret_cast<uint4*>(slot + ch * 16) = make_uint4(o[0], o[1], o[2], o[3]);
  }
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
    double bc[4];
    load_bias_corrections(kp, t, bc);      // issued before the evaluation, consumed after it
    float s32, inv;
    scale_of(kp, r32, s32, inv);
    double A, B, J, g;
    ev(inv, A, B);
    loss_and_grad(kp, s32, A, B, J, g);
    if (J < J_best) {
      J_best = J;
      r_sel = r32;
    }
    r32 = ad.step(kp, bc, r32, g, floor_r);
  }
  if (kp.select == EQ_SELECT_LAST) return r32;
  if (kp.iters > 0) {
    float s32, inv;
    scale_of(kp, r32, s32, inv);
    double A, B, J, g;
    ev(inv, A, B);
    loss_and_grad(kp, s32, A, B, J, g);
    if (J < J_best) r_sel = r32;
  }
  return r_sel;
}

// NT = threads per workgroup = units per round: 256 when two workgroups' pools fit the LDS of
// a compute unit, 512 (one workgroup per compute unit) for long rows; two wavefronts per SIMD
// either way.  K = 16-byte chunks of a row per thread (cols <= 8 * K * NT); rows are staged in
// batches of RB rows, 16 / K unless stated (16 chunks = 64 registers of row data per thread; a
// batch of 3 rows of 8 chunks, 96 registers, lets rows of which three fill a round of 512 be
// staged in one go: the planes are not live while rows are staged).
template <int DT, int NT, int K, int RB = 16 / K>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void quantize_units128(const MatDesc* __restrict__ mats,
                                                              const WorkItem* __restrict__ items, KParams kp,
                                                              uint32_t pool_slots) {
  typedef BatchScratch<RB, NT / kWave> Scratch;
  static_assert(sizeof(Scratch) <= kLdsHeader, "staging scratch must fit the LDS header");
  extern __shared__ __align__(16) unsigned char smem[];
  Scratch* sc = reinterpret_cast<Scratch*>(smem);
  unsigned char* pool = smem + kLdsHeader;
  const WorkItem it = items[blockIdx.x];
  const MatDesc md = mats[it.mat];
  const uint32_t upr = (uint32_t)md.upr;
  const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  int64_t next_row = it.row0;
  const int64_t row_end = (int64_t)it.row0 + it.nrows;
  int64_t unit_base = (int64_t)it.row0 * upr;               // matrix-wide index of the unit in slot 0
  uint32_t pool_units = 0;

  while (true) {
    // ---- fill: stage rows until a full round of units is available ----
    while (next_row < row_end && pool_units < (uint32_t)NT && pool_units + upr <= pool_slots) {
      int nb = 0;
      uint32_t pu = pool_units;
      while (nb < RB && next_row + nb < row_end && pu < (uint32_t)NT && pu + upr <= pool_slots) {
        pu += upr;
        ++nb;
      }
      stage_rows_batch<DT, NT, RB, K, Padded128Layout>(md, kp, next_row, nb, pool, pool_units * 16u, nullptr, sc);
      pool_units = pu;
      next_row += nb;
    }
    if (pool_units == 0) break;
    // whole rounds; a partly filled one only at the end of the range or when the pool has no
    // room for another row
    const uint32_t take = pool_units >= (uint32_t)NT ? (pool_units / NT) * NT : pool_units;

    for (uint32_t base = 0; base < take; base += NT) {
      const uint32_t slot_i = base + threadIdx.x;
      const bool valid = slot_i < take;
      unsigned char* slot = pool + (size_t)(valid ? slot_i : base) * kSlotBytes;

      // ---- range of the unit, and its block fixed-point planes ----
      // xi = x * 2^q with |xi| < 2^30, split into signed 16-bit planes xi = 65536 H + L
      float vmin, vmax;
      slot_min_max<DT>(slot, vmin, vmax);
      float r0;
      int z;
      const bool active = init_unit(kp, vmin, vmax, r0, z);
      const float clo = (float)(-z), chi = (float)(kp.L - z);
      const float mlo = clo + kMagic, mhi = chi + kMagic;     // exact: small integers next to 1.5 * 2^23
      const float r_start = active ? r0 : kp.D;              // an all-zero unit keeps s = 1
      int E = 0;
      (void)frexpf(fmaxf(-vmin, vmax), &E);                  // max |x| < 2^E
      const int q = 30 - E;
      // What follows works on the slot either in the input type or, for bf16, in the fp16 form
      // described at slot_fits_f16 (DX, with k = shift): planes, optimisation, emission.
      auto optimise = [&](auto dx, const int shift) -> float {
        constexpr int DX = decltype(dx)::value;
        const float unshift = ldexpf(1.0f, -shift);          // exact power of two
        uint32_t H[kPairs], Lo[kPairs];
        uint32_t frac_bits = 0;          // OR of the bit patterns of y - trunc(y): zero iff every y is an integer
        // every fp16 value is a multiple of 2^-24, so an exponent >= 24 needs no test (wavefront-uniform branch)
        const bool need_test = !(DX == EQ_F16 && __all(q - shift >= 24));
        if (need_test) build_planes<DX, true>(slot, q - shift, H, Lo, frac_bits);
        else build_planes<DX, false>(slot, q - shift, H, Lo, frac_bits);
        const bool exact = (frac_bits << 1) == 0;

        float r_sel = optimise_range(kp, r_start, [&](float inv, double& A, double& B) {
          eval_regs<DX>(slot, H, Lo, inv * unshift, mlo, mhi, q, A, B);
        });
        if (!exact) {
          r_sel = optimise_range(kp, r_start, [&](float inv, double& A, double& B) {
            eval_slot<DX>(slot, inv * unshift, clo, chi, A, B);
            B = ldexp(B, -shift);
          });
        }
        return r_sel;
      };
      // ---- emit (Algorithm 1, third step) ----
      auto emit = [&](auto dx, const int shift, const float r_sel) {
        constexpr int DX = decltype(dx)::value;
        float s32, inv;
        scale_of(kp, r_sel, s32, inv);
        emit_codes_to_slot<DX>(kp, slot, inv * ldexpf(1.0f, -shift), z);
        const int64_t gu = unit_base + slot_i;
        md.scales[gu] = s32;
        md.zps[gu] = (unsigned char)z;
      };
      // bf16 units are taken in their fp16 form when every unit of the WAVEFRONT has one (the choice
      // may differ between the wavefronts of a workgroup: both branches below are barrier-free, and
      // all wavefronts meet at the one barrier between optimisation and emission).  A lane without a
      // unit works on a copy of the round's first slot and discards the result; it may read that slot
      // while its owner converts or emits it, which only changes what is discarded.
      bool as_f16 = false;
      const int shift = 15 - E;
      if (DT == EQ_BF16) {
        as_f16 = __all(!valid || slot_fits_f16(slot, shift));
        if (as_f16 && valid) slot_bf16_to_f16(slot, shift);
      }
      float r_sel;
      if (DT == EQ_BF16 && as_f16) r_sel = optimise(std::integral_constant<int, EQ_F16>{}, shift);
      else r_sel = optimise(std::integral_constant<int, DT>{}, 0);
      __syncthreads();                // every lane has finished reading slots that are not its own
      if (valid) {
        if (DT == EQ_BF16 && as_f16) emit(std::integral_constant<int, EQ_F16>{}, shift, r_sel);
        else emit(std::integral_constant<int, DT>{}, 0, r_sel);
      }
      __syncthreads();
      copy_wave_codes(kp, md, pool, unit_base, base + wave * kWave, take, lane);
    }
    __syncthreads();
    // ---- carry the units that did not fill a round to the front of the pool ----
    const uint32_t left = pool_units - take;
    if (left) {
      const uint32_t nch = left * kSlotChunks, shift = take * kSlotChunks;
      for (uint32_t c0 = 0; c0 < nch; c0 += NT) {
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
