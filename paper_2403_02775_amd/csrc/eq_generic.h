// General kernel: one workgroup per row, one wavefront per unit at a time.
//
// Handles every supported shape (any unit length, 2..8 bits, both modes, all statistic
// scopes).  The row stays in LDS for the whole optimisation; HBM is read once and written
// once.  The unit-per-lane kernel in eq_fused128.h is the fast path for group_size 128.
#pragma once

#include "eq_common.h"
#include "eq_rowstage.h"

namespace eq {

// Codes and exact sums of one unit at 1/scale = inv (Eq. 1 and the two sums of Eq. 2).
// x: LDS, `nch` chunks of 8 elements.  B is a binary64 accumulation of exact binary32
// products; it is exact (hence order-independent) while sum |x c| < 2^53 ulp(min |x|).
template <int DT>
__device__ __forceinline__ void wave_eval_unit(const unsigned char* x, uint32_t nch, uint32_t lane, float inv, float clo,
                                               float chi, double& A, double& B) {
  int a = 0;
  double b = 0.0;
  for (uint32_t ch = lane; ch < nch; ch += kWave) {
    const uint4 v = *reinterpret_cast<const uint4*>(x + ch * 16u);
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
  A = (double)wave_sum(a);
  B = wave_sum(b);
}

template <int DT>
__global__ __launch_bounds__(kThreads) void quantize_rows_generic(const MatDesc* __restrict__ mats, KParams kp) {
  extern __shared__ __align__(16) unsigned char smem[];
  const MatDesc md = mats[blockIdx.y];
  const int64_t row = blockIdx.x;
  if (row >= md.rows || md.path != 0 || md.cols == 0) return;
  const uint32_t nchunks = (uint32_t)md.cols >> 3;
  StageScratch* sc = reinterpret_cast<StageScratch*>(smem);
  unsigned char* lds_row = smem + 256;
  unsigned char* maskb = lds_row + (size_t)nchunks * 16u;
  const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;

  if (kp.scope == EQ_STAT_GROUP && md.upr > 1) {
    // statistics per unit: each wavefront takes units round-robin
    stage_load_row<DT, LinearLayout>(md, row, lds_row, 0);
    __syncthreads();
    const uint32_t nch_u = (uint32_t)md.G >> 3;
    for (uint32_t u = wave; u < (uint32_t)md.upr; u += kWaves) {
      const unsigned char* x = lds_row + (size_t)u * nch_u * 16u;
      double s = 0.0;
      for (uint32_t ch = lane; ch < nch_u; ch += kWave) {
        const uint4 v = *reinterpret_cast<const uint4*>(x + ch * 16u);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) s += (double)widen16<DT>((w[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
      }
      const double cnt = (double)md.G;
      const double mu = wave_sum(s) / cnt;
      double q = 0.0;
      for (uint32_t ch = lane; ch < nch_u; ch += kWave) {
        const uint4 v = *reinterpret_cast<const uint4*>(x + ch * 16u);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const double d = (double)widen16<DT>((w[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu) - mu;
          q += d * d;
        }
      }
      const double sigma = sqrt(wave_sum(q) / cnt);
      const double thr = kp.n * sigma;
      for (uint32_t ch = lane; ch < nch_u; ch += kWave) {
        const uint4 v = *reinterpret_cast<const uint4*>(x + ch * 16u);
        maskb[u * nch_u + ch] = sigma > 0.0 ? (unsigned char)chunk_mask<DT>(v, mu, thr) : (unsigned char)0;
      }
    }
    stage_compact_row<LinearLayout>(md, row, lds_row, 0, maskb, sc);
  } else {
    stage_row<DT, LinearLayout>(md, kp, row, lds_row, 0, maskb, sc);
  }

  // ---- range optimisation, one wavefront per unit (Algorithm 1, second step) ----
  const uint32_t nch_u = (uint32_t)md.G >> 3;
  for (uint32_t u = wave; u < (uint32_t)md.upr; u += kWaves) {
    const unsigned char* x = lds_row + (size_t)u * nch_u * 16u;
    // min / max start at 0: max |x| is unchanged by it, and the asymmetric range includes 0 anyway
    float vmin = 0.0f, vmax = 0.0f;
    for (uint32_t ch = lane; ch < nch_u; ch += kWave) {
      const uint4 v = *reinterpret_cast<const uint4*>(x + ch * 16u);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float xv = widen16<DT>((w[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
        vmin = fminf(vmin, xv);
        vmax = fmaxf(vmax, xv);
      }
    }
    vmin = wave_min(vmin);
    vmax = wave_max(vmax);
    float r0;
    int z;
    const bool active = init_unit(kp, vmin, vmax, r0, z);
    const float clo = (float)(-z), chi = (float)(kp.L - z);
    float r_sel = kp.D;                  // s = 1 for a unit that is not optimised
    if (active) {
      float r32 = r0;
      r_sel = r0;
      double J_best = __builtin_inf();
      const double floor_r = (double)r0 * 0.0009765625;
      Adam ad;
      ad.init();
      for (int t = 0; t < kp.iters; ++t) {
        double bc[4];
        load_bias_corrections(kp, t, bc);
        float s32, inv;
        scale_of(kp, r32, s32, inv);
        double A, B, J, g;
        wave_eval_unit<DT>(x, nch_u, lane, inv, clo, chi, A, B);
        loss_and_grad(kp, s32, A, B, J, g);
        if (J < J_best) { J_best = J; r_sel = r32; }
        r32 = ad.step(kp, bc, r32, g, floor_r);
      }
      if (kp.select == EQ_SELECT_LAST) {
        r_sel = r32;
      } else if (kp.iters > 0) {
        float s32, inv;
        scale_of(kp, r32, s32, inv);
        double A, B, J, g;
        wave_eval_unit<DT>(x, nch_u, lane, inv, clo, chi, A, B);
        loss_and_grad(kp, s32, A, B, J, g);
        if (J < J_best) r_sel = r32;
      }
    }
    // ---- emit (Algorithm 1, third step): codes at the chosen range, 32 elements per lane ----
    float s32, inv;
    scale_of(kp, r_sel, s32, inv);
    const uint32_t nelem = (uint32_t)md.G;
    const unsigned short* xe = reinterpret_cast<const unsigned short*>(x);
    EQ_GLOBAL uint32_t* wrow = md.codes + row * (int64_t)md.words_per_row + (int64_t)u * ((int64_t)nelem * kp.bits / 32);
    for (uint32_t g32 = lane; g32 * 32u < nelem; g32 += kWave) {
      EQ_GLOBAL uint32_t* wp = wrow + g32 * (uint32_t)kp.bits;
      unsigned long long acc = 0;
      int nb = 0, wi = 0;
      for (uint32_t e = 0; e < 32u && g32 * 32u + e < nelem; ++e) {
        const float xv = widen16<DT>(xe[g32 * 32u + e]);
        const int c = (int)level_of(xv, inv, clo, chi);
        acc |= (unsigned long long)(uint32_t)(c + z) << nb;
        nb += kp.bits;
        if (nb >= 32) {
          wp[wi++] = (uint32_t)acc;
          acc >>= 32;
          nb -= 32;
        }
      }
      if (nb > 0) wp[wi] = (uint32_t)acc;
    }
    if (lane == 0) {
      md.scales[row * (int64_t)md.upr + u] = s32;
      md.zps[row * (int64_t)md.upr + u] = (unsigned char)z;
    }
  }
}

}  // namespace eq
