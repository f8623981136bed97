// Shared device-side definitions of the EasyQuant HIP path (gfx950 only).
//
// Arithmetic contract of the whole path (what makes results reproducible bit for bit):
//   * element work in binary32, one rounding per operation (compiled with
//     -ffp-contract=off: no fused multiply-add is formed from separate operations);
//   * the two sums of the gradient (Eq. 2), A = sum c^2 and B = sum x c, are exact;
//   * the scalar recurrence (loss, gradient, Adam on the range; Sec. 4.2) in binary64,
//     the range rounded to binary32 after every step.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "easyquant.h"

namespace eq {

constexpr int kThreads = 256;            // workgroup size of every kernel here
constexpr int kWave = 64;                // CDNA wavefront
constexpr int kWaves = kThreads / kWave;

// One matrix of a batch: inputs, outputs and its slice of the workspace.
struct MatDesc {
  const uint16_t* W;
  uint32_t* codes;
  float* scales;
  uint8_t* zps;
  uint32_t* out_row_ptr;
  uint32_t* out_col;
  uint16_t* out_val;
  int32_t* status;
  // workspace
  unsigned long long* cursor;   // next free staging entry
  uint32_t* row_count;          // outliers per row
  uint32_t* row_stage;          // first staging entry of the row
  uint32_t* st_col;             // staging (arrival order, one contiguous run per row)
  uint16_t* st_val;
  double* mat_stats;            // [0] mean, [1] sigma of the whole matrix (EQ_STAT_MATRIX)
  double* mat_partial;          // per-workgroup partial sums of the pre-pass
  int64_t ld;
  int64_t capacity;
  int32_t rows, cols;
  int32_t upr;                  // units per row
  int32_t G;                    // elements per unit
  int32_t words_per_row;
  int32_t path;                 // 0: general kernel, 1: unit-per-lane kernel
};

// Hyper-parameters in the form the kernels use them.
struct KParams {
  int32_t dtype, bits, mode, scope, select, iters;
  int32_t L;        // 2^bits - 1
  int32_t zsym;     // 2^(bits-1) - 1
  float D;          // level the range maps to: zsym (symmetric) or L (asymmetric)
  float pad_;
  double n;         // threshold of Eq. 3
  double lr, b1, b2, eps;
};

// 128-bit streaming load: the data is used once, so it is marked non-temporal.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream128(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// ---- 16-bit formats -------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ float widen16(uint32_t h) {
  if (DT == EQ_F16) return __half2float(__ushort_as_half((unsigned short)h));
  return __uint_as_float(h << 16);
}
template <int DT>
__device__ __forceinline__ bool nonfinite16(uint32_t h) {
  return DT == EQ_F16 ? ((h & 0x7C00u) == 0x7C00u) : ((h & 0x7F80u) == 0x7F80u);
}
template <int DT>
__device__ __forceinline__ uint32_t narrow16(float x) {   // round to nearest even
  if (DT == EQ_F16) return (uint32_t)__half_as_ushort(__float2half_rn(x));
  uint32_t b = __float_as_uint(x);
  return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// ---- reductions: every lane ends with the same bits -------------------------------------
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o));
  return v;
}
// Block-wide sums through a small LDS scratch (kWaves entries); ends with a barrier.
__device__ __forceinline__ double block_sum(double v, double* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = v;
  __syncthreads();
  double t = red[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) t += red[w];
  return t;
}
__device__ __forceinline__ uint32_t block_sum_u32(uint32_t v, uint32_t* red) {
  v = (uint32_t)wave_sum((int)v);
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = v;
  __syncthreads();
  uint32_t t = red[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) t += red[w];
  return t;
}

// ---- the scalar recurrence --------------------------------------------------------------
// Loss (minus the constant sum x^2) and its derivative with respect to the range at scale
// s = r / D, from the exact sums A and B:  loss = s^2 A - 2 s B + sum x^2;
// d loss / d s = 2 (s A - B) is Eq. 2 with Q[x_i] = s c_i; d s / d r = 1 / D.
__device__ __forceinline__ void loss_and_grad(float s32, double A, double B, float D, double& J, double& g) {
  const double s = (double)s32;
  const double e = s * A - B;
  J = s * (e - B);
  g = (2.0 * e) / (double)D;
}

// Adam (bias-corrected) on the range of one unit; moments in binary64.
struct Adam {
  double m, v, p1, p2;
  __device__ __forceinline__ void init() { m = 0.0; v = 0.0; p1 = 1.0; p2 = 1.0; }
  __device__ __forceinline__ float step(const KParams& kp, float r32, double g, double floor_r) {
    m = kp.b1 * m + (1.0 - kp.b1) * g;
    v = kp.b2 * v + (1.0 - kp.b2) * (g * g);
    p1 = p1 * kp.b1;
    p2 = p2 * kp.b2;
    const double mh = m / (1.0 - p1);
    const double vh = v / (1.0 - p2);
    const double r64 = (double)r32 - kp.lr * (mh / (sqrt(vh) + kp.eps));
    return (float)fmax(r64, floor_r);
  }
};

// Initial range and zero-point of a unit from the min / max of its normal values (outliers
// already replaced by 0).  Returns false for a unit that is not optimised (all zero).
__device__ __forceinline__ bool init_unit(const KParams& kp, float vmin, float vmax, float& r0, int& z) {
  if (kp.mode == EQ_SYMMETRIC) {
    r0 = fmaxf(-vmin, vmax);          // max |x|
    z = kp.zsym;
  } else {
    const float lo = fminf(vmin, 0.0f), hi = fmaxf(vmax, 0.0f);
    r0 = hi - lo;
    z = 0;
    if (r0 > 0.0f) {
      const float s0 = r0 / kp.D;
      const float zf = rintf((-lo) / s0);
      z = (int)fminf(fmaxf(zf, 0.0f), (float)kp.L);
    }
  }
  return r0 > 0.0f;
}

}  // namespace eq
