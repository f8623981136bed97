// Shared device-side definitions of the EasyQuant HIP path (gfx950 only).
//
// Arithmetic contract of the whole path (what makes results reproducible bit for bit):
//   * scale s = r / D and 1 / s in binary32; the level of an element is the exact product
//     x * (1 / s) rounded once to the nearest integer, ties to even (Eq. 1), then clamped
//     (compiled with -ffp-contract=off: no fused multiply-add is formed from separate
//     operations; the fused multiply-adds below are written out on purpose);
//   * the two sums of the gradient (Eq. 2), A = sum c^2 and B = sum x c, are exact;
//   * the scalar recurrence (loss, gradient, Adam on the range; Sec. 4.2) in binary64,
//     the range rounded to binary32 after every step.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "easyquant.h"

namespace eq {

constexpr int kThreads = 256;            // default workgroup size
constexpr int kWave = 64;                // CDNA wavefront
constexpr int kWaves = kThreads / kWave;
constexpr int kMaxWaves = 8;             // largest workgroup any kernel here uses: 512 threads

// Pointers into device memory carry the global address space: a pointer read back from a
// descriptor is otherwise a generic one, every access through it a FLAT instruction, and a
// workgroup barrier then has to wait for all of them (stores included), because a generic
// access might have been to LDS.
#define EQ_GLOBAL __attribute__((address_space(1)))

// One matrix of a batch: inputs, outputs and its slice of the workspace.
struct MatDesc {
  const EQ_GLOBAL uint16_t* W;
  EQ_GLOBAL uint32_t* codes;
  EQ_GLOBAL float* scales;
  EQ_GLOBAL uint8_t* zps;
  EQ_GLOBAL uint32_t* out_row_ptr;
  EQ_GLOBAL uint32_t* out_col;
  EQ_GLOBAL uint16_t* out_val;
  EQ_GLOBAL int32_t* status;
  // workspace
  EQ_GLOBAL unsigned long long* cursor;   // next free staging entry
  EQ_GLOBAL uint32_t* row_count;          // outliers per row
  EQ_GLOBAL uint32_t* row_stage;          // first staging entry of the row
  EQ_GLOBAL uint32_t* st_col;             // staging (arrival order, one contiguous run per row)
  EQ_GLOBAL uint16_t* st_val;
  EQ_GLOBAL double* mat_stats;            // [0] mean, [1] sigma of the whole matrix (EQ_STAT_MATRIX)
  EQ_GLOBAL double* mat_partial;          // per-workgroup partial sums of the pre-pass
  EQ_GLOBAL float* range;                 // per row: the range chosen by the sorted evaluation (eq_sorted.h), else null
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
  int32_t range_given;   // the kernel without optimisation steps emits at MatDesc::range[row] instead of the initial range
  double n;         // threshold of Eq. 3
  double lr, b1, b2, eps;
  double rD64;      // RN(1 / D) in binary64
  float rD32;       // RN(1 / D) in binary32
  float pad2_;
  const EQ_GLOBAL double* adam_tab;   // device: per step t (0-based) {1 - b1^(t+1), RN(1 / that), 1 - b2^(t+1), RN(1 / that)}
};

// ---- the sorted evaluation of rows with one range each (eq_sorted.h) ----
// A run of rows of one matrix whose records lie one after the other in the workspace of a launch.
struct SortSeg {
  int32_t mat, row0, nrows;
  int32_t first_group;      // index of the run's first group of 4 rows among the launch's groups
  int64_t first_row;        // index of its first row among the launch's rows
  int64_t ws_off;           // byte offset of its first record
};
// A row's record: a header (SortRecHeader, then the sum of all values at byte 16), then one 32-byte unit
// per chunk of 8 values in ascending order (outliers as 0): the 8 16-bit values, the exact binary64 sum
// of all values in front of them, 8 unused bytes.  A probe of a chunk therefore reads one cache line.
struct SortRecHeader {
  float r0;                 // initial range
  int32_t z;                // zero-point
  uint32_t flags;           // kRecExactSums | kRecSorted
  uint32_t pad;
};
constexpr size_t kSortRecHeader = 64;
constexpr size_t kSortUnit = 32;
__host__ __device__ inline size_t sort_record_bytes(int64_t cols) { return kSortRecHeader + ((size_t)cols / 8) * kSortUnit; }

// Relaxed device-scope atomics on global memory (the HIP wrappers take generic pointers).
__device__ __forceinline__ unsigned long long global_atomic_add(EQ_GLOBAL unsigned long long* p, unsigned long long v) {
  return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void global_atomic_or(EQ_GLOBAL int32_t* p, int32_t v) {
  (void)__hip_atomic_fetch_or(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 128-bit accesses to global memory (vector types without constructors: the HIP ones cannot be
// read through an address-space-qualified pointer).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef double f64x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 global_load128(const EQ_GLOBAL void* p) {
  const u32x4_t v = *reinterpret_cast<const EQ_GLOBAL u32x4_t*>(p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
// streaming variant: the data is used once, so it is marked non-temporal
__device__ __forceinline__ uint4 global_load_stream128(const EQ_GLOBAL void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const EQ_GLOBAL u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void global_store128(EQ_GLOBAL void* p, const uint4 v) {
  u32x4_t t;
  t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
  *reinterpret_cast<EQ_GLOBAL u32x4_t*>(p) = t;
}

// Range-checked view of `bytes` bytes at the wavefront-uniform address `base` (a raw buffer
// resource, stride 0): a load whose offset lies beyond the end returns zero and touches no
// memory, so ragged rows and absent rows need no branch around their loads, and the loads do
// not count as LDS traffic the way loads through generic pointers do.
typedef __amdgpu_buffer_rsrc_t BufferRsrc;
__device__ __forceinline__ BufferRsrc make_buffer(const EQ_GLOBAL void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);   // untyped 32-bit data
}
__device__ __forceinline__ uint32_t buffer_load32(BufferRsrc rs, uint32_t byte_offset) {
  return (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rs, (int)byte_offset, 0, 0);
}
__device__ __forceinline__ uint4 buffer_load_stream128(BufferRsrc rs, uint32_t byte_offset) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)byte_offset, 0, 2);           // 2: non-temporal
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void global_store_stream128(EQ_GLOBAL void* p, const uint4 v) {   // written once, not re-read
  u32x4_t t;
  t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
  __builtin_nontemporal_store(t, reinterpret_cast<EQ_GLOBAL u32x4_t*>(p));
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
// Block-wide sums through a small LDS scratch (kMaxWaves entries) for any workgroup size up
// to 512; the partial sums are combined in wavefront order by every thread; ends with a barrier.
__device__ __forceinline__ double block_sum(double v, double* red) {
  const int nw = (int)(blockDim.x / kWave);
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = v;
  __syncthreads();
  double t = red[0];
  for (int w = 1; w < nw; ++w) t += red[w];
  return t;
}
__device__ __forceinline__ uint32_t block_sum_u32(uint32_t v, uint32_t* red) {
  const int nw = (int)(blockDim.x / kWave);
  v = (uint32_t)wave_sum((int)v);
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = v;
  __syncthreads();
  uint32_t t = red[0];
  for (int w = 1; w < nw; ++w) t += red[w];
  return t;
}

// ---- Eq. 1: levels -----------------------------------------------------------------------
// 1.5 * 2^23: fma(x, inv, kMagic) is the exact x * inv plus kMagic rounded once to binary32;
// in [2^23, 2^24) the spacing is 1, so the result is kMagic + rint(x * inv) (ties to even;
// kMagic is even) whenever |x * inv| < 2^22.  The range floor r >= r0 / 1024 keeps
// |x * inv| <= 1024 D < 2^18.  Clamping after the rounding equals clamping before it
// because the bounds are integers.
constexpr float kMagic = 12582912.0f;
__device__ __forceinline__ float level_of(float x, float inv, float clo, float chi) {
  return fminf(fmaxf(__builtin_fmaf(x, inv, kMagic) - kMagic, clo), chi);
}

// ---- division by a value whose correctly rounded reciprocal is known -----------------------
// q0 = a * rb; two residual corrections with fused multiply-adds.  With rb = RN(1 / b) the
// last step returns the correctly rounded a / b (Markstein's theorem), i.e. the same bits as
// an IEEE division, at 5 operations instead of ~30.
// (binary64: the operands here are sums and products of binary32-range quantities, far from
// the ends of the binary64 range, so no guard is needed; a zero numerator returns zero.)
__host__ __device__ __forceinline__ double div_known_rcp(double a, double b, double rb) {
  const double q0 = a * rb;
  const double r0 = fma(-b, q0, a);
  const double q1 = fma(r0, rb, q0);
  const double r1 = fma(-b, q1, a);
  return fma(r1, rb, q1);
}
// binary32: a range close to the subnormals (or to overflow) takes the ordinary division.
__host__ __device__ __forceinline__ float div_known_rcp(float a, float b, float rb) {
  const float aa = fabsf(a);
  if (!(aa > 1e-30f && aa < 1e30f)) return a / b;
  const float q0 = a * rb;
  const float r0 = fmaf(-b, q0, a);
  const float q1 = fmaf(r0, rb, q0);
  const float r1 = fmaf(-b, q1, a);
  return fmaf(r1, rb, q1);
}

// ---- the scalar recurrence --------------------------------------------------------------
// Loss (minus the constant sum x^2) and its derivative with respect to the range at scale
// s = r / D, from the exact sums A and B:  loss = s^2 A - 2 s B + sum x^2;
// d loss / d s = 2 (s A - B) is Eq. 2 with Q[x_i] = s c_i; d s / d r = 1 / D.
__device__ __forceinline__ void loss_and_grad(const KParams& kp, float s32, double A, double B, double& J, double& g) {
  const double s = (double)s32;
  const double e = s * A - B;
  J = s * (e - B);
  g = div_known_rcp(2.0 * e, (double)kp.D, kp.rD64);
}

// Adam (bias-corrected) on the range of one unit; moments in binary64.
// The bias corrections 1 - beta^t are the same for every unit, so the host tabulates them
// together with their correctly rounded reciprocals (kp.adam_tab) and the two divisions by
// them cost 5 operations each.
struct Adam {
  double m, v;
  __device__ __forceinline__ void init() { m = 0.0; v = 0.0; }
  // bc = {1 - b1^t, RN(1 / .), 1 - b2^t, RN(1 / .)} of this step, loaded by the caller ahead of
  // the evaluation so that the memory latency is hidden behind it
  __device__ __forceinline__ float step(const KParams& kp, const double (&bc)[4], float r32, double g, double floor_r) {
    m = kp.b1 * m + (1.0 - kp.b1) * g;
    v = kp.b2 * v + (1.0 - kp.b2) * (g * g);
    const double mh = div_known_rcp(m, bc[0], bc[1]);
    const double vh = div_known_rcp(v, bc[2], bc[3]);
    const double r64 = (double)r32 - kp.lr * (mh / (sqrt(vh) + kp.eps));
    return (float)fmax(r64, floor_r);
  }
};
__device__ __forceinline__ void load_bias_corrections(const KParams& kp, int t, double (&bc)[4]) {
  const EQ_GLOBAL f64x2_t* p = reinterpret_cast<const EQ_GLOBAL f64x2_t*>(kp.adam_tab + 4 * t);
  const f64x2_t a = p[0], b = p[1];
  bc[0] = a.x; bc[1] = a.y; bc[2] = b.x; bc[3] = b.y;
}
// scale and reciprocal scale of a range (binary32, correctly rounded)
__device__ __forceinline__ void scale_of(const KParams& kp, float r32, float& s32, float& inv) {
  s32 = div_known_rcp(r32, kp.D, kp.rD32);
  inv = 1.0f / s32;
}

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
