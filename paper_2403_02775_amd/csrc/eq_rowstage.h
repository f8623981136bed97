// Row staging: the part of the path that touches HBM on the input side.
//
// A workgroup streams one row from HBM exactly once (128-bit coalesced loads) into LDS,
// computes the row's mean and sigma, builds the outlier mask of Eq. 3, compacts the
// outliers in column order into the staging area of the workspace, and replaces them by 0
// in the LDS copy, so that the range optimisation that follows only sees normal values
// (Sec. 4.2: only the normal elements are optimised).
#pragma once

#include "eq_common.h"

namespace eq {

// LDS placement of the 16-byte chunk `ch` (8 elements) of the staged row.
//   Linear : chunk ch at byte 16*ch.
//   Padded : every 128-element unit (16 chunks) is followed by one empty chunk, so that
//            lanes that each own one unit (stride 272 B) hit distinct banks on 128-bit reads.
// The batched staging keeps one outlier-mask byte per chunk (eq_rowbatch.h): mask_off(ch) is its
// place, in the pool itself (the padding chunk of the unit: 16 bytes for its 16 chunks) or in a
// separate area of one byte per chunk that the caller provides.  Either way the 16 bytes of a
// unit are contiguous and 16-byte aligned.
struct LinearLayout {
  static constexpr bool kMaskInPool = false;
  static __device__ __forceinline__ uint32_t off(uint32_t ch) { return ch * 16u; }
  static __device__ __forceinline__ uint32_t mask_off(uint32_t ch) { return ch; }
};
struct Padded128Layout {
  static constexpr bool kMaskInPool = true;
  static __device__ __forceinline__ uint32_t off(uint32_t ch) { return ch * 16u + (ch >> 4) * 16u; }
  static __device__ __forceinline__ uint32_t mask_off(uint32_t ch) { return (ch >> 4) * 272u + 256u + (ch & 15u); }
};

struct StageScratch {      // small LDS block used by the staging steps
  double red[kMaxWaves];
  uint32_t redu[kMaxWaves];
  uint32_t wtot[kMaxWaves];
  unsigned long long base;
};

// Mean and population sigma of `n` staged chunks starting at chunk `ch0`, by all threads of
// the workgroup (two passes over LDS, binary64).  Ends with a barrier.
template <int DT, class Layout>
__device__ __forceinline__ void block_mean_sigma(const unsigned char* lds_row, uint32_t ch0, uint32_t nchunks,
                                                 StageScratch* sc, double& mu, double& sigma) {
  double s = 0.0;
  for (uint32_t ch = threadIdx.x; ch < nchunks; ch += blockDim.x) {
    const uint4 v = *reinterpret_cast<const uint4*>(lds_row + Layout::off(ch0 + ch));
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      s += (double)widen16<DT>(w[k] & 0xFFFFu);
      s += (double)widen16<DT>(w[k] >> 16);
    }
  }
  const double cnt = (double)nchunks * 8.0;
  mu = block_sum(s, sc->red) / cnt;
  double q = 0.0;
  for (uint32_t ch = threadIdx.x; ch < nchunks; ch += blockDim.x) {
    const uint4 v = *reinterpret_cast<const uint4*>(lds_row + Layout::off(ch0 + ch));
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const double d0 = (double)widen16<DT>(w[k] & 0xFFFFu) - mu;
      const double d1 = (double)widen16<DT>(w[k] >> 16) - mu;
      q += d0 * d0;
      q += d1 * d1;
    }
  }
  sigma = sqrt(block_sum(q, sc->red) / cnt);
}

// Eq. 3 for one chunk: bit j set when element j is an outlier.
template <int DT>
__device__ __forceinline__ uint32_t chunk_mask(const uint4 v, double mu, double thr) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  uint32_t m = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const double d0 = fabs((double)widen16<DT>(w[k] & 0xFFFFu) - mu);
    const double d1 = fabs((double)widen16<DT>(w[k] >> 16) - mu);
    m |= (d0 >= thr ? 1u : 0u) << (2 * k);
    m |= (d1 >= thr ? 1u : 0u) << (2 * k + 1);
  }
  return m;
}

// Loads row `row` of matrix `md` into LDS (chunk ch -> Layout::off(ch0 + ch)) and flags
// non-finite values.  No barrier at the end.
template <int DT, class Layout>
__device__ __forceinline__ void stage_load_row(const MatDesc& md, int64_t row, unsigned char* lds_row, uint32_t ch0) {
  const uint32_t nchunks = (uint32_t)md.cols >> 3;
  const EQ_GLOBAL uint16_t* src = md.W + row * md.ld;
  bool bad = false;
  for (uint32_t ch = threadIdx.x; ch < nchunks; ch += blockDim.x) {
    const uint4 v = global_load_stream128(src + 8 * (size_t)ch);
    *reinterpret_cast<uint4*>(lds_row + Layout::off(ch0 + ch)) = v;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) bad = bad || nonfinite16<DT>(w[k] & 0xFFFFu) || nonfinite16<DT>(w[k] >> 16);
  }
  if (__any(bad) && (threadIdx.x & (kWave - 1)) == 0) global_atomic_or(md.status, EQ_S_NONFINITE);
}

// Given the mask bytes of the row's chunks (maskb[ch], LDS), counts the row's outliers,
// reserves a contiguous run in the staging area, writes (column, raw value) in ascending
// column order and zeroes the outliers in the LDS copy.  All threads of the workgroup call
// it; it starts and ends with a barrier.
template <class Layout>
__device__ __forceinline__ void stage_compact_row(const MatDesc& md, int64_t row, unsigned char* lds_row, uint32_t ch0,
                                                  const unsigned char* maskb, StageScratch* sc) {
  const uint32_t nchunks = (uint32_t)md.cols >> 3;
  const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  uint32_t cnt = 0;
  __syncthreads();
  for (uint32_t ch = threadIdx.x; ch < nchunks; ch += blockDim.x) cnt += __popc((uint32_t)maskb[ch]);
  const uint32_t total = block_sum_u32(cnt, sc->redu);
  if (threadIdx.x == 0) {
    unsigned long long b = 0;
    if (total) b = global_atomic_add(md.cursor, (unsigned long long)total);
    const bool fits = b + total <= (unsigned long long)md.capacity;
    md.row_count[row] = total;
    md.row_stage[row] = fits ? (uint32_t)b : 0xFFFFFFFFu;
    if (!fits) global_atomic_or(md.status, EQ_S_OUTLIER_OVERFLOW);
    sc->base = fits ? b : ~0ull;
  }
  __syncthreads();
  if (total == 0) return;
  const unsigned long long base = sc->base;
  const bool fits = base != ~0ull;
  uint32_t running = 0;
  for (uint32_t blk = 0; blk < nchunks; blk += blockDim.x) {
    const uint32_t ch = blk + threadIdx.x;
    const uint32_t m = ch < nchunks ? (uint32_t)maskb[ch] : 0u;
    const uint32_t c = __popc(m);
    // inclusive scan inside the wave, then across the waves
    uint32_t inc = c;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const uint32_t t = __shfl_up(inc, o);
      if (lane >= (uint32_t)o) inc += t;
    }
    if (lane == kWave - 1) sc->wtot[wave] = inc;
    __syncthreads();
    uint32_t before = 0, blk_total = 0;
    for (uint32_t w = 0; w < blockDim.x / kWave; ++w) {
      const uint32_t t = sc->wtot[w];
      if (w < wave) before += t;
      blk_total += t;
    }
    if (m) {
      unsigned long long pos = base + running + before + (inc - c);
      unsigned short* e = reinterpret_cast<unsigned short*>(lds_row + Layout::off(ch0 + ch));
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (m & (1u << j)) {
          if (fits) {
            md.st_col[pos] = ch * 8u + (uint32_t)j;
            md.st_val[pos] = e[j];
          }
          ++pos;
          e[j] = 0;
        }
      }
    }
    running += blk_total;
    __syncthreads();
  }
}

// Row scope (and matrix scope, whose mean / sigma come from a pre-pass): full staging of
// one row.  `maskb` needs cols/8 bytes of LDS.  Ends with a barrier; afterwards the LDS
// copy holds the normal values and 0 at outlier positions.
template <int DT, class Layout>
__device__ __forceinline__ void stage_row(const MatDesc& md, const KParams& kp, int64_t row, unsigned char* lds_row,
                                          uint32_t ch0, unsigned char* maskb, StageScratch* sc) {
  const uint32_t nchunks = (uint32_t)md.cols >> 3;
  stage_load_row<DT, Layout>(md, row, lds_row, ch0);
  __syncthreads();
  double mu, sigma;
  if (kp.scope == EQ_STAT_MATRIX) {
    mu = md.mat_stats[0];
    sigma = md.mat_stats[1];
  } else {
    block_mean_sigma<DT, Layout>(lds_row, ch0, nchunks, sc, mu, sigma);
  }
  const double thr = kp.n * sigma;
  const bool any_possible = sigma > 0.0;
  for (uint32_t ch = threadIdx.x; ch < nchunks; ch += blockDim.x) {
    const uint4 v = *reinterpret_cast<const uint4*>(lds_row + Layout::off(ch0 + ch));
    maskb[ch] = any_possible ? (unsigned char)chunk_mask<DT>(v, mu, thr) : (unsigned char)0;
  }
  stage_compact_row<Layout>(md, row, lds_row, ch0, maskb, sc);
}

}  // namespace eq
