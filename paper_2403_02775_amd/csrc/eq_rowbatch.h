// Batched row staging for the unit-per-lane kernel.
//
// Several rows are staged at once by all threads of the workgroup, with every 128-bit HBM
// load of the batch in flight before the first one is used, a handful of barriers per batch
// instead of per row, and one staging reservation per batch.  The row's data stays in
// registers from the load until it is written (once) to the LDS pool.
//
// Statistics (Eq. 3) take a fast path and an exact path with identical results:
//   fast  : sum x and sum x^2 in binary32 per thread, binary64 across threads.  The outlier
//           test is decided only for elements whose |x - mean| is farther than a relative
//           1e-4 from n*sigma; the error of the fast sums is below 2e-5 of the threshold
//           (<= 70 roundings of 2^-24 on sums whose terms are bounded through the guard
//           mean^2 < variance), so those decisions equal the exact ones.
//   exact : a row with an element inside that band, or with mean^2 >= variance (which also
//           covers constant rows), is redone with the two-pass binary64 sums.
#pragma once

#include "eq_common.h"
#include "eq_rowstage.h"

namespace eq {

constexpr float kBand = 1.0e-4f;

template <int RB, int K>
struct BatchScratch {
  float part[RB][kMaxWaves][2];      // per wavefront: sum x, sum x^2 of each row
  double dred[kMaxWaves];
  uint32_t wtot[RB][K][kMaxWaves];   // outliers per (row, chunk slice, wavefront)
  uint32_t rowtot[RB];
  unsigned long long rowbase[RB];    // staging position of the row, ~0 when it does not fit
  uint32_t slow[RB];
};

template <int DT>
__device__ __forceinline__ void chunk_floats(const uint4 v, float (&x)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    x[2 * k] = widen16<DT>(w[k] & 0xFFFFu);
    x[2 * k + 1] = widen16<DT>(w[k] >> 16);
  }
}

// Stages rows [row0, row0 + nrows), nrows <= RB, of matrix md: chunk ch of row r goes to
// Layout::off(ch0 + r * chunks_per_row + ch).  Thread t owns chunks t, t + NT, ... (K of them
// per row).  Ends with a barrier; afterwards the pool holds the normal values and 0 at
// outlier positions, and the outliers sit in the staging area (one run per row).
template <int DT, int NT, int RB, int K, class Layout>
__device__ __forceinline__ void stage_rows_batch(const MatDesc& md, const KParams& kp, int64_t row0, int nrows,
                                                 unsigned char* pool, uint32_t ch0, BatchScratch<RB, K>* sc) {
  const uint32_t nchunks = (uint32_t)md.cols >> 3;
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  constexpr int NW = NT / kWave;

  // ---- every load of the batch in flight ----
  uint4 v[RB][K];
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    const uint4* src = reinterpret_cast<const uint4*>(md.W + (row0 + r) * md.ld);
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const uint32_t ch = (uint32_t)i * NT + tid;
      v[r][i] = (r < nrows && ch < nchunks) ? load_stream128(src + ch) : make_uint4(0, 0, 0, 0);
    }
  }
  if (tid < (uint32_t)RB) sc->slow[tid] = 0;

  // ---- fast sums ----
  bool bad = false;
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int i = 0; i < K; ++i) {
      float x[8];
      chunk_floats<DT>(v[r][i], x);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        s1 += x[k];
        s2 = __builtin_fmaf(x[k], x[k], s2);
      }
    }
    // An Inf or NaN makes the sum of squares non-finite; only then look at the elements (for
    // bf16 a huge finite value can overflow the square too, so the sum alone does not decide).
    if (!(s2 < __builtin_inff())) {
#pragma unroll
      for (int i = 0; i < K; ++i) {
        const uint32_t w[4] = {v[r][i].x, v[r][i].y, v[r][i].z, v[r][i].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) bad = bad || nonfinite16<DT>(w[k] & 0xFFFFu) || nonfinite16<DT>(w[k] >> 16);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      s1 += __shfl_xor(s1, o);
      s2 += __shfl_xor(s2, o);
    }
    if (lane == 0) {
      sc->part[r][wave][0] = s1;
      sc->part[r][wave][1] = s2;
    }
  }
  if (__any(bad) && lane == 0) atomicOr(md.status, EQ_S_NONFINITE);
  __syncthreads();

  // ---- thresholds and masks ----
  const double cnt = (double)md.cols;
  uint32_t m[RB][K];
  float mu_f[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    double S1 = 0.0, S2 = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      S1 += (double)sc->part[r][w][0];
      S2 += (double)sc->part[r][w][1];
    }
    double mu, sigma;
    bool slow = false;
    if (kp.scope == EQ_STAT_MATRIX) {
      mu = md.mat_stats[0];
      sigma = md.mat_stats[1];
      slow = true;                       // whole-matrix statistics are exact already: decide every element exactly
    } else {
      mu = S1 / cnt;
      const double ms = S2 / cnt;        // mean square = variance + mean^2
      const double var = ms - mu * mu;
      slow = !(var + var > ms) || kp.n < 0.5;   // mean^2 >= variance, a constant row, NaN; or a threshold so
                                                 // small that the error of the mean is not negligible against it
      sigma = sqrt(fmax(var, 0.0));
    }
    const double thr = kp.n * sigma;
    mu_f[r] = (float)mu;
    const float thr_lo = (float)thr * (1.0f - kBand), thr_hi = (float)thr * (1.0f + kBand);
    bool border = false;
#pragma unroll
    for (int i = 0; i < K; ++i) {
      float x[8], d[8];
      chunk_floats<DT>(v[r][i], x);
#pragma unroll
      for (int k = 0; k < 8; ++k) d[k] = fabsf(x[k] - mu_f[r]);
      const float dmax = fmaxf(fmaxf(fmaxf(d[0], d[1]), fmaxf(d[2], d[3])), fmaxf(fmaxf(d[4], d[5]), fmaxf(d[6], d[7])));
      uint32_t mm = 0;
      if (dmax >= thr_lo) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          mm |= (d[k] >= thr_hi ? 1u : 0u) << k;
          border = border || (d[k] >= thr_lo && d[k] < thr_hi);
        }
      }
      const uint32_t ch = (uint32_t)i * NT + tid;
      m[r][i] = (r < nrows && ch < nchunks) ? mm : 0u;
    }
    if (r < nrows && (slow || border)) sc->slow[r] = 1u;    // benign race: every writer stores 1
  }
  __syncthreads();

  // ---- exact redo of the rows that asked for it (uniform branch per row) ----
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    if (r < nrows && sc->slow[r]) {
      double mu, sigma;
      if (kp.scope == EQ_STAT_MATRIX) {
        mu = md.mat_stats[0];
        sigma = md.mat_stats[1];
      } else {
        double s = 0.0;
#pragma unroll
        for (int i = 0; i < K; ++i) {
          float x[8];
          chunk_floats<DT>(v[r][i], x);
#pragma unroll
          for (int k = 0; k < 8; ++k) s += (double)x[k];     // absent chunks hold zeros
        }
        mu = block_sum(s, sc->dred) / cnt;
        double q = 0.0;
#pragma unroll
        for (int i = 0; i < K; ++i) {
          const uint32_t ch = (uint32_t)i * NT + tid;
          if (ch < nchunks) {
            float x[8];
            chunk_floats<DT>(v[r][i], x);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              const double dd = (double)x[k] - mu;
              q += dd * dd;
            }
          }
        }
        sigma = sqrt(block_sum(q, sc->dred) / cnt);
      }
      const double thr = kp.n * sigma;
#pragma unroll
      for (int i = 0; i < K; ++i) {
        const uint32_t ch = (uint32_t)i * NT + tid;
        m[r][i] = (ch < nchunks && sigma > 0.0) ? chunk_mask<DT>(v[r][i], mu, thr) : 0u;
      }
    }
  }

  // ---- values to the pool (raw; outliers are zeroed below by the thread that owns them) ----
#pragma unroll
  for (int r = 0; r < RB; ++r) {
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const uint32_t ch = (uint32_t)i * NT + tid;
      if (r < nrows && ch < nchunks)
        *reinterpret_cast<uint4*>(pool + Layout::off(ch0 + (uint32_t)r * nchunks + ch)) = v[r][i];
    }
  }

  // ---- outlier compaction in column order: chunk order is (slice i, thread) ----
  uint32_t inc[RB][K];
  bool any_mine = false;
#pragma unroll
  for (int r = 0; r < RB; ++r) {
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const uint32_t c = __popc(m[r][i]);
      any_mine = any_mine || c != 0;
      uint32_t s = c;
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t t = __shfl_up(s, o);
        if (lane >= (uint32_t)o) s += t;
      }
      inc[r][i] = s;
      if (lane == kWave - 1) sc->wtot[r][i][wave] = s;
    }
  }
  __syncthreads();
  if (tid < (uint32_t)RB) {
    uint32_t t = 0;
    if ((int)tid < nrows) {
      for (int i = 0; i < K; ++i)
        for (int w = 0; w < NW; ++w) t += sc->wtot[tid][i][w];
    }
    sc->rowtot[tid] = t;
  }
  __syncthreads();
  if (tid == 0) {
    uint32_t total = 0;
    for (int r = 0; r < nrows; ++r) total += sc->rowtot[r];
    unsigned long long b = 0;
    if (total) b = atomicAdd(md.cursor, (unsigned long long)total);
    for (int r = 0; r < nrows; ++r) {
      const uint32_t t = sc->rowtot[r];
      const bool fits = b + t <= (unsigned long long)md.capacity;
      md.row_count[row0 + r] = t;
      md.row_stage[row0 + r] = fits ? (uint32_t)b : 0xFFFFFFFFu;
      if (!fits) atomicOr(md.status, EQ_S_OUTLIER_OVERFLOW);
      sc->rowbase[r] = fits ? b : ~0ull;
      b += t;
    }
  }
  __syncthreads();
  if (any_mine) {
#pragma unroll
    for (int r = 0; r < RB; ++r) {
#pragma unroll
      for (int i = 0; i < K; ++i) {
        const uint32_t mm = m[r][i];
        if (mm) {
          uint32_t before = 0;
          for (int i2 = 0; i2 < i; ++i2)
            for (int w = 0; w < NW; ++w) before += sc->wtot[r][i2][w];
          for (uint32_t w = 0; w < wave; ++w) before += sc->wtot[r][i][w];
          const unsigned long long base = sc->rowbase[r];
          const bool fits = base != ~0ull;
          unsigned long long pos = base + before + (inc[r][i] - __popc(mm));
          const uint32_t ch = (uint32_t)i * NT + tid;
          unsigned short* e = reinterpret_cast<unsigned short*>(pool + Layout::off(ch0 + (uint32_t)r * nchunks + ch));
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            if (mm & (1u << j)) {
              if (fits) {
                md.st_col[pos] = ch * 8u + (uint32_t)j;
                md.st_val[pos] = e[j];
              }
              ++pos;
              e[j] = 0;
            }
          }
        }
      }
    }
  }
  __syncthreads();
}

}  // namespace eq
