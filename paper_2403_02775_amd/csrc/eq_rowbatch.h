// Batched row staging for the unit-per-lane kernel.
//
// Several rows are staged at once by all threads of the workgroup, with every 128-bit HBM
// load of the batch in flight before the first one is used, a handful of barriers per batch
// and one staging reservation per batch.
//
// Outliers are rare (< 1 % of the elements, Sec. 5), so only a few 16-byte chunks per thread
// hold one.  The bulk pass therefore does the minimum per element (the sums, and one test per
// chunk: can anything in it reach the threshold?), and the chunks that pass the test
// ("candidates") are queued per wavefront and dealt out evenly over its lanes, which decide
// their elements and leave one MASK BYTE per chunk (bit j: element j is an outlier) next to the
// data: in the 16 bytes of padding that follow every 128-element unit of the padded pool layout
// (one byte for each of its 16 chunks), or in a separate area for the linear layout.  After that
// the work goes per UNIT: a thread reads its unit's 16 mask bytes at once, the population counts
// are prefix-summed over the batch (rows and units in order), one thread reserves the batch's
// run of the staging list with a single atomic, and every thread writes its unit's outliers at
// run start + prefix and replaces them by 0 in the pool.  A row's run therefore comes out in
// ascending column order without any sorting, and no LDS atomic is involved.
//
// Statistics (Eq. 3) take a fast path and an exact path with identical results:
//   fast  : sum x and sum x^2 by packed dot products, mean and sigma in binary32.  The outlier
//           test is decided only for elements whose |x - mean| is farther than a relative
//           1e-4 from n*sigma; the error of the fast mean and threshold is below 2.7e-5 of the
//           threshold (<= 90 roundings of 2^-24 on quantities that are bounded through the
//           guard mean^2 < variance, n >= 0.5), so those decisions equal the exact ones.
//   exact : a row with an element inside that band, or that fails the guard (which also
//           covers constant rows and rows of mostly subnormal binary16 values), is redone from
//           its pool copy with the two-pass binary64 sums and decided element by element in
//           binary64.
#pragma once

#include <type_traits>

#include "eq_common.h"
#include "eq_rowstage.h"

namespace eq {

constexpr float kBand = 1.0e-4f;

constexpr int kQueue = 128;          // candidate chunks a wavefront can queue per batch

template <int RB, int NW>
struct BatchScratch {
  float part[RB][NW][2];             // per wavefront: sum x, sum x^2 of each row
  static constexpr int kW = NW > kMaxWaves ? NW : kMaxWaves;   // (kMaxWaves entries for every workgroup of up to 512 threads)
  double dred[kW];
  double mu[RB], thr[RB];            // exact mean and n*sigma of the rows that were redone
  float4 fast[RB];                   // fast mean, lower and upper end of the band around n*sigma
  unsigned long long base;           // start of the batch's run of the staging list
  uint32_t wtot[kW];                 // outliers found by each wavefront's units
  uint32_t slow[RB];                 // row takes the exact path
  uint32_t rowmax_bits[RB];          // for kernels with one range per row: bit patterns of max(x, 0) and
  uint32_t rownegmin_bits[RB];       // max(-x, 0) over the row's normal values
  // first the candidate chunks of each wavefront (row << 16 | chunk); once they are dealt with,
  // the exclusive prefix of the outlier counts of the batch's units (at most 1.5 NT + 1 of them)
  union {
    uint32_t queue[NW][kQueue];
    uint32_t pre[NW * kQueue];
  };
};

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bfloat2_t __attribute__((ext_vector_type(2)));

// Packed 16-bit floating-point minimum / maximum as single instructions (the generic minimum
// of the language first quiets a signalling NaN of each operand, one more instruction apiece;
// rows with a NaN are flagged and their results are unspecified anyway).
__device__ __forceinline__ uint32_t pk_min_f16(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ uint32_t pk_max_f16(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// Three-operand forms (IEEE-754 minimum / maximum: a NaN operand gives NaN, -0 < +0).
__device__ __forceinline__ uint32_t pk_min3_f16(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_pk_minimum3_f16 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ uint32_t pk_max3_f16(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_pk_maximum3_f16 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// s1 += x0 + x1, s2 += x0^2 + x1^2 for the two 16-bit values of w, one packed dot-product
// instruction each, accumulating in binary32.  Measured on gfx950 against exact sums: the
// result is within 3 * 2^-24 of the largest of its three terms; a subnormal binary16 operand
// is not flushed, its product carries a relative error of up to 2^-18 of that product.
template <int DT>
__device__ __forceinline__ void pair_sums(uint32_t w, float& s1, float& s2) {
  if (DT == EQ_F16) {
    const half2_t h = __builtin_bit_cast(half2_t, w);
    const half2_t ones = {(_Float16)1.0f, (_Float16)1.0f};
    s1 = __builtin_amdgcn_fdot2(h, ones, s1, false);
    s2 = __builtin_amdgcn_fdot2(h, h, s2, false);
  } else {
    const bfloat2_t h = __builtin_bit_cast(bfloat2_t, w);
    const bfloat2_t ones = __builtin_bit_cast(bfloat2_t, 0x3F803F80u);
    s1 = __builtin_amdgcn_fdot2_f32_bf16(h, ones, s1, false);
    s2 = __builtin_amdgcn_fdot2_f32_bf16(h, h, s2, false);
  }
}

// Sum over the wavefront by data-parallel primitives; lane 63 holds the total.
__device__ __forceinline__ float wave_sum_to_last(float v) {
  auto step = [&](auto ctrl, auto rows) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value,
                                                                 decltype(rows)::value, 0xF, true));
  };
  step(std::integral_constant<int, 0x111>{}, std::integral_constant<int, 0xF>{});   // row_shr:1
  step(std::integral_constant<int, 0x112>{}, std::integral_constant<int, 0xF>{});   // row_shr:2
  step(std::integral_constant<int, 0x114>{}, std::integral_constant<int, 0xF>{});   // row_shr:4
  step(std::integral_constant<int, 0x118>{}, std::integral_constant<int, 0xF>{});   // row_shr:8
  step(std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xA>{});   // row_bcast:15 -> rows 1, 3
  step(std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xC>{});   // row_bcast:31 -> rows 2, 3
  return v;
}

// Inclusive prefix sum over the wavefront (same steps as above: they form a scan).
__device__ __forceinline__ uint32_t wave_scan_inclusive(uint32_t v) {
  auto step = [&](auto ctrl, auto rows) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, decltype(ctrl)::value, decltype(rows)::value, 0xF, true);
  };
  step(std::integral_constant<int, 0x111>{}, std::integral_constant<int, 0xF>{});
  step(std::integral_constant<int, 0x112>{}, std::integral_constant<int, 0xF>{});
  step(std::integral_constant<int, 0x114>{}, std::integral_constant<int, 0xF>{});
  step(std::integral_constant<int, 0x118>{}, std::integral_constant<int, 0xF>{});
  step(std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xA>{});
  step(std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xC>{});
  return v;
}

// Largest binary16 value strictly below the binary32 value b, and smallest strictly above.
__device__ __forceinline__ uint32_t f16_below(float b) {
  uint32_t h = (uint32_t)__half_as_ushort(__float2half_rn(b));
  if (!(__half2float(__ushort_as_half((unsigned short)h)) < b)) {
    if ((h & 0x7FFFu) == 0u) h = 0x8001u;           // below zero: the smallest negative subnormal
    else h = (h & 0x8000u) ? h + 1u : h - 1u;
  }
  return h;
}
__device__ __forceinline__ uint32_t f16_above(float b) { return f16_below(-b) ^ 0x8000u; }

template <int DT>
__device__ __forceinline__ void chunk_floats(const uint4 v, float (&x)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    x[2 * k] = widen16<DT>(w[k] & 0xFFFFu);
    x[2 * k + 1] = widen16<DT>(w[k] >> 16);
  }
}

// Staging of rows [row0, row0 + nrows), nrows <= RB, of matrix md: chunk ch of row r goes to
// Layout::off(ch0 + r * chunks_per_row + ch).  Thread t owns chunks t, t + NT, ... (K of them
// per row).  Ends with a barrier; afterwards the pool holds the normal values and 0 at
// outlier positions, and the outliers sit in the staging area (one run per row, any order).
// Split in two so that a caller can have the next batch's loads in flight while it works.
// Issues every 128-bit load of rows [row0, row0 + nrows): thread t takes chunks t, t + NT, ...
// of each row; absent rows and chunks read as zero.
// WM ("wavefront-major", one row per batch): instead of chunks t, t + NT, ... thread t of wavefront
// w takes chunks c0(w) + lane, c0(w) + lane + 64, ... of the contiguous part [c0(w), c0(w + 1)) of
// the row that holds the units [w upr / NW, (w + 1) upr / NW): a wavefront then decides, writes and
// later emits its own units only, and the wavefronts of a workgroup meet at three barriers per
// batch (the sums, the counts, the reservation) instead of six.
template <int NT, bool WM>
__device__ __forceinline__ void wave_part(uint32_t nchunks, uint32_t& c0, uint32_t& c1) {
  constexpr uint32_t NW = NT / kWave;
  const uint32_t wave = threadIdx.x / kWave, upr = nchunks >> 4;
  c0 = WM ? ((wave * upr) / NW) << 4 : 0u;
  c1 = WM ? (((wave + 1u) * upr) / NW) << 4 : nchunks;
}
template <int NT, bool WM>
__device__ __forceinline__ uint32_t chunk_of(int i, uint32_t c0) {
  return WM ? c0 + (uint32_t)i * kWave + (threadIdx.x & (kWave - 1)) : (uint32_t)i * NT + threadIdx.x;
}

template <int NT, int RB, int K, bool WM = false>
__device__ __forceinline__ void batch_issue_loads(const MatDesc& md, int64_t row0, int nrows, uint4 (&v)[RB][K]) {
  uint32_t c0, c1;
  wave_part<NT, WM>((uint32_t)md.cols >> 3, c0, c1);
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    const bool present = r < nrows;
    // the view ends with the row, or with the wavefront's part of it: loads beyond read as zero
    const BufferRsrc rs = make_buffer(md.W + (present ? row0 + r : row0) * md.ld, present ? (WM ? c1 * 16u : (uint32_t)md.cols * 2u) : 0u);
#pragma unroll
    for (int i = 0; i < K; ++i) v[r][i] = buffer_load_stream128(rs, chunk_of<NT, WM>(i, c0) * 16u);
  }
}

// Everything after the loads (v = what batch_issue_loads returned for the same rows).  v is read
// up to the per-chunk outlier test; everything after that works on the pool copy, and
// `after_reservation_issued()` (called once by every thread, later than the last use of v) may
// overwrite v.  The rows must be whole units (cols a multiple of 128) and ch0 a multiple of 16.
// mask_area: one byte per chunk of the batch, 16-byte aligned, for layouts that do not keep the
// mask bytes in the pool (ignored otherwise).
// WRITE = false: statistics, mask and zeroing only; nothing goes to the staging list (a caller that
// only needs the normal values, the list being written by a later pass over the same rows).
template <int DT, int NT, int RB, int K, class Layout, bool WM = false, bool WRITE = true, class Hook>
__device__ __forceinline__ void stage_loaded_rows(const MatDesc& md, const KParams& kp, int64_t row0, int nrows,
                                                  unsigned char* pool, uint32_t ch0, unsigned char* mask_area,
                                                  BatchScratch<RB, NT / kWave>* sc, const uint4 (&v)[RB][K],
                                                  Hook&& after_reservation_issued) {
  static_assert(RB * K <= 32, "candidate flags are one 32-bit word");
  constexpr int NW = NT / kWave;
  static_assert((RB * K * NT) / 16 + 1 <= NW * kQueue, "the unit prefix must fit the space of the candidate queues");
  static_assert(!WM || RB == 1, "wavefront-major staging takes one row per batch");
  const uint32_t nchunks = (uint32_t)md.cols >> 3;
  uint32_t part_c0, part_c1;                               // the chunks this thread's wavefront looks after
  wave_part<NT, WM>(nchunks, part_c0, part_c1);
  const uint32_t upr = nchunks >> 4;                       // units per row
  const uint32_t nslots = (uint32_t)nrows * upr;           // units of the batch, in (row, column) order
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  unsigned char* const mb = Layout::kMaskInPool ? pool : mask_area;

  if (tid < (uint32_t)RB) sc->slow[tid] = 0;
  // no outliers anywhere yet (published by the barrier behind the sums; wavefront-major: a
  // wavefront clears the bytes of its own units, which no other wavefront ever touches)
  if (WM) {
    const uint32_t s = (part_c0 >> 4) + lane;
    if (s < (part_c1 >> 4)) *reinterpret_cast<uint4*>(mb + Layout::mask_off(ch0 + (s << 4))) = make_uint4(0, 0, 0, 0);
  } else {
    for (uint32_t s = tid; s < nslots; s += NT)
      *reinterpret_cast<uint4*>(mb + Layout::mask_off(ch0 + (s << 4))) = make_uint4(0, 0, 0, 0);
  }

  // ---- fast sums; the values go to the pool as they are ----
  bool bad = false;
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    float s1 = 0.0f, s2 = 0.0f, t1 = 0.0f, t2 = 0.0f;   // two chains each
#pragma unroll
    for (int i = 0; i < K; ++i) {
      pair_sums<DT>(v[r][i].x, s1, s2);
      pair_sums<DT>(v[r][i].y, t1, t2);
      pair_sums<DT>(v[r][i].z, s1, s2);
      pair_sums<DT>(v[r][i].w, t1, t2);
      const uint32_t ch = chunk_of<NT, WM>(i, part_c0);
      if (r < nrows && ch < part_c1)
        *reinterpret_cast<uint4*>(pool + Layout::off(ch0 + (uint32_t)r * nchunks + ch)) = v[r][i];
    }
    s1 += t1;
    s2 += t2;
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
    s1 = wave_sum_to_last(s1);
    s2 = wave_sum_to_last(s2);
    if (lane == kWave - 1) {
      sc->part[r][wave][0] = s1;
      sc->part[r][wave][1] = s2;
    }
  }
  if (__any(bad) && lane == 0) global_atomic_or(md.status, EQ_S_NONFINITE);
  __syncthreads();

  // ---- thresholds: lane r of every wavefront works out row r, all lanes get them as scalars ----
  const double cnt = (double)md.cols;
  float mu_f[RB], thr_lo[RB];             // bf16 rows: fast mean and lower end of the band
  uint32_t cand_hi[RB], cand_lo[RB];      // fp16 rows: binary16 pairs, a value beyond one of them may be an outlier
  uint32_t slow_rows;                     // bit r: row r takes the exact path
  {
    const uint32_t r = lane < (uint32_t)RB ? lane : 0u;
    float S1 = 0.0f, S2 = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      S1 += sc->part[r][w][0];
      S2 += sc->part[r][w][1];
    }
    float mu, thr;
    bool slow;
    if (kp.scope == EQ_STAT_MATRIX) {
      mu = (float)md.mat_stats[0];
      thr = (float)(kp.n * md.mat_stats[1]);
      slow = true;                        // the matrix-wide statistics are exact: decide every element exactly
    } else {
      // binary32 throughout: a dozen more roundings of 2^-24 on top of those of the sums
      const float rcnt = 1.0f / (float)md.cols;
      mu = S1 * rcnt;
      const float ms = S2 * rcnt;         // mean square = variance + mean^2
      const float var = ms - mu * mu;
      // exact path: mean^2 >= variance, a constant row, NaN; a threshold so small that the error of
      // the mean is not negligible against it; a row of (mostly) subnormal binary16 values
      slow = !(var + var > ms) || kp.n < 0.5 || !(ms >= 1.0e-8f);
      thr = (float)kp.n * __builtin_sqrtf(fmaxf(var, 0.0f));
    }
    const float lo = thr * (1.0f - kBand), hi = thr * (1.0f + kBand);
    // every wavefront stores the same bits, and reads them back itself: no barrier needed
    if (lane < (uint32_t)RB) sc->fast[lane] = make_float4(mu, lo, hi, 0.0f);
    // chunk test for binary16 rows: bounds strictly inside mean +- lo * (1 - 2^-10), the margin
    // covering the roundings of this sum and of |x - mean| in the candidate pass
    const float inner = lo * (1.0f - 0x1p-10f);
    const uint32_t bh = DT == EQ_F16 ? f16_below(mu + inner) : 0u, bl = DT == EQ_F16 ? f16_above(mu - inner) : 0u;
    const uint32_t sb = (uint32_t)__ballot(slow && lane < (uint32_t)nrows);
    slow_rows = sb & ((1u << RB) - 1u);
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) {
      if (DT == EQ_F16) {
        cand_hi[rr] = (uint32_t)__builtin_amdgcn_readlane((int)(bh | (bh << 16)), rr);
        cand_lo[rr] = (uint32_t)__builtin_amdgcn_readlane((int)(bl | (bl << 16)), rr);
      } else {
        mu_f[rr] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mu), rr));
        thr_lo[rr] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lo), rr));
      }
    }
  }
  if (lane < (uint32_t)RB && ((slow_rows >> lane) & 1u)) sc->slow[lane] = 1u;   // benign race: every writer stores 1

  // ---- one test per chunk: can any of its elements be an outlier? ----
  uint32_t cand = 0;                      // bit r * K + i: chunk i of row r needs a look
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    if (!((slow_rows >> r) & 1u)) {
#pragma unroll
      for (int i = 0; i < K; ++i) {
        bool maybe;
        if (DT == EQ_F16) {
          // the maximum of the chunk's values and the bound differs from the bound exactly when a
          // value lies above it (a bound of -0 with a value of +0 flags a chunk needlessly: harmless)
          const uint32_t mx = pk_max3_f16(pk_max3_f16(cand_hi[r], v[r][i].x, v[r][i].y), v[r][i].z, v[r][i].w);
          const uint32_t mn = pk_min3_f16(pk_min3_f16(cand_lo[r], v[r][i].x, v[r][i].y), v[r][i].z, v[r][i].w);
          maybe = ((mx ^ cand_hi[r]) | (mn ^ cand_lo[r])) != 0u;
        } else {
          float x[8];
          chunk_floats<DT>(v[r][i], x);
          float dmax = 0.0f;
#pragma unroll
          for (int k = 0; k < 8; ++k) dmax = fmaxf(dmax, fabsf(x[k] - mu_f[r]));
          maybe = dmax >= thr_lo[r];
        }
        const uint32_t ch = chunk_of<NT, WM>(i, part_c0);
        if (r < nrows && ch < part_c1 && maybe) cand |= 1u << (r * K + i);
      }
    }
  }

  // ---- candidates: decide their elements, leave the mask byte, notice borderline elements ----
  // The lanes that found candidates found different numbers of them, so the chunks are first queued
  // (row << 16 | chunk, in lane order) and then dealt out evenly, one per lane and pass over the
  // queue.  A wavefront with more candidates than the queue holds lets every lane work through its own.
  {
    auto body = [&](uint32_t r, uint32_t ch) {
      const uint4 c = *reinterpret_cast<const uint4*>(pool + Layout::off(ch0 + r * nchunks + ch));
      const float4 f = sc->fast[r];         // mean, lower and upper end of the band
      float x[8];
      chunk_floats<DT>(c, x);
      uint32_t m_lo = 0, m_hi = 0;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float d = fabsf(x[k] - f.x);
        m_lo |= (d >= f.y ? 1u : 0u) << k;
        m_hi |= (d >= f.z ? 1u : 0u) << k;
      }
      if (m_lo != m_hi) sc->slow[r] = 1u;   // an element inside the band: the row is redone exactly
      if (m_hi) mb[Layout::mask_off(ch0 + r * nchunks + ch)] = (unsigned char)m_hi;
    };
    const uint32_t mine = (uint32_t)__popc(cand);
    const uint32_t upto = wave_scan_inclusive(mine);
    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)upto, kWave - 1);
    if (total <= (uint32_t)kQueue) {
      uint32_t todo = cand, k = upto - mine;
      while (todo) {
        const int slot = __ffs((int)todo) - 1;
        todo &= todo - 1;
        const int r = slot / K, i = slot - r * K;
        sc->queue[wave][k++] = ((uint32_t)r << 16) | chunk_of<NT, WM>(i, part_c0);
      }
      __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
      __builtin_amdgcn_wave_barrier();
      for (uint32_t e = lane; e < total; e += kWave) {
        const uint32_t id = sc->queue[wave][e];
        body(id >> 16, id & 0xFFFFu);
      }
    } else {
      uint32_t todo = cand;
      while (__any(todo != 0)) {
        if (todo) {
          const int slot = __ffs((int)todo) - 1;
          todo &= todo - 1;
          const int r = slot / K, i = slot - r * K;
          body((uint32_t)r, chunk_of<NT, WM>(i, part_c0));
        }
      }
    }
  }
  // Interleaved chunks: the mask bytes of a unit come from several wavefronts, so all meet here.
  // Wavefront-major: a unit's bytes were written by its own wavefront, which can go on counting.
  if (!WM) __syncthreads();

  // ---- exact statistics and masks of the rows that asked for them ----
  // (a rare path: its loops over the thread's chunks stay rolled, which keeps its registers few)
  auto exact_redo = [&] {
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      if (r < nrows && sc->slow[r]) {
        double mu, sigma;
        if (kp.scope == EQ_STAT_MATRIX) {
          mu = md.mat_stats[0];
          sigma = md.mat_stats[1];
        } else {
          double s = 0.0;
#pragma unroll 1
          for (int i = 0; i < K; ++i) {
            const uint32_t ch = chunk_of<NT, WM>(i, part_c0);
            if (ch < part_c1) {
              float x[8];
              chunk_floats<DT>(*reinterpret_cast<const uint4*>(pool + Layout::off(ch0 + (uint32_t)r * nchunks + ch)), x);
#pragma unroll
              for (int k = 0; k < 8; ++k) s += (double)x[k];
            }
          }
          mu = block_sum(s, sc->dred) / cnt;
          double q = 0.0;
#pragma unroll 1
          for (int i = 0; i < K; ++i) {
            const uint32_t ch = chunk_of<NT, WM>(i, part_c0);
            if (ch < part_c1) {
              float x[8];
              chunk_floats<DT>(*reinterpret_cast<const uint4*>(pool + Layout::off(ch0 + (uint32_t)r * nchunks + ch)), x);
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
        // a row that took the exact path from the start (no chunk test was made): every chunk of the
        // thread; a row with an element inside the band: its candidate chunks anew (every other chunk
        // lies strictly inside the band's lower end, where the fast and the exact decision agree).
        // A constant scope has no outliers.
        uint32_t todo = (cand >> (r * K)) & ((1u << K) - 1u);
        if ((slow_rows >> r) & 1u) {
          todo = 0;
#pragma unroll
          for (int i = 0; i < K; ++i) todo |= chunk_of<NT, WM>(i, part_c0) < part_c1 ? 1u << i : 0u;
        }
        while (todo) {
          const int i = __ffs((int)todo) - 1;
          todo &= todo - 1;
          const uint32_t at = ch0 + (uint32_t)r * nchunks + chunk_of<NT, WM>(i, part_c0);
          const uint32_t mm = sigma > 0.0 ? chunk_mask<DT>(*reinterpret_cast<const uint4*>(pool + Layout::off(at)), mu, thr) : 0u;
          mb[Layout::mask_off(at)] = (unsigned char)mm;
        }
      }
    }
  };

  // ---- per unit: count ----
  // Interleaved: thread t takes the units [t q, (t + 1) q) of the batch (q = 1 unless the batch holds
  // more units than the workgroup has threads).  Wavefront-major: lane l takes unit l of its
  // wavefront's part.  Prefix sums over lanes, then over wavefronts.
  const uint32_t q = WM ? 1u : (nslots + NT - 1) / NT;
  const uint32_t s_first = WM ? min((part_c0 >> 4) + lane, part_c1 >> 4) : min(tid * q, nslots);
  const uint32_t s_last = WM ? min(s_first + 1u, part_c1 >> 4) : min(s_first + q, nslots);
  uint32_t mycnt, inc, before, total;
  auto count_units = [&] {
    mycnt = 0;
    for (uint32_t s = s_first; s < s_last; ++s) {
      const uint4 m = *reinterpret_cast<const uint4*>(mb + Layout::mask_off(ch0 + (s << 4)));
      mycnt += (uint32_t)(__popc(m.x) + __popc(m.y) + __popc(m.z) + __popc(m.w));
    }
    inc = wave_scan_inclusive(mycnt);
    before = 0;
    total = (uint32_t)__builtin_amdgcn_readlane((int)inc, kWave - 1);
    if (NW > 1) {
      if (lane == kWave - 1) sc->wtot[wave] = inc;
      __syncthreads();                                     // also publishes the rows' exact-path flags
      total = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const uint32_t t = sc->wtot[w];
        before += (uint32_t)w < wave ? t : 0u;
        total += t;
      }
    }
  };
  count_units();
  {
    bool any_slow = false;                                 // uniform over the workgroup
#pragma unroll
    for (int r = 0; r < RB; ++r) any_slow = any_slow || (r < nrows && sc->slow[r]);
    if (any_slow) {
      exact_redo();
      __syncthreads();
      count_units();
    }
  }
  {
    uint32_t run = before + inc - mycnt;                   // outliers of the batch in front of this thread's units
    for (uint32_t s = s_first; s < s_last; ++s) {
      sc->pre[s] = run;
      if (q > 1) {
        const uint4 m = *reinterpret_cast<const uint4*>(mb + Layout::mask_off(ch0 + (s << 4)));
        run += (uint32_t)(__popc(m.x) + __popc(m.y) + __popc(m.z) + __popc(m.w));
      }
    }
  }

  // ---- one reservation for the batch ----
  // Thread 0 issues the atomic, the caller's hook runs (the T = 0 kernel starts the loads of its
  // next batch there: v is dead by now, and loads issued after the atomic do not delay its
  // return, which is awaited by count), then thread 0 publishes the run's start.
  unsigned long long b = 0;
  if (tid == 0) {
    sc->pre[nslots] = total;
    if (WRITE && total) b = global_atomic_add(md.cursor, (unsigned long long)total);
  }
  after_reservation_issued();
  if (tid == 0) sc->base = b;            // nothing but this LDS store after the first use of b (each global
                                         // store in between would move the count that the wait is expressed in)
  __syncthreads();
  b = sc->base;
  // a row fits if its last entry does: rows come in order, so everything in front of it fits as well
  if (WRITE && tid < (uint32_t)nrows) {
    const uint32_t c0 = sc->pre[tid * upr], c1 = sc->pre[(tid + 1u) * upr];
    const bool fits = b + c1 <= (unsigned long long)md.capacity;
    md.row_count[row0 + tid] = c1 - c0;
    md.row_stage[row0 + tid] = fits ? (uint32_t)(b + c0) : 0xFFFFFFFFu;
    if (!fits) global_atomic_or(md.status, EQ_S_OUTLIER_OVERFLOW);
  }

  // ---- per unit: write (column, raw value) in ascending order, put 0 in the pool ----
  for (uint32_t s = s_first; s < s_last; ++s) {
    const uint4 m = *reinterpret_cast<const uint4*>(mb + Layout::mask_off(ch0 + (s << 4)));
    if ((m.x | m.y | m.z | m.w) == 0u) continue;
    // (floor(s / upr) as a multiply-high: exact for s < 2^20, 2 <= upr <= 4096; no division sequence)
    const uint32_t r = RB == 1 ? 0u : upr == 1u ? s : __umulhi(s, 0xFFFFFFFFu / upr + 1u);   // row of the batch,
    const uint32_t u = s - r * upr;                                                           // unit of the row
    const bool fits = WRITE && b + sc->pre[(r + 1u) * upr] <= (unsigned long long)md.capacity;
    unsigned long long pos = b + sc->pre[s];
    const uint32_t words[4] = {m.x, m.y, m.z, m.w};
#pragma unroll
    for (int wi = 0; wi < 4; ++wi) {
      uint32_t bits = words[wi];                           // 4 chunks of 8 elements
      while (bits) {
        const uint32_t bit = (uint32_t)__ffs((int)bits) - 1u;
        bits &= bits - 1u;
        const uint32_t chunk = 4u * (uint32_t)wi + (bit >> 3), j = bit & 7u;
        unsigned short* e = reinterpret_cast<unsigned short*>(pool + Layout::off(ch0 + (s << 4) + chunk)) + j;
        if (fits) {
          md.st_col[pos] = (u << 7) + (chunk << 3) + j;
          md.st_val[pos] = *e;
        }
        ++pos;
        *e = 0;
      }
    }
  }
  if (!WM) __syncthreads();              // wavefront-major: the units a wavefront goes on with are its own
}

template <int DT, int NT, int RB, int K, class Layout>
__device__ __forceinline__ void stage_rows_batch(const MatDesc& md, const KParams& kp, int64_t row0, int nrows,
                                                 unsigned char* pool, uint32_t ch0, unsigned char* mask_area,
                                                 BatchScratch<RB, NT / kWave>* sc) {
  uint4 v[RB][K];
  batch_issue_loads<NT, RB, K>(md, row0, nrows, v);     // every load of the batch in flight
  stage_loaded_rows<DT, NT, RB, K, Layout>(md, kp, row0, nrows, pool, ch0, mask_area, sc, v, [] {});
}

}  // namespace eq
