// Small kernels around the main pass: state reset, the CSR finish of the outlier list,
// whole-matrix statistics, and the dequantizer of Eq. 4.
#pragma once

#include "eq_common.h"
#include "eq_rowbatch.h"

namespace eq {

// Reset of the per-matrix cursor and status word (a kernel: the descriptors that hold the
// addresses live in device memory).
__global__ void reset_state(const MatDesc* __restrict__ mats, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  *mats[i].cursor = 0ull;
  *mats[i].status = 0;
  if (mats[i].rows == 0 || mats[i].cols == 0) {
    for (int r = 0; r <= mats[i].rows; ++r) mats[i].out_row_ptr[r] = 0u;
  }
}

// out_row_ptr = exclusive prefix sum of the per-row outlier counts.  One workgroup per matrix.
// `ids` (may be null): the matrices this launch looks after, one per workgroup.
__global__ __launch_bounds__(kThreads) void scan_row_counts(const MatDesc* __restrict__ mats, const int32_t* __restrict__ ids) {
  __shared__ uint32_t wtot[kWaves];
  const MatDesc md = mats[ids ? ids[blockIdx.x] : (int32_t)blockIdx.x];
  if (md.cols == 0) return;
  const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  uint32_t running = 0;
  for (int32_t r0 = 0; r0 < md.rows; r0 += kThreads) {
    const int32_t r = r0 + (int32_t)threadIdx.x;
    const uint32_t c = r < md.rows ? md.row_count[r] : 0u;
    uint32_t inc = c;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const uint32_t t = __shfl_up(inc, o);
      if (lane >= (uint32_t)o) inc += t;
    }
    if (lane == kWave - 1) wtot[wave] = inc;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t t = wtot[w];
      if ((uint32_t)w < wave) before += t;
      total += t;
    }
    if (r < md.rows) md.out_row_ptr[r] = running + before + (inc - c);
    running += total;
    __syncthreads();
  }
  if (threadIdx.x == 0) md.out_row_ptr[md.rows] = running;
}

// Moves each row's staged run to its CSR position.  Every producer writes a row's run in ascending
// column order already (the batched staging per unit, the general kernel per chunk), so this is a
// plain copy: one wavefront takes kMoveRows consecutive rows, reads their bookkeeping with one lane
// per row, and copies the runs with all loads of a row group in flight (rows of more than 64
// entries take further passes).
constexpr int kMoveRows = 16;

__global__ __launch_bounds__(kThreads) void move_outliers(const MatDesc* __restrict__ mats, const int32_t* __restrict__ ids) {
  const MatDesc md = mats[ids ? ids[blockIdx.y] : (int32_t)blockIdx.y];
  const int64_t row0 = ((int64_t)blockIdx.x * kWaves + threadIdx.x / kWave) * kMoveRows;
  if (row0 >= md.rows || md.cols == 0) return;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  // lane r: bookkeeping of row row0 + r
  uint32_t cnt_l = 0, src_l = 0, dst_l = 0;
  if (lane < (uint32_t)kMoveRows && row0 + lane < md.rows) {
    cnt_l = md.row_count[row0 + lane];
    src_l = md.row_stage[row0 + lane];
    dst_l = md.out_row_ptr[row0 + lane];
    // a row that was not staged, or whose run does not fit the output arrays, is left out
    if (src_l == 0xFFFFFFFFu || (unsigned long long)dst_l + cnt_l > (unsigned long long)md.capacity) cnt_l = 0;
  }
  constexpr int kGroup = 4;                                // rows whose loads are in flight together
#pragma unroll
  for (int g = 0; g < kMoveRows; g += kGroup) {
    uint32_t cnt[kGroup], src[kGroup], dst[kGroup], col[kGroup];
    uint16_t val[kGroup];
#pragma unroll
    for (int r = 0; r < kGroup; ++r) {
      cnt[r] = (uint32_t)__builtin_amdgcn_readlane((int)cnt_l, g + r);
      src[r] = (uint32_t)__builtin_amdgcn_readlane((int)src_l, g + r);
      dst[r] = (uint32_t)__builtin_amdgcn_readlane((int)dst_l, g + r);
      col[r] = 0;
      val[r] = 0;
      if (lane < cnt[r]) {
        col[r] = md.st_col[src[r] + lane];
        val[r] = md.st_val[src[r] + lane];
      }
    }
#pragma unroll
    for (int r = 0; r < kGroup; ++r) {
      if (lane < cnt[r]) {
        md.out_col[dst[r] + lane] = col[r];
        md.out_val[dst[r] + lane] = val[r];
      }
      for (uint32_t e = lane + kWave; e < cnt[r]; e += kWave) {        // long runs (uniform trip count)
        md.out_col[dst[r] + e] = md.st_col[src[r] + e];
        md.out_val[dst[r] + e] = md.st_val[src[r] + e];
      }
    }
  }
}

// ---- whole-matrix statistics (Eq. 3 as printed: mean and sigma of W) ---------------------
// Pass 1: per-workgroup partial sums of x; pass 2: of (x - mean)^2; a one-workgroup finish
// after each.  Partials are combined in a fixed order, so the result does not depend on timing.
template <int DT>
__global__ __launch_bounds__(kThreads) void matrix_partial_sums(const MatDesc* __restrict__ mats, int pass) {
  __shared__ double red[kWaves];
  const MatDesc md = mats[blockIdx.y];
  if (md.rows == 0 || md.cols == 0) return;
  const double mu = pass ? md.mat_stats[0] : 0.0;
  const uint32_t nchunks = (uint32_t)md.cols >> 3;
  double s = 0.0;
  for (int64_t row = blockIdx.x; row < md.rows; row += gridDim.x) {
    const EQ_GLOBAL uint16_t* src = md.W + row * md.ld;
    for (uint32_t ch = threadIdx.x; ch < nchunks; ch += kThreads) {
      const uint4 v = global_load128(src + 8 * (size_t)ch);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const double d = (double)widen16<DT>((w[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu) - mu;
        s += pass ? d * d : d;
      }
    }
  }
  s = block_sum(s, red);
  if (threadIdx.x == 0) md.mat_partial[blockIdx.x] = s;
}

__global__ __launch_bounds__(kThreads) void matrix_finish_sums(const MatDesc* __restrict__ mats, int pass, int nparts) {
  __shared__ double red[kWaves];
  const MatDesc md = mats[blockIdx.x];
  if (md.rows == 0 || md.cols == 0) return;
  double s = 0.0;
  for (int i = threadIdx.x; i < nparts; i += kThreads) s += md.mat_partial[i];
  s = block_sum(s, red);
  if (threadIdx.x == 0) {
    const double cnt = (double)md.rows * (double)md.cols;
    md.mat_stats[pass] = pass ? sqrt(s / cnt) : s / cnt;
  }
}

// ---- Eq. 4 ---------------------------------------------------------------------------
struct DeqDesc {
  const EQ_GLOBAL uint32_t* codes;
  const EQ_GLOBAL float* scales;
  const EQ_GLOBAL uint8_t* zps;
  const EQ_GLOBAL uint32_t* out_row_ptr;
  const EQ_GLOBAL uint32_t* out_col;      // null: no outlier list
  const EQ_GLOBAL uint16_t* out_val;
  EQ_GLOBAL uint16_t* W;
  int64_t ld;
  int32_t rows, cols, upr, G, words_per_row, bits;
};

// Eq. 4 for one chunk of 8 consecutive elements of a row: scale * (code - zero_point), outliers
// included (their slot holds the zero level, so they come out as 0).  8 codes are `bits` whole
// bytes of the row's bit stream, which sit in at most three aligned words (the row is padded to
// whole words).
template <int DT>
__device__ __forceinline__ uint4 dequantize_chunk(const DeqDesc& d, int64_t row, uint32_t ch) {
  const uint32_t byte0 = ch * (uint32_t)d.bits;
  const EQ_GLOBAL uint32_t* wp = d.codes + row * (int64_t)d.words_per_row + (byte0 >> 2);
  const uint32_t last_word = (uint32_t)d.words_per_row - 1u;
  const uint32_t w0 = wp[0];
  const uint32_t w1 = (byte0 >> 2) + 1u <= last_word ? wp[1] : 0u;
  const uint32_t w2 = (byte0 >> 2) + 2u <= last_word ? wp[2] : 0u;
  const uint32_t sh = (byte0 & 3u) * 8u;
  unsigned long long lo = ((unsigned long long)w1 << 32) | w0;
  unsigned long long acc = sh ? (lo >> sh) | ((unsigned long long)w2 << (64u - sh)) : lo;
  const int64_t unit = row * (int64_t)d.upr + (ch * 8u) / (uint32_t)d.G;
  const float s = d.scales[unit];
  const int z = (int)d.zps[unit];
  const uint32_t mask = (1u << d.bits) - 1u;
  uint32_t h[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const uint32_t u = (uint32_t)acc & mask;
    acc >>= d.bits;
    float prod = s * (float)((int)u - z);
    // Eq. 4 is evaluated as a binary32 product that is then rounded to the 16-bit type.  The
    // empty asm keeps the compiler from fusing both into one rounding (v_fma_mixlo_f16).
    asm volatile("" : "+v"(prod));
    h[k] = narrow16<DT>(prod);
  }
  return make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
}

// Byte N of a word as binary32 (v_cvt_f32_ubyteN; written out because the compiler, knowing that
// only four bits of each byte can be set, otherwise takes a bit-field extract and a convert).
template <int N>
__device__ __forceinline__ float byte_to_float(uint32_t w) {
  float f;
  if (N == 0) asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(f) : "v"(w));
  else if (N == 1) asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(f) : "v"(w));
  else if (N == 2) asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(f) : "v"(w));
  else asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(f) : "v"(w));
  return f;
}

// The same for 4-bit codes, from the chunk's one code word: nibbles to bytes, bytes to binary32,
// then exactly the arithmetic above (subtract the zero-point, one binary32 product, one rounding
// to the 16-bit type).
template <int DT>
__device__ __forceinline__ uint4 dequantize_chunk4(uint32_t w, float s, float zf) {
  const uint32_t even = w & 0x0F0F0F0Fu, odd = (w >> 4) & 0x0F0F0F0Fu;      // elements 0 2 4 6 / 1 3 5 7
  const float u[8] = {byte_to_float<0>(even), byte_to_float<0>(odd), byte_to_float<1>(even), byte_to_float<1>(odd),
                      byte_to_float<2>(even), byte_to_float<2>(odd), byte_to_float<3>(even), byte_to_float<3>(odd)};
  uint32_t h[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    float prod = s * (u[k] - zf);
    asm volatile("" : "+v"(prod));      // two roundings, as in dequantize_chunk
    h[k] = narrow16<DT>(prod);
  }
  return make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
}

constexpr int kDeqChunks = 4;      // chunks per thread and segment: a segment is 4 * 256 * 8 = 8192 columns

// Eq. 4, dense and sparse part in one pass over the output: one workgroup per row walks the
// row in segments.  A segment's dense results go to LDS, the row's outliers that fall into
// the segment (the list is sorted by column, so they are the next entries of the row's run)
// overwrite their 16-bit slots there, and the segment leaves with coalesced 128-bit stores.
// Each output byte is written to HBM once; there is no read-modify-write of cache lines.
// Without an outlier list the results go straight from registers to HBM.
// FOUR: 4-bit codes, one code word per chunk, all of a segment's words in flight together.
template <int DT, bool FOUR>
__global__ __launch_bounds__(kThreads) void dequantize_rows(DeqDesc d) {
  __shared__ uint4 seg[kDeqChunks * kThreads];
  const int64_t row = blockIdx.x;
  const uint32_t tid = threadIdx.x;
  const uint32_t nchunks = (uint32_t)d.cols >> 3;
  const bool sparse = d.out_col != nullptr;
  uint32_t next = 0, end = 0;                  // the row's outliers not yet written
  if (sparse) {
    next = d.out_row_ptr[row];
    end = d.out_row_ptr[row + 1];
  }
  const bool per_row = d.upr == 1;
  float s_row = 0.0f, z_row = 0.0f;
  if (FOUR && per_row) {
    s_row = d.scales[row];
    z_row = (float)d.zps[row];
  }
  const BufferRsrc crow = make_buffer(d.codes + row * (int64_t)d.words_per_row, FOUR ? (uint32_t)d.words_per_row * 4u : 0u);
  EQ_GLOBAL uint16_t* orow = d.W + row * d.ld;
  for (uint32_t ch0 = 0; ch0 < nchunks; ch0 += kDeqChunks * kThreads) {
    // the next entries of the row's list, loaded ahead of the dense work
    const uint32_t i_first = next + tid;
    uint32_t col_first = 0xFFFFFFFFu;
    uint16_t val_first = 0;
    if (sparse && i_first < end) {
      col_first = d.out_col[i_first];
      val_first = d.out_val[i_first];
    }
    uint4 res[kDeqChunks];
    if (FOUR) {
      uint32_t wq[kDeqChunks];
#pragma unroll
      for (int j = 0; j < kDeqChunks; ++j) wq[j] = buffer_load32(crow, (ch0 + (uint32_t)j * kThreads + tid) * 4u);
#pragma unroll
      for (int j = 0; j < kDeqChunks; ++j) {
        float s = s_row, zf = z_row;
        if (!per_row) {                          // uniform
          const uint32_t ch = min(ch0 + (uint32_t)j * kThreads + tid, nchunks - 1u);
          const int64_t unit = row * (int64_t)d.upr + (ch * 8u) / (uint32_t)d.G;
          s = d.scales[unit];
          zf = (float)d.zps[unit];
        }
        res[j] = dequantize_chunk4<DT>(wq[j], s, zf);
      }
    } else {
#pragma unroll
      for (int j = 0; j < kDeqChunks; ++j) {
        const uint32_t ch = ch0 + (uint32_t)j * kThreads + tid;
        res[j] = ch < nchunks ? dequantize_chunk<DT>(d, row, ch) : make_uint4(0, 0, 0, 0);
      }
    }
    if (sparse) {                                // uniform
#pragma unroll
      for (int j = 0; j < kDeqChunks; ++j) seg[j * kThreads + tid] = res[j];
      const uint32_t col0 = ch0 * 8u, col1 = min(col0 + kDeqChunks * kThreads * 8u, (uint32_t)d.cols);
      uint32_t taken;
      bool first = true;
      do {                                       // uniform: every thread sees the same counts
        __syncthreads();                         // dense results (or the previous patches) are in place
        uint32_t col = col_first;
        uint16_t val = val_first;
        if (!first) {
          const uint32_t i = next + tid;
          col = 0xFFFFFFFFu;
          if (i < end) {
            col = d.out_col[i];
            val = d.out_val[i];
          }
        }
        first = false;
        const bool mine = col >= col0 && col < col1;
        if (mine) reinterpret_cast<uint16_t*>(seg)[col - col0] = val;
        taken = (uint32_t)__syncthreads_count(mine);
        next += taken;
      } while (taken == (uint32_t)kThreads);     // all of this batch fell into the segment: there may be more
#pragma unroll
      for (int j = 0; j < kDeqChunks; ++j) res[j] = seg[j * kThreads + tid];   // the entries this thread wrote itself
    }
#pragma unroll
    for (int j = 0; j < kDeqChunks; ++j) {
      const uint32_t ch = ch0 + (uint32_t)j * kThreads + tid;
      if (ch < nchunks) global_store_stream128(orow + 8 * (size_t)ch, res[j]);
    }
  }
}

// ---- Eq. 4 fused with a matrix-vector product ----------------------------------------------
// y = W^ x for the reconstruction W^ of Eq. 4 (every element rounded to the 16-bit type exactly
// as dequantize_rows writes it), without W^ ever reaching HBM: the kernel reads bits/8 bytes per
// weight instead of 2.  A workgroup takes kMvRows consecutive rows; a thread keeps its chunks
// of x in registers for all of them, products and sums are binary32.  An outlier's slot holds
// the zero level, so the dense part contributes 0 there and the row's sparse list is added on
// top as val * x[col].
constexpr int kMvRows = 8;
constexpr int kMvChunks = 2;

template <int DT>
__device__ __forceinline__ float dot8(const uint4 w, const uint4 x, float acc) {
  const uint32_t a[4] = {w.x, w.y, w.z, w.w}, b[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    // one packed dot-product instruction per pair, accumulating in binary32 (both formats)
    if (DT == EQ_F16) {
      typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
      acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a[k]), __builtin_bit_cast(half2_t, b[k]), acc, false);
    } else {
      typedef __bf16 bfloat2_t __attribute__((ext_vector_type(2)));
      acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bfloat2_t, a[k]), __builtin_bit_cast(bfloat2_t, b[k]), acc, false);
    }
  }
  return acc;
}

// MODE 0: any code width (dequantize_chunk).  MODE 1: 4-bit codes, one code word per chunk
// (dequantize_chunk4).  MODE 2: 4-bit codes and one range per row (rows whose length is not a
// multiple of 32; the others take dequant_matvec_rows4 below): the 16 values a weight of a row
// can take, fl16(fl32(s (u - z))) for u = 0..15, are tabulated in LDS once and every weight is
// one 16-bit LDS read (two address instructions) instead of five arithmetic instructions.
// MODE 3: 4-bit codes with groups of 128 or more elements that tile the 4096-column segments (or
// are tiled by them): the same tables per (row, group) of a segment, at most 256 of them, built
// by one thread each while the segment's loads are in flight, double-buffered so that one barrier
// per segment suffices; scale and zero-point of the next segment's tables are loaded a segment
// ahead.  MODE 4: the same for groups of 64 elements, two tables per thread.  The host checks the
// group size (eq_dequant_matvec).
template <int DT, int MODE>
__global__ __launch_bounds__(kThreads) void dequant_matvec(DeqDesc d, const EQ_GLOBAL uint16_t* __restrict__ x,
                                                            EQ_GLOBAL float* __restrict__ y) {
  constexpr bool FOUR = MODE != 0;
  constexpr bool TABLES = MODE == 3 || MODE == 4;        // tables per (row, group) of a segment
  constexpr int TPT = MODE == 4 ? 2 : 1;                 // tables built per thread and segment
  __shared__ float red[kMvRows][kWaves];
  __shared__ uint16_t lut[kMvRows][16];
  __shared__ __align__(16) uint16_t lut3[TABLES ? 2 : 1][TABLES ? TPT * kThreads : 1][16];
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int64_t row0 = (int64_t)blockIdx.x * kMvRows;
  const int nrows = (int)min((int64_t)kMvRows, (int64_t)d.rows - row0);
  const uint32_t nchunks = (uint32_t)d.cols >> 3;
  const bool per_row = d.upr == 1;
  uint32_t rp[kMvRows + 1];                              // the rows' sparse ranges (loaded early, used last)
#pragma unroll
  for (int r = 0; r <= kMvRows; ++r) rp[r] = d.out_col ? d.out_row_ptr[row0 + min(r, nrows)] : 0u;   // absent rows: empty
  float acc[kMvRows], srow[kMvRows], zrow[kMvRows];
#pragma unroll
  for (int r = 0; r < kMvRows; ++r) {
    acc[r] = 0.0f;
    srow[r] = 0.0f;
    zrow[r] = 0.0f;
    if (MODE == 1 && per_row && r < nrows) {
      srow[r] = d.scales[row0 + r];
      zrow[r] = (float)d.zps[row0 + r];
    }
  }
  if (MODE == 2) {
    if (tid < (uint32_t)(kMvRows * 16)) {
      const int r = (int)(tid >> 4), u = (int)(tid & 15u);
      const int64_t row = row0 + (r < nrows ? r : 0);
      float prod = d.scales[row] * ((float)u - (float)d.zps[row]);
      asm volatile("" : "+v"(prod));      // two roundings, as in dequantize_chunk
      lut[r][u] = (uint16_t)narrow16<DT>(prod);
    }
    __syncthreads();
  }
  // range-checked views of the rows' code words: chunks past the end of a row and rows past the
  // end of the matrix read as zero words without touching memory (their x chunk is zero too)
  BufferRsrc crow[kMvRows];
#pragma unroll
  for (int r = 0; r < kMvRows; ++r)
    crow[r] = make_buffer(d.codes + (r < nrows ? row0 + r : row0) * (int64_t)d.words_per_row,
                          FOUR && r < nrows ? (uint32_t)d.words_per_row * 4u : 0u);
  auto sparse_part = [&] {
    if (!d.out_col) return;
    // Every wavefront takes the sparse lists of two of the workgroup's rows, one contiguous stretch
    // of the CSR arrays, in a strided walk; an entry belongs to the first of the two rows if its
    // index lies below the second row's start.  (The rows' sums are combined over all threads at
    // the end anyway, so it does not matter which thread adds an entry.)
    static_assert(kMvRows == 2 * kWaves, "two rows per wavefront");
    const uint32_t w2 = 2u * (uint32_t)__builtin_amdgcn_readfirstlane((int)wave);
    uint32_t b = 0, m = 0, e = 0;
#pragma unroll
    for (int r = 0; r <= kMvRows; ++r) {
      if ((uint32_t)r == w2) b = rp[r];
      if ((uint32_t)r == w2 + 1u) m = rp[r];
      if ((uint32_t)r == w2 + 2u) e = rp[r];
    }
    float sa = 0.0f, sb = 0.0f;
    constexpr int kAhead = 4;                            // entries per thread in flight (two dependent loads each)
    for (uint32_t i0 = b + lane; i0 < e; i0 += kAhead * kWave) {
      uint32_t col[kAhead];
      float val[kAhead], xg[kAhead];
#pragma unroll
      for (int a = 0; a < kAhead; ++a) {
        const uint32_t i = i0 + (uint32_t)a * kWave;
        col[a] = i < e ? d.out_col[i] : 0xFFFFFFFFu;
        val[a] = i < e ? widen16<DT>(d.out_val[i]) : 0.0f;
      }
#pragma unroll
      for (int a = 0; a < kAhead; ++a) xg[a] = col[a] < (uint32_t)d.cols ? widen16<DT>(x[col[a]]) : 0.0f;
#pragma unroll
      for (int a = 0; a < kAhead; ++a) {
        const uint32_t i = i0 + (uint32_t)a * kWave;
        const float prod = val[a] * xg[a];
        sa += i < m ? prod : 0.0f;
        sb += i < m ? 0.0f : prod;
      }
    }
#pragma unroll
    for (int r = 0; r < kMvRows; ++r) acc[r] += (uint32_t)r == w2 ? sa : ((uint32_t)r == w2 + 1u ? sb : 0.0f);
  };
  // MODE 3 / 4: tables per (row, group) of a segment.  gps = groups per segment (1 when a group spans
  // whole segments); table t < kMvRows * gps is that of row t / gps, group t % gps; thread tid builds
  // tables tid, tid + 256, ...
  constexpr uint32_t kSegCols = kMvChunks * kThreads * 8u;
  const uint32_t lg = (uint32_t)__ffs(d.G) - 1u;                       // with tables the group size is a power of two
  const uint32_t gps = TABLES ? ((uint32_t)d.G >= kSegCols ? 1u : kSegCols >> lg) : 1u;
  uint32_t tab_of[kMvChunks];                              // which of a row's tables serves chunk j of this thread
#pragma unroll
  for (int j = 0; j < kMvChunks; ++j) tab_of[j] = gps == 1u ? 0u : (((uint32_t)j * kThreads + tid) * 8u) >> lg;
  float s_tab[TPT], z_tab[TPT];                            // scale and zero-point of this thread's next tables
  auto load_table_params = [&](uint32_t ch0n) {
#pragma unroll
    for (int k = 0; k < TPT; ++k) {
      const uint32_t t = tid + (uint32_t)k * kThreads;
      const uint32_t t_row = t / gps, t_grp = t - t_row * gps;
      const uint32_t col = ch0n * 8u + (gps == 1u ? 0u : t_grp << lg);
      s_tab[k] = 0.0f;                                     // a table nobody reads: zeros (finite)
      z_tab[k] = 0.0f;
      if (t_row < (uint32_t)nrows && t < (uint32_t)kMvRows * gps && col < (uint32_t)d.cols) {
        const int64_t unit = (row0 + t_row) * (int64_t)d.upr + (col >> lg);
        s_tab[k] = d.scales[unit];
        z_tab[k] = (float)d.zps[unit];
      }
    }
  };
#pragma unroll
  for (int k = 0; k < TPT; ++k) s_tab[k] = z_tab[k] = 0.0f;
  if (TABLES) load_table_params(0u);
  uint32_t buf = 0;
  for (uint32_t ch0 = 0; ch0 < nchunks; ch0 += kMvChunks * kThreads) {
    uint4 xv[kMvChunks];
#pragma unroll
    for (int j = 0; j < kMvChunks; ++j) {
      const uint32_t ch = ch0 + (uint32_t)j * kThreads + tid;
      xv[j] = ch < nchunks ? global_load128(x + 8 * (size_t)ch) : make_uint4(0, 0, 0, 0);
    }
    if (FOUR) {
      uint32_t wq[kMvRows][kMvChunks];                   // every code load of the segment in flight
#pragma unroll
      for (int r = 0; r < kMvRows; ++r)
#pragma unroll
        for (int j = 0; j < kMvChunks; ++j)
          wq[r][j] = buffer_load32(crow[r], (ch0 + (uint32_t)j * kThreads + tid) * 4u);
      if (TABLES) {
#pragma unroll
        for (int k = 0; k < TPT; ++k) {
          const uint32_t t = tid + (uint32_t)k * kThreads;
          if (t < (uint32_t)kMvRows * gps) {
            uint32_t h[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
              float prod = s_tab[k] * ((float)u - z_tab[k]);
              asm volatile("" : "+v"(prod));    // two roundings, as in dequantize_chunk
              h[u] = narrow16<DT>(prod);
            }
            uint4* dst = reinterpret_cast<uint4*>(&lut3[buf][t][0]);
            dst[0] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
            dst[1] = make_uint4(h[8] | (h[9] << 16), h[10] | (h[11] << 16), h[12] | (h[13] << 16), h[14] | (h[15] << 16));
          }
        }
        load_table_params(ch0 + kMvChunks * kThreads);     // for the next segment (past the end: no load)
        // the tables of this segment are complete; the other buffer, which the next segment
        // rewrites, was last read before this barrier
        __syncthreads();
      }
#pragma unroll
      for (int r = 0; r < kMvRows; ++r) {
#pragma unroll
        for (int j = 0; j < kMvChunks; ++j) {
          float s = srow[r], zf = zrow[r];
          if (MODE == 1 && !per_row) {                   // uniform
            const uint32_t ch = min(ch0 + (uint32_t)j * kThreads + tid, nchunks - 1u);
            const int64_t unit = (r < nrows ? row0 + r : row0) * (int64_t)d.upr + (ch * 8u) / (uint32_t)d.G;
            s = d.scales[unit];
            zf = (float)d.zps[unit];
          }
          uint4 wv;
          if (MODE == 2 || TABLES) {
            // byte offsets into the table, four at a time: even elements, odd elements
            const uint32_t w = wq[r][j];
            uint32_t ev = (w << 1) & 0x1E1E1E1Eu, od = (w >> 3) & 0x1E1E1E1Eu;
            asm("" : "+v"(ev), "+v"(od));     // keep the two words: a byte of them is one bit-field extract away
            const unsigned char* tab = MODE == 2 ? reinterpret_cast<const unsigned char*>(&lut[r][0])
                                                 : reinterpret_cast<const unsigned char*>(&lut3[buf][(uint32_t)r * gps + tab_of[j]][0]);
            typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
            uint32_t pr[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              ushort2_t h;
              h.x = *reinterpret_cast<const unsigned short*>(tab + ((ev >> (8 * k)) & 0xFFu));
              h.y = *reinterpret_cast<const unsigned short*>(tab + ((od >> (8 * k)) & 0xFFu));
              pr[k] = __builtin_bit_cast(uint32_t, h);
            }
            wv = make_uint4(pr[0], pr[1], pr[2], pr[3]);
          } else {
            wv = dequantize_chunk4<DT>(wq[r][j], s, zf);
          }
          acc[r] = dot8<DT>(wv, xv[j], acc[r]);
        }
      }
      buf ^= 1u;
    } else {
#pragma unroll
      for (int r = 0; r < kMvRows; ++r) {
        if (r < nrows) {                                 // uniform
#pragma unroll
          for (int j = 0; j < kMvChunks; ++j) {
            const uint32_t ch = ch0 + (uint32_t)j * kThreads + tid;
            if (ch < nchunks) acc[r] = dot8<DT>(dequantize_chunk<DT>(d, row0 + r, ch), xv[j], acc[r]);
          }
        }
      }
    }
  }
  sparse_part();
#pragma unroll
  for (int r = 0; r < kMvRows; ++r) {
    float v = acc[r];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if (lane == 0) red[r][wave] = v;
  }
  __syncthreads();
  if (tid < (uint32_t)nrows) {
    float t = red[tid][0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) t += red[tid][w];
    y[row0 + tid] = t;
  }
}

// ---- the same for the paper's own format: 4-bit codes, one range per row ---------------------
// (cols a multiple of 32).  A thread takes 32 consecutive columns of a segment of 8192: one
// 128-bit load of codes per row (a wavefront reads 1 KB of a row's stream at a time) and four
// chunks of x that serve all kMvRows rows of the workgroup.  Weights come from tables in LDS: the
// 16 values a weight of the row can take, fl16(fl32(s (u - z))), and from them the 256 PAIRS of
// values that a byte of the code stream (two neighbouring weights) can stand for, as packed words
// (1 KB per row).  LOOKUP selects how the four pairs of a code word are fetched: all from the table
// of pairs (one random 32-bit read per pair: few vector instructions, but 64 lanes spread over 256
// words collide in the LDS banks), all from the table of single values (two 16-bit reads that never
// collide, five vector instructions per pair), or two and two.
enum { kLookupPairs = 0, kLookupMixed = 1, kLookupSingles = 2 };
constexpr int kMvRowChunks = 4;          // chunks of 8 columns per thread and segment

template <int DT, int LOOKUP>
__global__ __launch_bounds__(kThreads) void dequant_matvec_rows4(DeqDesc d, const EQ_GLOBAL uint16_t* __restrict__ x,
                                                                  EQ_GLOBAL float* __restrict__ y) {
  __shared__ float red[kMvRows][kWaves];
  __shared__ __align__(16) uint16_t lut[kMvRows][16];
  __shared__ uint32_t lut_pair[kMvRows][256];
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int64_t row0 = (int64_t)blockIdx.x * kMvRows;
  const int nrows = (int)min((int64_t)kMvRows, (int64_t)d.rows - row0);
  const uint32_t nchunks = (uint32_t)d.cols >> 3;
  uint32_t rp[kMvRows + 1];                              // the rows' sparse ranges (loaded early, used last)
#pragma unroll
  for (int r = 0; r <= kMvRows; ++r) rp[r] = d.out_col ? d.out_row_ptr[row0 + min(r, nrows)] : 0u;   // absent rows: empty
  if (tid < (uint32_t)(kMvRows * 16)) {
    const int r = (int)(tid >> 4), u = (int)(tid & 15u);
    const int64_t row = row0 + (r < nrows ? r : 0);
    float prod = d.scales[row] * ((float)u - (float)d.zps[row]);
    asm volatile("" : "+v"(prod));        // two roundings, as in dequantize_chunk
    lut[r][u] = (uint16_t)narrow16<DT>(prod);
  }
  __syncthreads();
  static_assert(kThreads == 256, "one thread per byte value");
#pragma unroll
  for (int r = 0; r < kMvRows; ++r)        // low nibble = the even column (low half of the pair), high nibble = the odd one
    lut_pair[r][tid] = (uint32_t)lut[r][tid & 15u] | ((uint32_t)lut[r][tid >> 4] << 16);
  __syncthreads();
  // range-checked views of the rows' code words: words past the end of a row and rows past the
  // end of the matrix read as zero without touching memory (their x chunk is zero too)
  BufferRsrc crow[kMvRows];
#pragma unroll
  for (int r = 0; r < kMvRows; ++r)
    crow[r] = make_buffer(d.codes + (r < nrows ? row0 + r : row0) * (int64_t)d.words_per_row,
                          r < nrows ? (uint32_t)d.words_per_row * 4u : 0u);
  float acc[kMvRows];
#pragma unroll
  for (int r = 0; r < kMvRows; ++r) acc[r] = 0.0f;
  // ---- the rows' sparse lists: every wavefront takes those of two rows, one contiguous stretch of
  // the CSR arrays, in a strided walk (see dequant_matvec) ----
  auto sparse_part = [&] {
    if (!d.out_col) return;
    static_assert(kMvRows == 2 * kWaves, "two rows per wavefront");
    const uint32_t w2 = 2u * (uint32_t)__builtin_amdgcn_readfirstlane((int)wave);
    uint32_t b = 0, m = 0, e = 0;
#pragma unroll
    for (int r = 0; r <= kMvRows; ++r) {
      if ((uint32_t)r == w2) b = rp[r];
      if ((uint32_t)r == w2 + 1u) m = rp[r];
      if ((uint32_t)r == w2 + 2u) e = rp[r];
    }
    float sa = 0.0f, sb = 0.0f;
    constexpr int kAhead = 4;                            // entries per thread in flight (two dependent loads each)
    for (uint32_t i0 = b + lane; i0 < e; i0 += kAhead * kWave) {
      uint32_t col[kAhead];
      float val[kAhead], xg[kAhead];
#pragma unroll
      for (int a = 0; a < kAhead; ++a) {
        const uint32_t i = i0 + (uint32_t)a * kWave;
        col[a] = i < e ? d.out_col[i] : 0xFFFFFFFFu;
        val[a] = i < e ? widen16<DT>(d.out_val[i]) : 0.0f;
      }
#pragma unroll
      for (int a = 0; a < kAhead; ++a) xg[a] = col[a] < (uint32_t)d.cols ? widen16<DT>(x[col[a]]) : 0.0f;
#pragma unroll
      for (int a = 0; a < kAhead; ++a) {
        const uint32_t i = i0 + (uint32_t)a * kWave;
        const float prod = val[a] * xg[a];
        sa += i < m ? prod : 0.0f;
        sb += i < m ? 0.0f : prod;
      }
    }
#pragma unroll
    for (int r = 0; r < kMvRows; ++r) acc[r] += (uint32_t)r == w2 ? sa : ((uint32_t)r == w2 + 1u ? sb : 0.0f);
  };
  // The walk is a chain of dependent loads (entry, then x at its column) with little to do in
  // between.  Workgroups start together and would all reach it together at the end, with nothing
  // left to hide it behind: every other workgroup takes it first, under its neighbours' dense part.
  const bool sparse_first = (blockIdx.x & 1u) != 0u;
  if (sparse_first) sparse_part();
  // Rolling prefetch: a row's code words for the next segment are requested as soon as this
  // segment's have been used (same registers), and the next chunks of x at the top of the segment,
  // so that every wavefront has loads in flight while it computes (without this the wavefronts of a
  // SIMD fall into step: all wait for memory, then all compute).
  constexpr uint32_t kSeg = kMvRowChunks * kThreads;     // chunks per segment
  auto load_x = [&](uint32_t ch0, uint4 (&xv)[kMvRowChunks]) {
    const uint32_t c0 = ch0 + kMvRowChunks * tid;
#pragma unroll
    for (int j = 0; j < kMvRowChunks; ++j)
      xv[j] = c0 + (uint32_t)j < nchunks ? global_load128(x + 8 * (size_t)(c0 + j)) : make_uint4(0, 0, 0, 0);
  };
  uint4 xv[kMvRowChunks], xn[kMvRowChunks], wq[kMvRows];
  load_x(0u, xv);
#pragma unroll
  for (int r = 0; r < kMvRows; ++r) wq[r] = buffer_load_stream128(crow[r], kMvRowChunks * tid * 4u);
  for (uint32_t ch0 = 0; ch0 < nchunks; ch0 += kSeg) {
    const uint32_t c_next = ch0 + kSeg + kMvRowChunks * tid;   // this thread's first chunk (= code word) of the next segment
    load_x(ch0 + kSeg, xn);                                     // (past the end: zeros, no load)
#pragma unroll
    for (int r = 0; r < kMvRows; ++r) {
      const unsigned char* tab2 = reinterpret_cast<const unsigned char*>(&lut_pair[r][0]);
      const unsigned char* tab1 = reinterpret_cast<const unsigned char*>(&lut[r][0]);
      const uint32_t words[4] = {wq[r].x, wq[r].y, wq[r].z, wq[r].w};
      wq[r] = buffer_load_stream128(crow[r], c_next * 4u);     // beyond the row: zeros, no memory access
#pragma unroll
      for (int j = 0; j < kMvRowChunks; ++j) {
        const uint32_t w = words[j];
        typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
        uint32_t pr[4];
        constexpr int kFromPairs = LOOKUP == kLookupPairs ? 4 : LOOKUP == kLookupMixed ? 2 : 0;
#pragma unroll
        for (int k = 0; k < kFromPairs; ++k)
          pr[k] = *reinterpret_cast<const uint32_t*>(tab2 + (((w >> (8 * k)) & 0xFFu) << 2));
        if (kFromPairs < 4) {
          // byte offsets into the table of single values, four at a time: even elements, odd elements
          uint32_t ev = (w << 1) & 0x1E1E1E1Eu, od = (w >> 3) & 0x1E1E1E1Eu;
          asm("" : "+v"(ev), "+v"(od));       // keep the two words: a byte of them is one bit-field extract away
#pragma unroll
          for (int k = kFromPairs; k < 4; ++k) {
            ushort2_t h;
            h.x = *reinterpret_cast<const unsigned short*>(tab1 + ((ev >> (8 * k)) & 0xFFu));
            h.y = *reinterpret_cast<const unsigned short*>(tab1 + ((od >> (8 * k)) & 0xFFu));
            pr[k] = __builtin_bit_cast(uint32_t, h);
          }
        }
        acc[r] = dot8<DT>(make_uint4(pr[0], pr[1], pr[2], pr[3]), xv[j], acc[r]);
      }
    }
#pragma unroll
    for (int j = 0; j < kMvRowChunks; ++j) xv[j] = xn[j];
  }
  if (!sparse_first) sparse_part();
#pragma unroll
  for (int r = 0; r < kMvRows; ++r) {
    float v = acc[r];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if (lane == 0) red[r][wave] = v;
  }
  __syncthreads();
  if (tid < (uint32_t)nrows) {
    float t = red[tid][0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) t += red[tid][w];
    y[row0 + tid] = t;
  }
}


}  // namespace eq
