// One range per row (the paper's per-channel setting, Sec. 5) with the two sums of Eq. 2 taken from
// the row's SORTED normal values instead of from every element.
//
// The level of an element, rint(x / s) clamped to [clo, chi] (Eq. 1), never decreases with x.  In
// ascending order the elements with level <= l are therefore a prefix of the row, of length n_l,
// and with P[n] = x_(1) + ... + x_(n) (the n smallest values), summation by parts gives
//     A = sum c^2 = chi^2 N - sum_{l = clo}^{chi - 1} (2 l + 1) n_l
//     B = sum x c = chi P[N] - sum_{l = clo}^{chi - 1} P[n_l]
// over the 2^bits - 1 boundaries between neighbouring levels.  One optimisation step then costs a
// search for each n_l and one prefix sum apiece, whatever the row's length, instead of a visit of all
// N elements; n_l moves by a few positions per step, so the search starts where it ended last time.
// The sums are the same integers (A) and the same exactly representable binary64 values (B) as the
// direct evaluation gives, the scalar recurrence is the one of eq_common.h: same bits.
//
//   sorted_prepare : stages a row as every other kernel does (eq_rowbatch.h: statistics, outlier
//                    mask, outliers replaced by 0; nothing written to the outlier list here), then
//                    sorts the 16-bit values in LDS (counting sort into 4096 or 8192 value-linear buckets,
//                    ranks inside a bucket by counting) and writes a record per row to the
//                    workspace: header, then per chunk of 8 sorted values the values and the exact sum of
//                    everything in front of them.
//   sorted_iterate : 16 lanes per row, one per boundary, 4 rows per wavefront; Adam on the range
//                    (Algorithm 1, second step); leaves the chosen range of every row.
// The codes, scales, zero-points and the outlier list are then written by the kernel without
// optimisation steps (eq_rtn128.h), which takes the range it is given instead of the initial one.
//
// A row whose prefix sums might not be exact in binary64 (values spread over more than some 35 binary
// orders of magnitude), or whose values pile up in one bucket (hundreds of equal values), is
// evaluated element by element from its record instead, like the general kernel does.
#pragma once

#include "eq_fused128.h"

namespace eq {

constexpr int kSortThreads = 256;              // workgroup of sorted_prepare for rows of up to 8192 elements (512 or 1024 beyond)
// NB value-linear buckets (+2: zero has a bucket of its own): 4096 for rows of up to 8192 elements,
// 8192 beyond.  16-bit counters, two to a word (a row has at most 32768 elements).
constexpr int sort_counters(int nb) { return nb + 16; }
constexpr uint32_t kSortBigBucket = 512;       // a larger bucket (other than zero's) leaves the row unsorted
constexpr uint32_t kRecExactSums = 1u, kRecSorted = 2u;

struct SortScratch {
  double wsum[16];                             // (up to 1024 threads)
  uint32_t wcnt[16];
  uint32_t minnz_bits;                         // smallest non-zero |x| of the row (bit pattern)
  uint32_t big_bucket;
};

template <int NT>
constexpr size_t sort_header_bytes() {
  return (sizeof(BatchScratch<1, NT / kWave>) + sizeof(SortScratch) + 255u) & ~(size_t)255u;
}
// dynamic LDS of sorted_prepare for rows of `cols` elements: staging pool (reused for the sorted
// values), the values bucket by bucket, the bucket counters
inline size_t sort_prepare_lds(size_t header, int64_t cols, int nb) {
  return header + (size_t)(cols / 128) * kSlotBytes + (size_t)cols * 2 + (size_t)sort_counters(nb) * 2;
}

// Can every sum the sorted evaluation forms be exact in binary64?  All values are multiples of
// 2^ue (the unit in the last place of the smallest non-zero |x|) and smaller than 2^ea; the largest
// sum is below 32 N times that.
template <int DT>
__device__ __forceinline__ bool sorted_sums_exact(float amax, uint32_t minnz_bits, uint32_t cols) {
  if (!(amax > 0.0f)) return true;
  int ea = 0;
  (void)frexpf(amax, &ea);
  const int e = DT == EQ_F16 ? (int)(minnz_bits >> 10) : (int)(minnz_bits >> 7);
  const int ue = DT == EQ_F16 ? max(e, 1) - 15 - 10 : max(e, 1) - 127 - 7;
  const int lc = 32 - __clz((int)cols - 1);
  return lc + 5 + ea <= 53 + ue;
}

// Segment of the chunk's row j.
__device__ __forceinline__ int find_seg_by_row(const SortSeg* __restrict__ segs, int nsegs, int64_t j) {
  int lo = 0, hi = nsegs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (segs[mid].first_row <= j) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// NT threads (256 for rows of up to 8192 elements, three workgroups per compute unit; 512 or 1024 beyond),
// K 16-byte chunks of the row per thread.  A workgroup walks through rows j, j + G, j + 2 G, ... of the
// launch, the loads of its next row in flight while it sorts this one.
// Wavefronts per SIMD the kernel is compiled for: what its LDS lets a compute unit hold (three
// 256-thread workgroups; two 512-thread ones for rows of up to some 14 000 elements; one 1024-thread
// workgroup for longer rows: every phase of the sort waits on
// LDS round trips, and four wavefronts per SIMD hide them better than the two of a 512-thread
// workgroup with twice the registers, 18 % less time on rows of 22016).
template <int NT, int K>
constexpr int sort_waves_per_simd() { return NT == 256 ? 3 : 4; }

template <int DT, int NT, int K, int NB>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(sort_waves_per_simd<NT, K>(), sort_waves_per_simd<NT, K>()))) void sorted_prepare(const MatDesc* __restrict__ mats, const SortSeg* __restrict__ segs,
                                                     int nsegs, int64_t total_rows, EQ_GLOBAL unsigned char* __restrict__ ws,
                                                     KParams kp) {
  constexpr int NW = NT / kWave;
  constexpr int kSortBuckets = NB, kSortCounters = sort_counters(NB);
  typedef BatchScratch<1, NW> Scratch;
  extern __shared__ __align__(16) unsigned char smem[];
  Scratch* sc = reinterpret_cast<Scratch*>(smem);
  SortScratch* ss = reinterpret_cast<SortScratch*>(smem + sizeof(Scratch));
  unsigned char* pool = smem + sort_header_bytes<NT>();
  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;

  // (descriptors and segments are read where they are used, through pointers that are the same for
  // the whole workgroup: copies of them that change from row to row would live in scratch memory)
  int64_t j = blockIdx.x;
  if (j >= total_rows) return;
  const SortSeg* sg = segs + find_seg_by_row(segs, nsegs, j);
  const MatDesc* md = mats + sg->mat;
  const uint32_t cols = (uint32_t)md->cols, nchunks = cols >> 3, upr = cols >> 7;   // the same for every row of the launch
  uint16_t* tmp = reinterpret_cast<uint16_t*>(pool + (size_t)upr * kSlotBytes);
  uint32_t* cntw = reinterpret_cast<uint32_t*>(tmp + cols); // 16-bit counts, then the buckets' first positions, in pairs
  const uint16_t* cnt = reinterpret_cast<const uint16_t*>(cntw);
  uint16_t* out = reinterpret_cast<uint16_t*>(pool);        // the pool is free once its values sit in tmp
  const size_t rec_bytes = sort_record_bytes(cols);

  uint4 v[1][K];
  int64_t row = sg->row0 + (j - sg->first_row);
  batch_issue_loads<NT, 1, K, true>(*md, row, 1, v);
  for (;;) {
    const int64_t jn = j + gridDim.x;
    const bool more = jn < total_rows;
    const SortSeg* sgn = sg;
    if (more && jn >= sg->first_row + sg->nrows) sgn = segs + find_seg_by_row(segs, nsegs, jn);
    const MatDesc* mdn = mats + sgn->mat;
    const int64_t rown = more ? sgn->row0 + (jn - sgn->first_row) : row;

    if (tid == 0) {
      sc->rowmax_bits[0] = 0;
      sc->rownegmin_bits[0] = 0;
      ss->minnz_bits = 0xFFFFFFFFu;
      ss->big_bucket = 0;
    }
    for (uint32_t i = tid; i < (uint32_t)kSortCounters / 2; i += NT) cntw[i] = 0;
    stage_loaded_rows<DT, NT, 1, K, Padded128Layout, true, false>(*md, kp, row, 1, pool, 0u, nullptr, sc, v, [&] {
      batch_issue_loads<NT, 1, K, true>(*mdn, rown, more ? 1 : 0, v);
    });
    __syncthreads();                                         // wavefront-major staging ends without one

    // ---- extremes of the normal values (0 included, as everywhere) ----
    if (tid < upr) {
      float umin, umax;
      slot_min_max<DT>(pool + (size_t)tid * kSlotBytes, umin, umax);
      atomicMax(&sc->rowmax_bits[0], __float_as_uint(umax));
      atomicMax(&sc->rownegmin_bits[0], __float_as_uint(0.0f - umin));
    }
    __syncthreads();
    const float vmax = __uint_as_float(sc->rowmax_bits[0]);
    const float vmin = -__uint_as_float(sc->rownegmin_bits[0]);
    const float bscale = vmax > vmin ? (float)(kSortBuckets - 1) / (vmax - vmin) : 0.0f;
    // monotone in x; zeros (of either sign) alone in the bucket between the negative and the positive values
    auto bucket = [&](float x) {
      int b = (int)((x - vmin) * bscale);
      b = b < 0 ? 0 : (b > kSortBuckets - 1 ? kSortBuckets - 1 : b);
      return (uint32_t)b + (x > 0.0f ? 2u : x == 0.0f ? 1u : 0u);
    };
    const uint32_t zero_bucket = bucket(0.0f);

    // ---- histogram; every element remembers its arrival number in its bucket ----
    uint32_t slots[K][4];                                    // 16 bits each, two to a register
    uint32_t minnz = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const uint32_t ch = (uint32_t)i * NT + tid;
#pragma unroll
      for (int k = 0; k < 4; ++k) slots[i][k] = 0;
      if (ch < nchunks) {
        const uint4 q = *reinterpret_cast<const uint4*>(pool + Padded128Layout::off(ch));
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const uint32_t h = (w[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu;
          const uint32_t bk = bucket(widen16<DT>(h));
          const uint32_t old = atomicAdd(&cntw[bk >> 1], 1u << ((bk & 1u) * 16));   // (no carry: a count stays below 2^16)
          slots[i][k >> 1] |= ((old >> ((bk & 1u) * 16)) & 0xFFFFu) << ((k & 1) * 16);
          const uint32_t a = h & 0x7FFFu;
          minnz = min(minnz, a ? a : 0xFFFFFFFFu);
        }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) minnz = min(minnz, (uint32_t)__shfl_xor((int)minnz, o));
    if (lane == 0) atomicMin(&ss->minnz_bits, minnz);
    __syncthreads();

    // ---- exclusive scan of the bucket counts: consecutive counters per thread (the last thread takes the rest) ----
    {
      constexpr int per = kSortBuckets / NT;                 // counters per thread: 32 or 16
      constexpr int last_extra = kSortCounters - kSortBuckets;
      constexpr int words = (per + last_extra) / 2;
      uint32_t cw[words], s = 0;
      const int mine = tid == NT - 1 ? per + last_extra : per;
#pragma unroll
      for (int k = 0; k < words; ++k) {
        cw[k] = 2 * k < mine ? cntw[(tid * per) / 2 + k] : 0u;
        const uint32_t c0 = cw[k] & 0xFFFFu, c1 = cw[k] >> 16;
        s += c0 + c1;
        if ((c0 > kSortBigBucket && tid * per + 2 * k != zero_bucket) || (c1 > kSortBigBucket && tid * per + 2 * k + 1 != zero_bucket))
          ss->big_bucket = 1u;                               // benign race: every writer stores 1
      }
      const uint32_t inc = wave_scan_inclusive(s);
      if (lane == kWave - 1) ss->wcnt[wave] = inc;
      __syncthreads();
      uint32_t a = inc - s;
#pragma unroll
      for (int w = 0; w < NW; ++w) a += (uint32_t)w < wave ? ss->wcnt[w] : 0u;
#pragma unroll
      for (int k = 0; k < words; ++k) {
        if (2 * k < mine) {
          const uint32_t c0 = cw[k] & 0xFFFFu, c1 = cw[k] >> 16;
          cntw[(tid * per) / 2 + k] = a | ((a + c0) << 16);  // first positions: at most cols <= 32768, 16 bits hold them
          a += c0 + c1;
        }
      }
    }
    __syncthreads();
    const bool ranked = ss->big_bucket == 0u;

    // ---- into the buckets, in arrival order ----
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const uint32_t ch = (uint32_t)i * NT + tid;
      if (ch < nchunks) {
        const uint4 q = *reinterpret_cast<const uint4*>(pool + Padded128Layout::off(ch));
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const uint32_t h = (w[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu;
          const uint32_t slot = (slots[i][k >> 1] >> ((k & 1) * 16)) & 0xFFFFu;
          const uint32_t stored = h ^ (0x8000u | (uint32_t)__builtin_amdgcn_sbfe(h, 15, 1));   // the key, see below
          tmp[cnt[bucket(widen16<DT>(h))] + slot] = (uint16_t)stored;
        }
      }
    }
    __syncthreads();

    // ---- rank inside the bucket: the values below, and the equal ones that arrived earlier ----
    // tmp holds keys (the 16-bit patterns made monotone as unsigned integers); key and position in one
    // word compare as "smaller, or equal and earlier".  Two elements of the bucket per turn, their reads
    // in flight together (a read past the bucket's end stays inside the workgroup's LDS and is not counted):
    // the loop waits for LDS, not for the ALU, and one element per turn takes 10 % longer over the whole
    // kernel; three per turn gain nothing more, four lose.
    auto unkey = [](uint32_t k) { return (k ^ (0x8000u | ~(uint32_t)__builtin_amdgcn_sbfe(k, 15, 1))) & 0xFFFFu; };
    auto rank_in_bucket = [&](uint32_t kx, uint32_t p, uint32_t a, uint32_t e) {
      uint32_t rank = 0;
      const uint32_t me = (kx << 16) | p;
      for (uint32_t q = a; q < e; q += 2) {
        const uint32_t q0 = tmp[q], q1 = tmp[q + 1];
        rank += (uint32_t)(((q0 << 16) | q) < me) + (uint32_t)((q + 1 < e) & (((q1 << 16) | (q + 1)) < me));
      }
      return a + rank;
    };
    for (uint32_t p = tid; p < cols; p += NT) {
      const uint32_t kx = tmp[p];
      const uint32_t h = unkey(kx);
      const uint32_t b = bucket(widen16<DT>(h));
      uint32_t at = p;
      if (ranked && b != zero_bucket) at = rank_in_bucket(kx, p, cnt[b], cnt[b + 1]);
      out[at] = (uint16_t)h;
    }
    __syncthreads();

    // ---- the record: header, then per chunk its 8 values and the exact sum of all values in front of them ----
    EQ_GLOBAL unsigned char* rec = ws + sg->ws_off + (size_t)(j - sg->first_row) * rec_bytes;
    {
      for (uint32_t c = tid; c < nchunks; c += NT) global_store128(rec + kSortRecHeader + (size_t)c * kSortUnit, reinterpret_cast<const uint4*>(out)[c]);
      const uint32_t cpt = (nchunks + NT - 1) / NT;
      const uint32_t c0 = min(tid * cpt, nchunks), c1 = min(c0 + cpt, nchunks);
      auto chunk_sum = [&](uint32_t c) {
        const uint4 q = reinterpret_cast<const uint4*>(out)[c];
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
        double s = 0.0;
#pragma unroll
        for (int k = 0; k < 8; ++k) s += (double)widen16<DT>((w[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
        return s;
      };
      double s = 0.0;
      for (uint32_t c = c0; c < c1; ++c) s += chunk_sum(c);
      double inc = s;                                        // inclusive scan over the wavefront
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const double t = __shfl_up(inc, o);
        if (lane >= (uint32_t)o) inc += t;
      }
      if (lane == kWave - 1) ss->wsum[wave] = inc;
      __syncthreads();
      double a = inc - s;
#pragma unroll
      for (int w = 0; w < NW; ++w) a += (uint32_t)w < wave ? ss->wsum[w] : 0.0;
      for (uint32_t c = c0; c < c1; ++c) {
        *(EQ_GLOBAL double*)(rec + kSortRecHeader + (size_t)c * kSortUnit + 16) = a;
        a += chunk_sum(c);
      }
      if (c1 == nchunks && c0 < c1) *(EQ_GLOBAL double*)(rec + 16) = a;   // the sum of the whole row
      if (tid == 0) {
        float r0;
        int z;
        (void)init_unit(kp, vmin, vmax, r0, z);
        const bool exact = sorted_sums_exact<DT>(fmaxf(-vmin, vmax), ss->minnz_bits, cols);
        // the header (SortRecHeader) as one 128-bit store
        global_store128(rec, make_uint4(__float_as_uint(r0), (uint32_t)z,
                                        (exact ? kRecExactSums : 0u) | (ranked ? kRecSorted : 0u), 0u));
      }
    }
    if (!more) break;
    __syncthreads();                                         // the pool and the counters are refilled
    j = jn;
    sg = sgn;
    md = mdn;
    row = rown;
  }
}

// ---- sums over the 16 lanes of a row (lanes 16 k .. 16 k + 15), result in every one of them ----
__device__ __forceinline__ int row16_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x128, 0xF, 0xF, false);   // row_ror:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x124, 0xF, 0xF, false);   // row_ror:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x122, 0xF, 0xF, false);   // row_ror:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x121, 0xF, 0xF, false);   // row_ror:1
  return v;
}
template <int CTRL>
__device__ __forceinline__ double row_ror(double v) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, false);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double row16_sum(double v) {
  v += row_ror<0x128>(v);
  v += row_ror<0x124>(v);
  v += row_ror<0x122>(v);
  v += row_ror<0x121>(v);
  return v;
}

// The window of the row's record that a lane keeps in LDS: kWinChunks consecutive chunks (8 values
// and the prefix sum in front of them each) around its boundary, as a ring (chunk c sits in slot
// c mod kWinChunks).  A step of Adam moves a boundary by a few dozen positions at most, so nearly
// every probe is served from the window.  After each search the window is moved by up to kWinFetch
// chunks towards where the boundary is heading (its chunk plus the last move): their loads are issued
// before the scalar recurrence and land in the ring at the start of the next search, so their latency
// stays off the critical path.  A probe
// outside the window (the first steps, when the range still moves fast) refills it whole.
constexpr int kWinChunks = 4;
constexpr int kWinFetch = 2;
constexpr int kWinStride = kWinChunks * 24 + 16;             // bytes per lane (a multiple of 16)

template <int DT>
__global__ __launch_bounds__(kWave) void sorted_iterate(const MatDesc* __restrict__ mats, const SortSeg* __restrict__ segs,
                                                         int nsegs, int total_groups, const EQ_GLOBAL unsigned char* __restrict__ ws,
                                                         KParams kp) {
  __shared__ __align__(16) unsigned char win_all[kWave * kWinStride];
  const int lane = (int)threadIdx.x;
  const int group = (int)blockIdx.x;
  if (group >= total_groups) return;
  int lo = 0, hi = nsegs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (segs[mid].first_group <= group) lo = mid; else hi = mid - 1;
  }
  const SortSeg sg = segs[lo];
  const MatDesc md = mats[sg.mat];
  const int rin = 4 * (group - sg.first_group) + (lane >> 4);
  const bool live = rin < sg.nrows;
  const int N = md.cols, nblk = N >> 3;
  const EQ_GLOBAL unsigned char* rec = ws + sg.ws_off + (size_t)(live ? rin : sg.nrows - 1) * sort_record_bytes(N);
  SortRecHeader hd;
  {
    const uint4 q = global_load128(rec);
    hd.r0 = __uint_as_float(q.x); hd.z = (int32_t)q.y; hd.flags = q.z; hd.pad = 0;
  }
  const EQ_GLOBAL unsigned char* units = rec + kSortRecHeader;   // per chunk: 8 values, then the sum of all values in front of them
  auto unit_q = [&](int c) { return global_load128(units + (size_t)c * kSortUnit); };
  auto unit_P = [&](int c) { return *(const EQ_GLOBAL double*)(units + (size_t)c * kSortUnit + 16); };
  unsigned char* win = win_all + lane * kWinStride;          // values at 0, prefix sums at 16 * kWinChunks
  int wj0 = 0;                                               // the window holds chunks [wj0, wj0 + kWinChunks)
  bool wvalid = false;
  int pf_shift = 0;                                          // chunks on their way: up to +-kWinFetch towards higher / lower positions
  int j_last = 0, dj_last = 0;                               // chunk of the boundary at the last search, and its last move
  uint4 pf_q[kWinFetch];
  double pf_P[kWinFetch];
  auto win_q = [&](int c) -> uint4& { return *reinterpret_cast<uint4*>(win + (c & (kWinChunks - 1)) * 16); };
  auto win_P = [&](int c) -> double& { return *reinterpret_cast<double*>(win + kWinChunks * 16 + (c & (kWinChunks - 1)) * 8); };

  const int b = lane & 15;
  const int nbound = kp.L;                                   // boundaries between neighbouring levels (<= 15)
  const int clo = -hd.z, chi = kp.L - hd.z;
  const int lev = clo + min(b, nbound - 1);                  // this lane's boundary lies between lev and lev + 1
  const bool counts = b < nbound;
  const int wA = counts ? 2 * lev + 1 : 0;
  const float thr = kMagic + (float)lev;                     // exact: a small integer next to 1.5 * 2^23
  const bool fast = (hd.flags & (kRecExactSums | kRecSorted)) == (kRecExactSums | kRecSorted);
  const double PN = *(const EQ_GLOBAL double*)(rec + 16);
  const bool act = hd.r0 > 0.0f;

  float r32 = act ? hd.r0 : kp.D, r_sel = r32;               // an all-zero row keeps s = 1
  double J_best = __builtin_inf();
  const double floor_r = (double)hd.r0 * 0.0009765625;
  Adam ad;
  ad.init();
  int n = N >> 1;

  for (int t = 0;; ++t) {
    const bool last = t == kp.iters;
    if (last && kp.select == EQ_SELECT_LAST) break;
    double bc[4];
    if (!last) load_bias_corrections(kp, t, bc);
    float s32, inv;
    scale_of(kp, r32, s32, inv);
    int ia = 0;
    double db = 0.0;
    if (fast) {
      // ---- n = number of elements whose level is <= lev, and P[n] ----
      // Probes of whole 8-element chunks, starting with the one that held the boundary last time:
      // inside the chunk the boundary is found at once; a chunk entirely on one side moves the search
      // on, by doubling steps until the boundary is bracketed, then by halving.  The first search of a
      // row halves from the start and reads the record itself.
      const bool first = t == 0;
      int nlo = 0, nhi = N, d = 1;
      int j = min(n >> 3, nblk - 1);
      bool have_lo = first, have_hi = first, done = false;
      double Pn = 0.0;
      if (pf_shift != 0) {
        // the chunks asked for after the last search have arrived: into the ring
        const int m = pf_shift > 0 ? pf_shift : -pf_shift;
#pragma unroll
        for (int k = 0; k < kWinFetch; ++k) {
          if (k < m) {
            const int c = pf_shift > 0 ? wj0 + kWinChunks + k : wj0 - 1 - k;
            win_q(c) = pf_q[k];
            win_P(c) = pf_P[k];
          }
        }
        wj0 += pf_shift;
        pf_shift = 0;
      }
      if (wvalid) {
        // the window first: the levels of its chunks' first values tell which chunk holds the boundary
        // (c of them are on the lower side, whatever their order in the ring), or that it lies outside
        int c = 0;
#pragma unroll
        for (int k = 0; k < kWinChunks; ++k) {
          const float x0 = widen16<DT>(*reinterpret_cast<const uint16_t*>(win + k * 16));   // slot k, some chunk of the window
          c += __builtin_fmaf(x0, inv, kMagic) <= thr ? 1 : 0;
        }
        // a boundary outside the window is looked for where its last move points, in steps of that size
        const int ahead = max(1, dj_last < 0 ? -dj_last : dj_last);
        if (c > 0) {
          j = wj0 + c - 1;
          nlo = 8 * j;
          have_lo = true;
          if (c < kWinChunks) { nhi = 8 * j + 8; have_hi = true; }
          else { j = min(max(j, j_last + dj_last), nblk - 1); d = ahead; }
        } else {
          nhi = 8 * wj0;                                     // P[nhi] = 0 if this is the row's start, else found by the probes
          have_hi = true;
          j = max(min(wj0 - 1, j_last + dj_last), 0);
          d = ahead;
          if (wj0 == 0) { n = 0; done = true; }
        }
      }
      while (!__all(done)) {
        if (!done) {
          uint4 q;
          double Pj;
          if (first) {
            q = unit_q(j);
            Pj = unit_P(j);
          } else {
            if (!wvalid || j < wj0 || j >= wj0 + kWinChunks) {
              // refill, with j in the middle
              wj0 = max(0, min(j - kWinChunks / 2 + 1, nblk - kWinChunks));
              wvalid = true;
#pragma unroll
              for (int k = 0; k < kWinChunks; ++k) {
                const int c = wj0 + k;
                win_q(c) = unit_q(c);
                win_P(c) = unit_P(c);
              }
            }
            q = win_q(j);
            Pj = win_P(j);
          }
          const uint32_t w[4] = {q.x, q.y, q.z, q.w};
          int cnt = 0;
          double part = 0.0;
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            const float xv = widen16<DT>((w[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
            const bool le = __builtin_fmaf(xv, inv, kMagic) <= thr;
            cnt += le ? 1 : 0;
            part += le ? (double)xv : 0.0;
          }
          if (cnt > 0 && cnt < 8) { n = 8 * j + cnt; Pn = Pj + part; done = true; }
          else if (cnt == 8) { nlo = 8 * j + 8; have_lo = true; Pn = Pj + part; }
          else { nhi = 8 * j; have_hi = true; Pn = Pj; }
          if (!done && nlo >= nhi) { n = nlo; done = true; }
          if (!done) {
            if (have_lo && have_hi) j = (nlo + nhi) >> 4;
            else if (have_lo) { j = min(j + d, nblk - 1); d <<= 1; }
            else { j = max(j - d, 0); d <<= 1; }
          }
        }
      }
      ia = wA * n;
      db = counts ? Pn : 0.0;
      const int j_now = min(n, N - 1) >> 3;
      dj_last = t > 0 ? j_now - j_last : 0;
      const int j_next = j_now + dj_last;
      j_last = j_now;
      if (wvalid && !last) {
        // the window's middle goes where the boundary is heading: ask for the next chunks on that side
        // now, they are stored when the next search begins
        const int want0 = max(0, min(j_next - kWinChunks / 2 + 1, nblk - kWinChunks));
        const int shift = want0 - wj0;
        pf_shift = shift > kWinFetch ? kWinFetch : shift < -kWinFetch ? -kWinFetch : shift;
        if (pf_shift != 0) {
#pragma unroll
          for (int k = 0; k < kWinFetch; ++k) {
            int c = pf_shift > 0 ? wj0 + kWinChunks + k : wj0 - 1 - k;
            c = max(0, min(c, nblk - 1));                    // (those beyond the shift are not used)
            pf_q[k] = unit_q(c);
            pf_P[k] = unit_P(c);
          }
        }
      }
    } else {
      // ---- element by element (binary64 accumulation of exact products, like the general kernel) ----
      const float fclo = (float)clo, fchi = (float)chi;
      for (int ch = b; ch < nblk; ch += 16) {
        const uint4 q = unit_q(ch);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const float xv = widen16<DT>((w[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
          const float c = level_of(xv, inv, fclo, fchi);
          const int ci = (int)c;
          ia += ci * ci;
          db += (double)(xv * c);
        }
      }
    }
    const int SA = row16_sum(ia);
    const double SB = row16_sum(db);
    const double A = fast ? (double)(chi * chi * N - SA) : (double)SA;
    const double B = fast ? (double)chi * PN - SB : SB;
    double J, g;
    loss_and_grad(kp, s32, A, B, J, g);
    if (J < J_best) { J_best = J; r_sel = r32; }
    if (last) break;
    const float r_new = ad.step(kp, bc, r32, g, floor_r);
    if (act) r32 = r_new;
  }
  if (kp.select == EQ_SELECT_LAST) r_sel = r32;
  if (live && b == 0) md.range[sg.row0 + rin] = r_sel;
}

}  // namespace eq
