// Host side of the C ABI declared in include/easyquant.h: argument checks, workspace
// carving, descriptor upload and kernel launches.  Every step of the quantization path
// runs in the kernels; nothing here touches weight data.
#include <hip/hip_runtime.h>

#include <cmath>
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <atomic>
#include <mutex>
#include <numeric>
#include <vector>

#include "easyquant.h"
#include "eq_common.h"
#include "eq_channel128.h"
#include "eq_fused128.h"
#include "eq_generic.h"
#include "eq_launch.h"
#include "eq_post.h"
#include "eq_rowstage.h"
#include "eq_testing.h"

// Scratch memory of eq_quantize_matrix_noalloc: every GPU the library's code object is loaded
// on holds its own copy of this array, at its own address, until the process ends.  In host code
// the name is only a handle for hipGetSymbolAddress; kernels and copies get the address that
// call returned for the device at hand.
static __device__ __align__(256) unsigned char scratch[EQ_STATIC_SCRATCH_BYTES];

namespace {

using namespace eq;

thread_local int g_last_hip_error = 0;

// Address of `scratch` on the current device, looked up once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
unsigned char* g_scratch_ptr[kMaxDevices] = {};


// ---- kernel-selection overrides for tests and measurements (eq_testing.h); 0 = default ----
std::atomic<int64_t> g_override[EQ_OVR_COUNT] = {};
inline int64_t override_of(int which) { return g_override[which].load(std::memory_order_relaxed); }

// ---- optional event bracketing of the main kernels (eq_profile_*) ----
// (calls from several host threads may bracket kernels at once: the list has a lock)
std::atomic<bool> g_profile{false};
std::mutex g_events_lock;
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_events;

struct ScopedKernelTimer {
  hipStream_t st;
  hipEvent_t a = nullptr, b = nullptr;
  explicit ScopedKernelTimer(hipStream_t s, bool enabled = true) : st(s) {
    if (!g_profile || !enabled) return;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { a = b = nullptr; return; }
    (void)hipEventRecord(a, st);
  }
  // drops the bracket: nothing is added to the list
  void cancel() {
    if (!a) return;
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    a = b = nullptr;
  }
  ~ScopedKernelTimer() {
    if (!a) return;
    (void)hipEventRecord(b, st);
    std::lock_guard<std::mutex> hold(g_events_lock);
    g_events.emplace_back(a, b);
  }
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// A caller's device pointer as the descriptors store it (global address space).
template <class T>
inline EQ_GLOBAL T* dev(T* p) { return (EQ_GLOBAL T*)p; }

constexpr int kMatrixStatParts = 1024;   // workgroups of the whole-matrix statistics pre-pass

bool params_ok(const eq_params* p) {
  if (p->dtype != EQ_F16 && p->dtype != EQ_BF16) return false;
  if (p->bits < 2 || p->bits > 8) return false;
  if (p->mode != EQ_SYMMETRIC && p->mode != EQ_ASYMMETRIC) return false;
  if (p->stat_scope < EQ_STAT_ROW || p->stat_scope > EQ_STAT_MATRIX) return false;
  if (p->select != EQ_SELECT_BEST && p->select != EQ_SELECT_LAST) return false;
  if (p->iters < 0 || p->group_size < 0) return false;
  if (!(p->n_sigma >= 0.0f)) return false;                 // NaN or negative
  if (!(p->lr >= 0.0f) || !std::isfinite(p->lr)) return false;
  if (!(p->beta1 >= 0.0f && p->beta1 < 1.0f) || !(p->beta2 >= 0.0f && p->beta2 < 1.0f)) return false;
  if (!(p->eps > 0.0f) || !std::isfinite(p->eps)) return false;   // 0 would make a zero gradient's step 0 / 0
  return true;
}

int shape_check(int64_t rows, int64_t cols, int64_t ld, const eq_params* p) {
  if (rows < 0 || cols < 0 || rows > 0x7FFFFFFF) return EQ_E_SHAPE;
  if (cols % 8) return EQ_E_SHAPE;
  if (cols > EQ_MAX_COLS) return EQ_E_UNSUPPORTED;
  if (ld < cols || ld % 8) return EQ_E_SHAPE;
  if (p->group_size) {
    if (p->group_size % 32 || cols % p->group_size) return EQ_E_SHAPE;
  }
  return EQ_OK;
}

KParams make_kparams(const eq_params* p) {
  KParams k;
  std::memset(&k, 0, sizeof(k));
  k.dtype = p->dtype; k.bits = p->bits; k.mode = p->mode; k.scope = p->stat_scope;
  k.select = p->select; k.iters = p->iters;
  k.L = (1 << p->bits) - 1;
  k.zsym = (1 << (p->bits - 1)) - 1;
  k.D = p->mode == EQ_SYMMETRIC ? (float)k.zsym : (float)k.L;
  k.n = (double)p->n_sigma;
  k.lr = (double)p->lr; k.b1 = (double)p->beta1; k.b2 = (double)p->beta2; k.eps = (double)p->eps;
  k.rD64 = 1.0 / (double)k.D;
  k.rD32 = 1.0f / k.D;
  k.adam_tab = nullptr;
  return k;
}

// Bias corrections of Adam for steps 1..T and their correctly rounded reciprocals, in the
// order the kernels read them (Adam::step).  The running products are formed exactly as the
// recurrence defines them: p <- p * beta in binary64.
std::vector<double> make_adam_table(const eq_params* p) {
  std::vector<double> tab((size_t)std::max(p->iters, 1) * 4, 1.0);
  const double b1 = (double)p->beta1, b2 = (double)p->beta2;
  double p1 = 1.0, p2 = 1.0;
  for (int t = 0; t < p->iters; ++t) {
    p1 = p1 * b1;
    p2 = p2 * b2;
    tab[4 * (size_t)t + 0] = 1.0 - p1;
    tab[4 * (size_t)t + 1] = 1.0 / (1.0 - p1);
    tab[4 * (size_t)t + 2] = 1.0 - p2;
    tab[4 * (size_t)t + 3] = 1.0 / (1.0 - p2);
  }
  return tab;
}

// Byte offsets of everything that lives in the workspace, and the launch plan.
struct Plan {
  size_t descs = 0;                     // MatDesc[n]
  size_t items = 0;                     // WorkItem[]
  size_t adam = 0;                      // double[4 * max(T, 1)]
  std::vector<size_t> cursor, row_count, row_stage, st_col, st_val, mat_stats, mat_partial;
  std::vector<int32_t> path;            // per matrix: 0 = general kernel, 1 = unit-per-lane kernel, 2 = per-channel lane kernel
  std::vector<LaneClass> classes;
  // The CSR finish (row pointers, then the move of the staged runs) goes group by group: the matrices
  // of each launch class in launch order, then everything else.  finish_ids lists the matrices in
  // that order (uploaded behind the work items), a group is [first, first + count) of it.
  struct FinishGroup { size_t first = 0, count = 0; int32_t max_rows = 0; };
  std::vector<int32_t> finish_ids;
  std::vector<FinishGroup> finish_groups;   // classes.size() + 1 of them
  size_t ids = 0;                       // int32_t[n]
  std::vector<WorkItem> work;
  // sorted evaluation of per-channel rows (eq_sorted.h): the segments of all chunks (uploaded behind
  // the ids), the chunks, the per-row ranges of each matrix and the one region that holds a chunk's records
  std::vector<SortSeg> segs;
  std::vector<SortChunk> chunks;
  size_t segs_off = 0;
  std::vector<size_t> range;            // per matrix: float[rows], or 0
  size_t sort_ws = 0, sort_ws_bytes = 0;
  bool any_general = false;
  size_t total = 0;
};

// Records of the sorted evaluation that a launch may hold at once: the rows of a class are cut into
// chunks of at most this many bytes (some 87 000 rows of 8192 elements: enough wavefronts of
// sorted_iterate to fill the chip several times over).
constexpr size_t kSortBudgetBytes = (size_t)2 << 30;
constexpr int64_t kSideItems = 160;               // work items of the long-row class when it runs beside the others (T = 0)
constexpr int64_t kSortMinCols = 2048;
// Rows are optimised from their sorted values when steps x (columns - kSortStepCols) >= kSortPasses x columns:
// sorting a row costs as much as kSortPasses direct evaluations of it, a step from the sorted row as much as
// a direct evaluation of kSortStepCols elements whatever the row's length.
constexpr int64_t kSortPasses = 57;               // (bf16: kSortPassesBf16; its staging, done twice on this route, is the slower one)
constexpr int64_t kSortPassesBf16 = 80;
constexpr int64_t kSortStepCols = 960;

int64_t clamp_capacity(int64_t c) { return c < 0 ? 0 : (c > 0xFFFFFFFEll ? 0xFFFFFFFEll : c); }

// The unit-per-lane kernel serves group_size 128 with row or matrix statistics and rows that
// fit its LDS pool; everything else goes to the general kernel.
bool lane_kernel_ok(int64_t rows, int64_t cols, const eq_params* p) {
  return p->group_size == kG && p->stat_scope != EQ_STAT_GROUP && rows > 0 && cols > 0 && cols <= 32768;
}

// The per-channel lane kernel serves rows of 2048 .. 32768 elements in multiples of 128 (a
// per-group statistic scope is the row scope when the row is the unit).
bool channel_kernel_ok(int64_t rows, int64_t cols, const eq_params* p) {
  return (p->group_size == 0 || p->group_size == cols) && rows > 0 && cols % kG == 0 && cols >= 2048 && cols <= 32768;
}

// Share of the lanes that have a unit when rows of `upr` units are staged into a pool of `slots`
// slots and taken out in rounds of `nt` (the fill and take rules of quantize_units128): a pool
// that cannot hold a whole number of rounds plus a row runs a partly filled round now and then.
double lane_use_of_rounds(int64_t upr, int64_t nt, int64_t slots) {
  int64_t pool = 0, used = 0, offered = 0;
  for (int i = 0; i < 2048; ++i) {
    while (pool < nt && pool + upr <= slots) pool += upr;
    if (pool == 0) return 0.0;                       // not even one row fits
    const int64_t take = pool >= nt ? (pool / nt) * nt : pool;
    used += take;
    offered += (take + nt - 1) / nt * nt;
    pool -= take;
  }
  return (double)used / (double)offered;
}

Plan make_plan(int32_t n, const int64_t* rows, const int64_t* cols, const int64_t* cap, const eq_params* p,
               bool allow_sorted) {
  Plan pl;
  pl.path.assign((size_t)n, 0);
  std::vector<char> wants_range((size_t)n, 0);
  // ---- launch plan ----
  std::vector<int32_t> order;
  const bool force_general = override_of(EQ_OVR_FORCE_GENERAL) == 1;   // test / measurement override
  for (int32_t i = 0; i < n; ++i) {
    if (force_general) {
      if (rows[i] > 0 && cols[i] > 0) pl.any_general = true;
    } else if (lane_kernel_ok(rows[i], cols[i], p)) {
      pl.path[(size_t)i] = 1;
      order.push_back(i);
    } else if (channel_kernel_ok(rows[i], cols[i], p)) {
      pl.path[(size_t)i] = 2;
      order.push_back(i);
    } else if (rows[i] > 0 && cols[i] > 0) {
      pl.any_general = true;
    }
  }
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return cols[a] < cols[b]; });
  // Without optimisation steps the row-length classes of a batch run side by side on two streams
  // (launch_all).  The kernel for the longest rows, when it is the multi-wavefront one and holds a minor
  // share of the elements, is then started first with FEW, LONG work items (kSideItems workgroups in all),
  // so that it keeps about one workgroup on every other compute unit for the whole step instead of taking
  // the chip for itself at the end, where it runs at 48 % of the memory bandwidth: on the 65B-shaped set
  // 34.35 instead of 35.55 ms per step (alternating measurements in one process; 160 to 420 items: 34.35 to
  // 34.55 ms, 1000 and more: no gain).
  int64_t all_elems = 0, longest_cols = 0, longest_elems = 0;
  size_t distinct = 0;
  for (size_t k = 0; k < order.size(); ++k) {
    const int64_t c = cols[order[k]];
    if (k == 0 || c != cols[order[k - 1]]) { ++distinct; longest_cols = c; longest_elems = 0; }
    all_elems += rows[order[k]] * c;
    longest_elems += rows[order[k]] * c;
  }
  const bool side_by_side = p->iters == 0 && distinct >= 2 && override_of(EQ_OVR_CLASS_STREAMS) != 1;
  const bool few_long_items = side_by_side && longest_cols > 8192 && longest_elems * 20 <= all_elems * 7;   // at most 35 %
  for (size_t k = 0; k < order.size();) {
    size_t e = k;
    int64_t total_units = 0;
    const int64_t c = cols[order[k]];
    const int64_t upr = c / kG;
    while (e < order.size() && cols[order[e]] == c) total_units += rows[order[e++]] * upr;
    LaneClass lc;
    lc.cols = (int32_t)c;
    lc.upr = (int32_t)upr;
    const bool chan_keep128 = override_of(EQ_OVR_CHANNEL_KERNEL) == 128;
    // one range per row, at most 4 bits, optimisation steps: Adam runs on the sorted rows (eq_sorted.h)
    // and the kernel without optimisation steps emits at the ranges it leaves
    // (measured on the 65B-shaped set at lr = 1e-3, each row length by itself: the two evaluations take the
    // same time at 55 steps for rows of 22016 and at 60 for rows of 8192; the rule adds 8 % to that: 60 and 65
    // steps, 75 for rows of 4096, 108 for rows of 2048; for bf16 1.4 times as many: on the 7B-shaped bf16 set
    // the two take the same time at 80 steps for rows of 4096 and at 89 for rows of 11008)
    const bool chan_sorted = pl.path[(size_t)order[k]] == 2 && p->bits <= 4 && allow_sorted && !chan_keep128 &&
                             c >= kSortMinCols && override_of(EQ_OVR_SORTED_ROWS) != 1 &&
                             ((int64_t)p->iters * (c - kSortStepCols) >= (p->dtype == EQ_BF16 ? kSortPassesBf16 : kSortPasses) * c ||
                              (p->iters > 0 && override_of(EQ_OVR_SORTED_ROWS) == 2));
    const bool chan_rtn = pl.path[(size_t)order[k]] == 2 && (p->iters == 0 || chan_sorted) && !chan_keep128;
    if (pl.path[(size_t)order[k]] == 2 && !chan_rtn) {
      // per-channel: a round is floor(256 / segments) whole rows; items are multiples of that
      lc.kind = 2;
      lc.threads = kChanThreads;
      const int64_t per_thread = (c / 8 + kChanThreads - 1) / kChanThreads;
      lc.chunks_per_thread = per_thread <= 1 ? 1 : per_thread <= 2 ? 2 : per_thread <= 4 ? 4 : per_thread <= 8 ? 8 : 16;
      lc.pool_slots = kChanThreads;
      lc.lds_bytes = (size_t)kChanHeader + (size_t)kChanThreads * kSlotBytes;
      int64_t rpr = std::min<int64_t>(kChanThreads / upr, kChanMaxRows);
      if (p->bits <= 4 && (c == 2048 || c == 4096 || c == 8192)) lc.kind = 7;   // lane count known at compile time
      // rows with 4-bit codes whose 128-element segments would leave many of the 256 lanes
      // idle (the MLP down-projections of the LLaMA shapes): equal pieces over all lanes instead
      // (eq_channel_split.h).  chunks_per_thread selects the instantiation.
      const int split = c == 86 * 256 ? 1 : c == 86 * 128 ? 2 : c == 54 * 256 ? 3 : c == 70 * 256 ? 4 : 0;
      if (split && p->bits == 4 && !chan_keep128) {
        lc.kind = 5;
        rpr = split == 2 ? 2 : 1;
        lc.chunks_per_thread = split;
        lc.lds_bytes = (size_t)kChanHeader + (size_t)rpr * (size_t)c * 2 + (size_t)rpr * (size_t)c / 8;   // rows, then one mask byte per chunk
      }
      int64_t target = std::min<int64_t>(8192, std::max<int64_t>(kChanThreads, total_units / 16384));
      if (override_of(EQ_OVR_UNITS_PER_ITEM) > 0) target = override_of(EQ_OVR_UNITS_PER_ITEM);
      int64_t rpi = std::max<int64_t>(rpr, target / upr);
      rpi -= rpi % rpr;
      lc.first_item = pl.work.size();
      lc.rows_per_item = rpi;
      for (size_t j = k; j < e; ++j) {
        const int32_t m = order[j];
        for (int64_t r = 0; r < rows[m]; r += rpi)
          pl.work.push_back(WorkItem{m, (int32_t)r, (int32_t)std::min<int64_t>(rpi, rows[m] - r), 0});
      }
      lc.n_items = pl.work.size() - lc.first_item;
      pl.classes.push_back(lc);
      k = e;
      continue;
    }
    if (p->iters == 0 || chan_sorted) {
      // no optimisation steps: the HBM-bound kernel, one round per batch of 16 / K rows
      // (per-channel rows: the same kernel with one range per row)
      lc.kind = chan_rtn ? 6 : 3;
      if (chan_sorted) {
        lc.sorted = true;
        lc.first_chunk = pl.chunks.size();
        const size_t rec = sort_record_bytes(c);
        int64_t chunk_rows = std::max<int64_t>(4, (int64_t)(kSortBudgetBytes / rec) & ~(int64_t)3);
        if (override_of(EQ_OVR_SORT_CHUNK_ROWS) > 0)
          chunk_rows = std::max<int64_t>(4, std::min<int64_t>(chunk_rows, override_of(EQ_OVR_SORT_CHUNK_ROWS)) & ~(int64_t)3);
        SortChunk ch;
        ch.first_seg = pl.segs.size();
        for (size_t j = k; j < e; ++j) {
          const int32_t m = order[j];
          wants_range[(size_t)m] = 1;
          for (int64_t r = 0; r < rows[m];) {
            if (ch.rows == chunk_rows) {
              ch.n_segs = pl.segs.size() - ch.first_seg;
              pl.chunks.push_back(ch);
              ch = SortChunk();
              ch.first_seg = pl.segs.size();
            }
            const int64_t take = std::min<int64_t>(rows[m] - r, chunk_rows - ch.rows);
            SortSeg sg;
            sg.mat = m; sg.row0 = (int32_t)r; sg.nrows = (int32_t)take;
            sg.first_group = (int32_t)ch.groups;
            sg.first_row = ch.rows;
            sg.ws_off = (int64_t)((size_t)ch.rows * rec);
            pl.segs.push_back(sg);
            ch.rows += take;
            ch.groups += (take + 3) / 4;
            r += take;
          }
        }
        ch.n_segs = pl.segs.size() - ch.first_seg;
        if (ch.n_segs) pl.chunks.push_back(ch);
        lc.n_chunks = pl.chunks.size() - lc.first_chunk;
        for (size_t q = lc.first_chunk; q < pl.chunks.size(); ++q)
          pl.sort_ws_bytes = std::max(pl.sort_ws_bytes, (size_t)pl.chunks[q].rows * rec);
      }
      // longer rows take four wavefronts (two workgroups per compute unit, 15 % faster on rows of
      // 22016 than one of eight);
      // one-wavefront workgroups for rows of up to 8192 (a row, or a batch of short rows, per wavefront:
      // no workgroup barrier anywhere, every wait is the wavefront's own)
      lc.threads = c > 8192 ? 256 : 64;
      if (override_of(EQ_OVR_RTN_THREADS) == 128 && c <= 8192) lc.threads = 128;
      // three wavefronts where the chunks per thread stay the same power of two (8 up to 12288
      // columns, 16 up to 24576): fewer idle lanes and empty load slots (11008: 90 % instead of 67 %)
      if ((c > 8192 && c <= 12288) || (c > 16384 && c <= 24576)) lc.threads = 192;
      if (override_of(EQ_OVR_RTN_THREADS) == 256) lc.threads = 256;
      if (override_of(EQ_OVR_RTN_THREADS) == 512 && c > 8192) lc.threads = 512;
      const int64_t per_thread = (c / 8 + lc.threads - 1) / lc.threads;
      lc.chunks_per_thread = per_thread <= 1 ? 1 : per_thread <= 2 ? 2 : per_thread <= 4 ? 4 : per_thread <= 8 ? 8 : 16;
      if (lc.threads == 512 && lc.chunks_per_thread < 4) lc.chunks_per_thread = 4;
      const int64_t rpb = 16 / lc.chunks_per_thread;
      lc.pool_slots = (uint32_t)(rpb * upr);
      lc.lds_bytes = (size_t)kLdsHeader + (size_t)lc.pool_slots * kSlotBytes;
      // a launch is a few milliseconds long, so its tail (compute units running dry while the last
      // items finish) weighs more than an item's start-up (one batch whose loads are not prefetched):
      // some 30 000 items per launch, of 2048 to 8192 units each (measured on the 65B- and 7B-shaped
      // sets against items 2, 4 and 8 times as large: 4 % and 8 % faster)
      int64_t target = std::min<int64_t>(8192, std::max<int64_t>(2048, total_units / 32768));
      if (override_of(EQ_OVR_UNITS_PER_ITEM) > 0) target = override_of(EQ_OVR_UNITS_PER_ITEM);
      if (few_long_items && c == longest_cols && override_of(EQ_OVR_UNITS_PER_ITEM) <= 0) target = std::max<int64_t>(target, total_units / kSideItems);
      int64_t rpi = std::max<int64_t>(rpb, target / upr);
      rpi -= rpi % rpb;
      lc.first_item = pl.work.size();
      lc.rows_per_item = rpi;
      lc.rows_per_step = rpb;
      // Interleaved items: a matrix of nbatch batches gets G = ceil(nbatch / (rpi / rpb)) workgroups, and
      // workgroup g takes batches g, g + G, g + 2 G, ...  Workgroups are dispatched in order, so at any
      // time the chip reads one contiguous window of each of the few matrices it is working on (HBM
      // pages and channels are used evenly), instead of a thousand streams half a megabyte apart.
      for (size_t j = k; j < e; ++j) {
        const int32_t m = order[j];
        const int64_t nbatch = (rows[m] + rpb - 1) / rpb;
        const int64_t G = (nbatch + rpi / rpb - 1) / (rpi / rpb);
        for (int64_t g = 0; g < G; ++g)
          pl.work.push_back(WorkItem{m, (int32_t)(g * rpb), (int32_t)(rows[m] - g * rpb), (int32_t)(G * rpb)});
      }
      lc.n_items = pl.work.size() - lc.first_item;
      pl.classes.push_back(lc);
      k = e;
      continue;
    }
    // Pool size: a round's worth of units minus what a fill can leave behind, plus one row.
    // With 256-thread workgroups two pools must share the 160 KB of LDS of a compute unit;
    // rows too long for that get one 512-thread workgroup per compute unit, whose pool is
    // capped by the LDS (a fill that finds no room then runs a partly filled round).
    constexpr size_t kLdsPerCu = 160 * 1024;
    const size_t fixed = kLdsHeader;
    auto pool_for = [&](int64_t nt) {
      const int64_t gg = std::gcd(upr, nt);
      return (int64_t)(upr >= nt && upr % nt == 0 ? upr : nt - gg + upr);
    };
    int64_t nt = kThreads;
    int64_t slots = pool_for(nt);
    bool two_per_cu = fixed + (size_t)slots * kSlotBytes <= kLdsPerCu / 2 && c / 8 <= 4 * kThreads;
    if (!two_per_cu && c / 8 <= 8 * kThreads) {
      // Two 256-thread workgroups with pools cut down to half the LDS each still keep (almost) every
      // lane busy for some row lengths (11008: 98 %), and then one workgroup computes while the
      // other stages, which a single 512-thread workgroup per compute unit cannot do.
      const int64_t capped = (int64_t)((kLdsPerCu / 2 - fixed) / kSlotBytes);
      if (lane_use_of_rounds(upr, nt, capped) >= 0.95) {
        two_per_cu = true;
        slots = capped;
      }
    }
    if (!two_per_cu) {
      nt = 512;
      slots = std::min<int64_t>(pool_for(nt), (int64_t)((kLdsPerCu - 64 - fixed) / kSlotBytes));
    }
    lc.threads = (int32_t)nt;
    {
      const int64_t per_thread = (c / 8 + nt - 1) / nt;
      lc.chunks_per_thread = per_thread <= 1 ? (nt == 512 ? 2 : 1) : per_thread <= 2 ? 2 : per_thread <= 4 ? 4 : 8;
    }
    lc.pool_slots = (uint32_t)slots;
    lc.lds_bytes = fixed + (size_t)lc.pool_slots * kSlotBytes;
    // rows of which three fill a round (22016 columns for 512 lanes, 11008 for 256): all three staged
    // as one batch instead of two and one
    if (lc.chunks_per_thread == 8 && 3 * upr >= nt && 3 * upr <= slots) lc.rows_per_batch = 3;
    const int64_t g = std::gcd(upr, nt);
    // rows per work item: enough units to amortise the partly filled last round of an item,
    // few enough that the grid has dozens of items per compute unit (the last items of a launch
    // run on a partly idle chip); a multiple of the period after which rows fill whole rounds
    // when that fits
    int64_t target = std::min<int64_t>(8192, std::max<int64_t>(nt, total_units / 16384));
    // an item's last round is partly filled when rows do not tile the rounds: at least four
    // rounds per item as long as that still leaves a thousand items
    if (target < 4 * nt && total_units / (4 * nt) >= 1024) target = 4 * nt;
    if (override_of(EQ_OVR_UNITS_PER_ITEM) > 0) target = override_of(EQ_OVR_UNITS_PER_ITEM);   // tuning / test override
    const int64_t period = nt / g;
    // as many rows as fill a whole number of rounds as nearly as possible from below: the last
    // round of an item runs with the lanes that are left
    const int64_t rounds = std::max<int64_t>(1, (target + nt / 2) / nt);
    int64_t rpi = std::max<int64_t>(1, rounds * nt / upr);
    if (rpi >= period) rpi -= rpi % period;
    lc.first_item = pl.work.size();
    lc.rows_per_item = rpi;
    for (size_t j = k; j < e; ++j) {
      const int32_t m = order[j];
      for (int64_t r = 0; r < rows[m]; r += rpi)
        pl.work.push_back(WorkItem{m, (int32_t)r, (int32_t)std::min<int64_t>(rpi, rows[m] - r), 0});
    }
    lc.n_items = pl.work.size() - lc.first_item;
    pl.classes.push_back(lc);
    k = e;
  }
  // ---- finish groups ----
  {
    std::vector<char> taken((size_t)n, 0);
    size_t k = 0;
    for (const LaneClass& lc : pl.classes) {
      Plan::FinishGroup g;
      g.first = pl.finish_ids.size();
      while (k < order.size() && cols[order[k]] == lc.cols) {
        pl.finish_ids.push_back(order[k]);
        g.max_rows = std::max<int32_t>(g.max_rows, (int32_t)rows[order[k]]);
        taken[(size_t)order[k]] = 1;
        ++k;
      }
      g.count = pl.finish_ids.size() - g.first;
      pl.finish_groups.push_back(g);
    }
    Plan::FinishGroup rest;
    rest.first = pl.finish_ids.size();
    for (int32_t i = 0; i < n; ++i)
      if (!taken[(size_t)i]) {
        pl.finish_ids.push_back(i);
        if (cols[i] > 0) rest.max_rows = std::max<int32_t>(rest.max_rows, (int32_t)rows[i]);
      }
    rest.count = pl.finish_ids.size() - rest.first;
    pl.finish_groups.push_back(rest);
  }
  // ---- workspace layout ----
  size_t off = 0;
  pl.descs = off;
  off = align_up(off + sizeof(MatDesc) * (size_t)n, 256);
  pl.items = off;
  off = align_up(off + sizeof(WorkItem) * pl.work.size(), 256);
  pl.ids = off;
  off = align_up(off + sizeof(int32_t) * (size_t)n, 256);
  pl.segs_off = off;
  off = align_up(off + sizeof(SortSeg) * pl.segs.size(), 256);
  pl.adam = off;
  off = align_up(off + sizeof(double) * 4 * (size_t)std::max(p->iters, 1), 256);
  for (int32_t i = 0; i < n; ++i) {
    const size_t r = (size_t)rows[i];
    const size_t c = (size_t)clamp_capacity(cap[i]);
    pl.cursor.push_back(off);      off = align_up(off + 8, 256);
    pl.row_count.push_back(off);   off = align_up(off + 4 * r, 256);
    pl.row_stage.push_back(off);   off = align_up(off + 4 * r, 256);
    pl.st_col.push_back(off);      off = align_up(off + 4 * c, 256);
    pl.st_val.push_back(off);      off = align_up(off + 2 * c, 256);
    if (p->stat_scope == EQ_STAT_MATRIX) {
      pl.mat_stats.push_back(off);   off = align_up(off + 16, 256);
      pl.mat_partial.push_back(off); off = align_up(off + 8 * (size_t)kMatrixStatParts, 256);
    } else {
      pl.mat_stats.push_back(0);
      pl.mat_partial.push_back(0);
    }
    if (wants_range[(size_t)i]) {
      pl.range.push_back(off);       off = align_up(off + 4 * r, 256);
    } else {
      pl.range.push_back(0);
    }
  }
  pl.sort_ws = off;
  off = align_up(off + pl.sort_ws_bytes, 256);
  pl.total = off;
  return pl;
}

#define EQ_HIP(call)                                  \
  do {                                                \
    hipError_t e_ = (call);                           \
    if (e_ != hipSuccess) {                           \
      g_last_hip_error = (int)e_;                     \
      return EQ_E_HIP;                                \
    }                                                 \
  } while (0)

int static_scratch_of_current_device(unsigned char** out) {
  int device = -1;
  EQ_HIP(hipGetDevice(&device));
  if (device < 0 || device >= kMaxDevices) return EQ_E_UNSUPPORTED;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    EQ_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || ((uintptr_t)ptr & 255)) return EQ_E_WORKSPACE;
    g_scratch_ptr[device] = static_cast<unsigned char*>(ptr);
  }
  *out = g_scratch_ptr[device];
  return EQ_OK;
}

// ---- pinned host blocks for the descriptor upload ---------------------------------------------
// A call packs what it uploads into one of these and records an event behind the copy; a block is
// taken again only when its event has completed, so its bytes outlive the copy whatever the
// runtime does with host memory.  Blocks are allocated on demand (a few at most: one per call in
// flight), kept for the life of the process, and handed out under a lock.
struct PinnedBlock {
  void* host = nullptr;
  size_t bytes = 0;
  hipEvent_t done = nullptr;
  bool in_use = false;          // between acquire and release
  bool pending = false;         // a copy from it has been enqueued: `done` says when it is over
};
std::mutex g_pinned_lock;
std::vector<PinnedBlock*> g_pinned;

PinnedBlock* acquire_pinned(size_t bytes) {
  std::lock_guard<std::mutex> hold(g_pinned_lock);
  PinnedBlock* pick = nullptr;
  for (PinnedBlock* b : g_pinned) {
    if (b->in_use) continue;
    if (b->pending && hipEventQuery(b->done) != hipSuccess) continue;    // its copy is still on its way
    b->pending = false;
    if (!pick || (pick->bytes < bytes && b->bytes > pick->bytes)) pick = b;
    if (pick->bytes >= bytes) break;
  }
  if (!pick) {
    if (g_pinned.size() >= 16) {
      // many calls in flight: wait for the oldest block instead of growing without bound
      for (PinnedBlock* b : g_pinned)
        if (!b->in_use) { pick = b; break; }
      if (!pick) { g_last_hip_error = (int)hipErrorOutOfMemory; return nullptr; }
      hipError_t e = hipEventSynchronize(pick->done);
      if (e != hipSuccess) { g_last_hip_error = (int)e; return nullptr; }
      pick->pending = false;
    } else {
      pick = new PinnedBlock();
      hipError_t e = hipEventCreateWithFlags(&pick->done, hipEventDisableTiming);
      if (e != hipSuccess) { g_last_hip_error = (int)e; delete pick; return nullptr; }
      g_pinned.push_back(pick);
    }
  }
  if (pick->bytes < bytes) {
    if (pick->host) (void)hipHostFree(pick->host);
    pick->host = nullptr;
    pick->bytes = 0;
    const size_t want = align_up(bytes + bytes / 4, 65536);
    hipError_t e = hipHostMalloc(&pick->host, want, hipHostMallocDefault);
    if (e != hipSuccess) { g_last_hip_error = (int)e; pick->host = nullptr; return nullptr; }
    pick->bytes = want;
  }
  pick->in_use = true;
  return pick;
}

void release_pinned(PinnedBlock* b, hipStream_t st, bool copy_enqueued) {
  std::lock_guard<std::mutex> hold(g_pinned_lock);
  if (copy_enqueued && hipEventRecord(b->done, st) == hipSuccess) b->pending = true;
  else if (copy_enqueued) (void)hipStreamSynchronize(st);   // no event: make sure the copy is over instead
  b->in_use = false;
}

// A second stream per device (default priority), on which the CSR finish of one launch class runs
// while the next class's main kernel occupies the caller's stream.  Ordered by events on both sides.
std::mutex g_aux_lock;
hipStream_t g_aux_stream[kMaxDevices] = {};

int aux_stream_of_current_device(hipStream_t* out) {
  int device = -1;
  EQ_HIP(hipGetDevice(&device));
  if (device < 0 || device >= kMaxDevices) return EQ_E_UNSUPPORTED;
  std::lock_guard<std::mutex> hold(g_aux_lock);
  if (!g_aux_stream[device]) EQ_HIP(hipStreamCreateWithFlags(&g_aux_stream[device], hipStreamNonBlocking));
  *out = g_aux_stream[device];
  return EQ_OK;
}

// Row pointers and the move of the staged runs for one group of matrices.
int launch_finish(const MatDesc* dmats, const int32_t* dids, const Plan::FinishGroup& g, hipStream_t st) {
  if (g.count == 0) return EQ_OK;
  const int32_t* ids = dids ? dids + g.first : nullptr;
  hipLaunchKernelGGL(scan_row_counts, dim3((unsigned)g.count), dim3(kThreads), 0, st, dmats, ids);
  EQ_HIP(hipGetLastError());
  if (g.max_rows > 0) {
    const int rows_per_block = kWaves * kMoveRows;
    hipLaunchKernelGGL(move_outliers, dim3((unsigned)((g.max_rows + rows_per_block - 1) / rows_per_block), (unsigned)g.count),
                       dim3(kThreads), 0, st, dmats, ids);
    EQ_HIP(hipGetLastError());
  }
  return EQ_OK;
}

// dids: the plan's finish_ids on the device, or null for a single matrix (its id is the block index).
template <int DT>
int launch_all(int32_t n, const MatDesc* dmats, const WorkItem* ditems, const int32_t* dids, const SortSeg* dsegs,
               unsigned char* dsort, const std::vector<MatDesc>& h, const Plan& pl, const KParams& kp, hipStream_t st) {
  int32_t max_rows = 0, gen_rows = 0, gen_cols = 0;
  for (const MatDesc& m : h) {
    if (m.cols == 0 || m.rows == 0) continue;
    max_rows = std::max(max_rows, m.rows);
    if (m.path == 0) {
      gen_rows = std::max(gen_rows, m.rows);
      gen_cols = std::max(gen_cols, m.cols);
    }
  }
  hipLaunchKernelGGL(reset_state, dim3((n + 255) / 256), dim3(256), 0, st, dmats, n);
  EQ_HIP(hipGetLastError());
  if (max_rows > 0 && kp.scope == EQ_STAT_MATRIX) {
    for (int pass = 0; pass < 2; ++pass) {
      hipLaunchKernelGGL(matrix_partial_sums<DT>, dim3(kMatrixStatParts, n), dim3(kThreads), 0, st, dmats, pass);
      EQ_HIP(hipGetLastError());
      hipLaunchKernelGGL(matrix_finish_sums, dim3(n), dim3(kThreads), 0, st, dmats, pass, kMatrixStatParts);
      EQ_HIP(hipGetLastError());
    }
  }
  // The finish of a group is hidden under the main kernel of the next one (it moves a few GB and
  // would otherwise stand alone at the end): it goes to the second stream whenever another main
  // kernel follows on the caller's stream.
  const bool have_general = gen_rows > 0;
  hipStream_t aux = nullptr;
  bool aux_used = false;
  int rc = EQ_OK;
  // Without optimisation steps the main kernels are bound by memory, the one for long rows (three
  // wavefronts meeting at barriers) more by its latency than by bandwidth: the row-length classes then
  // alternate between the caller's stream and the second one, each followed by its own finish, so that
  // the kernels of two classes share the chip, the longest rows first and in few, long work items
  // (make_plan; with optimisation steps the kernels are bound by instruction issue and nothing
  // changes).  Classes of the
  // sorted evaluation share one region of records and always run one after the other.
  int busy_classes = 0;
  bool any_sorted = false;
  for (const LaneClass& lc : pl.classes) {
    busy_classes += lc.n_items != 0;
    any_sorted = any_sorted || lc.sorted;
  }
  bool concurrent = false;
  hipStream_t const caller_stream = st;
  // Side by side the kernels' own durations overlap: one bracket around all of them, up to the join.  It
  // opens BEFORE the second stream is released: an event recorded between the release and the first
  // launch delays the caller's stream by a moment, the second stream's kernel then takes the chip
  // first, and the order that this mode lives on (longest rows first) is lost (measured: 35.5 instead
  // of 32.2 ms per step on the 65B-shaped set, slower than one class after the other).
  ScopedKernelTimer* whole = nullptr;
  if (dids && busy_classes >= 2 && !any_sorted && override_of(EQ_OVR_CLASS_STREAMS) != 1 &&
      (kp.iters == 0 || override_of(EQ_OVR_CLASS_STREAMS) == 2) && aux_stream_of_current_device(&aux) == EQ_OK) {
    hipEvent_t ev = nullptr;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) == hipSuccess) {
      whole = new ScopedKernelTimer(caller_stream);
      concurrent = hipEventRecord(ev, st) == hipSuccess && hipStreamWaitEvent(aux, ev, 0) == hipSuccess;
      (void)hipEventDestroy(ev);
      aux_used = concurrent;
      if (!concurrent) {
        whole->cancel();
        delete whole;
        whole = nullptr;
      }
    }
  }
  size_t launched = 0;
  // side by side: the longest rows first (see make_plan)
  for (size_t cii = 0; cii < pl.classes.size() && rc == EQ_OK; ++cii) {
    const size_t ci = concurrent ? pl.classes.size() - 1 - cii : cii;
    const LaneClass& lc = pl.classes[ci];
    if (lc.n_items == 0) continue;
    st = (concurrent && (launched++ & 1)) ? aux : caller_stream;
    // the kernels of each family are instantiated in a translation unit of their own (eq_launch.h)
    const LaneKernel lk = (lc.kind == 3 || lc.kind == 6) ? pick_rtn_kernel<DT>(lc)
                          : (lc.kind == 2 || lc.kind == 5 || lc.kind == 7) ? pick_channel_kernel<DT>(lc) : pick_units_kernel<DT>(lc);
    const void* fn = lk.fn;
    const LaneLaunch launch = lk.launch;
    if (!fn) { rc = EQ_E_UNSUPPORTED; break; }
    const size_t lds_bytes = lk.lds_bytes ? lk.lds_bytes : lc.lds_bytes;
    if (lds_bytes > 65536 && hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess) {
      g_last_hip_error = (int)hipGetLastError();
      rc = EQ_E_HIP;
      break;
    }
    {
      ScopedKernelTimer tm(st, !concurrent);
      KParams kq = kp;
      if (lc.sorted) {
        // chunk by chunk: the records, then Adam on them; the ranges go to MatDesc::range
        const SortKernels sk = pick_sorted_kernels<DT>(lc);
        if (!sk.prepare || !sk.iterate || !dsegs || !dsort) { rc = EQ_E_UNSUPPORTED; break; }
        if (sk.prepare_lds > 160u * 1024u - 64u) { rc = EQ_E_UNSUPPORTED; break; }
        if (sk.prepare_lds > 65536 &&
            hipFuncSetAttribute(sk.prepare_fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sk.prepare_lds) != hipSuccess) {
          g_last_hip_error = (int)hipGetLastError();
          rc = EQ_E_HIP;
          break;
        }
        for (size_t q = lc.first_chunk; q < lc.first_chunk + lc.n_chunks; ++q) {
          const SortChunk& ch = pl.chunks[q];
          SortLaunchArgs a;
          a.mats = dmats; a.segs = dsegs + ch.first_seg; a.nsegs = (int32_t)ch.n_segs;
          a.rows = ch.rows; a.groups = ch.groups; a.ws = dsort;
          sk.prepare(lc, a, kp, st);
          sk.iterate(lc, a, kp, st);
        }
        if (hipGetLastError() != hipSuccess) { rc = EQ_E_HIP; break; }
        kq.range_given = 1;
      }
      launch(lc, dmats, ditems, kq, st);
    }
    if (hipGetLastError() != hipSuccess) { rc = EQ_E_HIP; break; }
    if (concurrent) {
      rc = launch_finish(dmats, dids, pl.finish_groups[ci], st);
      continue;
    }
    bool more_main = have_general;
    for (size_t cj = ci + 1; cj < pl.classes.size(); ++cj) more_main = more_main || pl.classes[cj].n_items != 0;
    hipEvent_t ev = nullptr;
    if (dids && more_main && (aux || aux_stream_of_current_device(&aux) == EQ_OK) &&
        hipEventCreateWithFlags(&ev, hipEventDisableTiming) == hipSuccess) {
      const bool ok = hipEventRecord(ev, st) == hipSuccess && hipStreamWaitEvent(aux, ev, 0) == hipSuccess;
      (void)hipEventDestroy(ev);                       // released once it has completed
      if (ok) {
        aux_used = true;
        rc = launch_finish(dmats, dids, pl.finish_groups[ci], aux);
        continue;
      }
    }
    rc = launch_finish(dmats, dids, pl.finish_groups[ci], st);
  }
  st = caller_stream;
  auto join_aux = [&] {
    // whatever went to the second stream is part of this call: the caller's stream waits for it
    hipEvent_t ev = nullptr;
    bool joined = false;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) == hipSuccess) {
      joined = hipEventRecord(ev, aux) == hipSuccess && hipStreamWaitEvent(st, ev, 0) == hipSuccess;
      (void)hipEventDestroy(ev);
    }
    if (!joined) (void)hipStreamSynchronize(aux);          // no event: wait on the host instead
    aux_used = false;
  };
  if (concurrent) {
    join_aux();
    delete whole;                                          // closes the bracket on the caller's stream, behind the join
  }
  if (rc == EQ_OK && gen_rows > 0) {
    const size_t lds = 256 + (size_t)gen_cols * 2 + (size_t)gen_cols / 8;
    if (lds > 65536 && hipFuncSetAttribute(reinterpret_cast<const void*>(&quantize_rows_generic<DT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      rc = EQ_E_HIP;
    if (rc == EQ_OK) {
      {
        ScopedKernelTimer tm(st);
        hipLaunchKernelGGL(quantize_rows_generic<DT>, dim3(gen_rows, n), dim3(kThreads), lds, st, dmats, kp);
      }
      if (hipGetLastError() != hipSuccess) rc = EQ_E_HIP;
    }
  }
  if (rc == EQ_OK) rc = launch_finish(dmats, dids, pl.finish_groups.back(), st);
  if (aux_used) join_aux();
  return rc;
}

// Argument checks and the descriptor shared by the two consumers of a quantized matrix.
int make_deq_desc(const eq_qmatrix* q, int64_t rows, int64_t cols, const eq_params* p, DeqDesc* d) {
  if (!q || !p) return EQ_E_NULL;
  if (p->dtype != EQ_F16 && p->dtype != EQ_BF16) return EQ_E_PARAM;
  if (p->bits < 2 || p->bits > 8 || p->group_size < 0) return EQ_E_PARAM;
  if (rows < 0 || cols < 0 || rows > 0x7FFFFFFF || cols % 8) return EQ_E_SHAPE;
  if (cols > EQ_MAX_COLS) return EQ_E_UNSUPPORTED;
  if (p->group_size && (p->group_size % 32 || cols % p->group_size)) return EQ_E_SHAPE;
  std::memset(d, 0, sizeof(*d));
  if (rows == 0 || cols == 0) {
    d->rows = (int32_t)rows;
    d->cols = (int32_t)cols;
    return EQ_OK;
  }
  if (!q->codes || !q->scales || !q->zero_points || !q->out_row_ptr) return EQ_E_NULL;
  if ((uintptr_t)q->codes & 3) return EQ_E_ALIGN;
  const bool sparse = q->out_col && q->out_val;
  d->codes = dev(q->codes); d->scales = dev(q->scales); d->zps = dev(q->zero_points);
  d->out_row_ptr = dev(q->out_row_ptr);
  d->out_col = sparse ? dev(q->out_col) : nullptr;
  d->out_val = sparse ? dev(q->out_val) : nullptr;
  d->rows = (int32_t)rows; d->cols = (int32_t)cols;
  d->G = p->group_size ? p->group_size : (int32_t)cols;
  d->upr = d->cols / d->G;
  d->words_per_row = (int32_t)eq_code_words_per_row(cols, p->bits);
  d->bits = p->bits;
  return EQ_OK;
}


// Host-visible checks of a batch and its launch plan (no HIP call).
int check_and_plan(int32_t n, const void* const* W, const int64_t* rows, const int64_t* cols, const int64_t* ld,
                   const eq_params* p, const eq_qmatrix* outs, bool allow_sorted, Plan& pl) {
  if (!W || !rows || !cols || !ld || !p || !outs) return EQ_E_NULL;
  if (!params_ok(p)) return EQ_E_PARAM;
  std::vector<int64_t> caps((size_t)n);
  for (int32_t i = 0; i < n; ++i) {
    const int rc = shape_check(rows[i], cols[i], ld[i], p);
    if (rc != EQ_OK) return rc;
    const eq_qmatrix& o = outs[i];
    if (!o.out_row_ptr || !o.status) return EQ_E_NULL;
    if (o.out_capacity < 0) return EQ_E_SHAPE;
    const bool empty = rows[i] == 0 || cols[i] == 0;
    if (!empty && (!W[i] || !o.codes || !o.scales || !o.zero_points)) return EQ_E_NULL;
    if (o.out_capacity > 0 && (!o.out_col || !o.out_val)) return EQ_E_NULL;
    if (((uintptr_t)W[i] & 15) || ((uintptr_t)o.codes & 15) || ((uintptr_t)o.scales & 3) ||
        ((uintptr_t)o.out_row_ptr & 3) || ((uintptr_t)o.out_col & 3) || ((uintptr_t)o.out_val & 1) ||
        ((uintptr_t)o.status & 3))
      return EQ_E_ALIGN;
    caps[(size_t)i] = o.out_capacity;
  }
  pl = make_plan(n, rows, cols, caps.data(), p, allow_sorted);
  return EQ_OK;
}

// The matrices' descriptors, their workspace slices carved out of `ws` as the plan lays them out.
int fill_descriptors(int32_t n, const void* const* W, const int64_t* rows, const int64_t* cols, const int64_t* ld,
                     const eq_params* p, const eq_qmatrix* outs, const Plan& pl, unsigned char* ws, std::vector<MatDesc>& h) {
  h.resize((size_t)n);
  for (int32_t i = 0; i < n; ++i) {
    MatDesc& m = h[(size_t)i];
    std::memset(&m, 0, sizeof(m));
    const eq_qmatrix& o = outs[i];
    m.W = dev(static_cast<const uint16_t*>(W[i]));
    m.codes = dev(o.codes); m.scales = dev(o.scales); m.zps = dev(o.zero_points);
    m.out_row_ptr = dev(o.out_row_ptr); m.out_col = dev(o.out_col); m.out_val = dev(o.out_val); m.status = dev(o.status);
    m.cursor = dev(reinterpret_cast<unsigned long long*>(ws + pl.cursor[(size_t)i]));
    m.row_count = dev(reinterpret_cast<uint32_t*>(ws + pl.row_count[(size_t)i]));
    m.row_stage = dev(reinterpret_cast<uint32_t*>(ws + pl.row_stage[(size_t)i]));
    m.st_col = dev(reinterpret_cast<uint32_t*>(ws + pl.st_col[(size_t)i]));
    m.st_val = dev(reinterpret_cast<uint16_t*>(ws + pl.st_val[(size_t)i]));
    if (p->stat_scope == EQ_STAT_MATRIX) {
      m.mat_stats = dev(reinterpret_cast<double*>(ws + pl.mat_stats[(size_t)i]));
      m.mat_partial = dev(reinterpret_cast<double*>(ws + pl.mat_partial[(size_t)i]));
    }
    if (pl.range[(size_t)i]) m.range = dev(reinterpret_cast<float*>(ws + pl.range[(size_t)i]));
    m.ld = ld[i];
    m.capacity = clamp_capacity(o.out_capacity);
    m.rows = (int32_t)rows[i];
    m.cols = (int32_t)cols[i];
    m.G = p->group_size ? p->group_size : (int32_t)cols[i];
    m.upr = m.G ? m.cols / m.G : 0;
    m.words_per_row = (int32_t)eq_code_words_per_row(cols[i], p->bits);
    m.path = pl.path[(size_t)i];
  }
  return EQ_OK;
}

// ---- the allocation-free entry point ----------------------------------------------------------
// What eq_quantize_batch copies from host memory into its workspace, written by a kernel from
// by-value arguments instead: the one descriptor, the work items (a matrix is cut into items of
// rows_per_item rows, the last one shorter), Adam's bias corrections 1 - beta^t with their
// correctly rounded reciprocals (the running products formed as the recurrence defines them,
// p <- p * beta in binary64; the division is the IEEE one), and the reset of cursor and status.
constexpr int kNoallocMaxIters = 65536;   // the table is filled by one thread: a bound on that loop

struct SingleSetup {
  MatDesc md;
  MatDesc* dmats;
  WorkItem* ditems;
  EQ_GLOBAL double* dtab;
  int64_t rows_per_item;
  int64_t item_stride, rows_per_step;     // interleaved items (item_stride != 0): see make_plan
  int32_t n_items, iters;
  double b1, b2;
};

__global__ __launch_bounds__(kThreads) void setup_single_matrix(SingleSetup s) {
  if (blockIdx.x == 0) {
    if (threadIdx.x == 0) {
      s.dmats[0] = s.md;
      *s.md.cursor = 0ull;
      *s.md.status = 0;
    }
    if (threadIdx.x == kWave) {            // another wavefront than the one that writes the descriptor
      double p1 = 1.0, p2 = 1.0;
      for (int t = 0; t < s.iters; ++t) {
        p1 = p1 * s.b1;
        p2 = p2 * s.b2;
        s.dtab[4 * (size_t)t + 0] = 1.0 - p1;
        s.dtab[4 * (size_t)t + 1] = 1.0 / (1.0 - p1);
        s.dtab[4 * (size_t)t + 2] = 1.0 - p2;
        s.dtab[4 * (size_t)t + 3] = 1.0 / (1.0 - p2);
      }
      if (s.iters == 0) {
        s.dtab[0] = 1.0; s.dtab[1] = 1.0; s.dtab[2] = 1.0; s.dtab[3] = 1.0;
      }
    }
    return;
  }
  const int64_t i = (int64_t)(blockIdx.x - 1) * kThreads + threadIdx.x;
  if (i < s.n_items) {
    const int64_t r0 = s.item_stride ? i * s.rows_per_step : i * s.rows_per_item;
    WorkItem it;
    it.mat = 0;
    it.row0 = (int32_t)r0;
    it.nrows = (int32_t)(s.item_stride || s.md.rows - r0 < s.rows_per_item ? s.md.rows - r0 : s.rows_per_item);
    it.stride = (int32_t)s.item_stride;
    s.ditems[i] = it;
  }
}

}  // namespace

extern "C" {

void eq_default_params(eq_params* p) {
  if (!p) return;
  p->dtype = EQ_F16; p->bits = 4; p->group_size = 0; p->mode = EQ_SYMMETRIC; p->stat_scope = EQ_STAT_ROW;
  p->n_sigma = 3.0f; p->iters = 100; p->lr = 1e-3f; p->beta1 = 0.9f; p->beta2 = 0.999f; p->eps = 1e-8f;
  p->select = EQ_SELECT_BEST;
}

const char* eq_strerror(int code) {
  switch (code) {
    case EQ_OK: return "ok";
    case EQ_E_NULL: return "a required pointer is NULL";
    case EQ_E_SHAPE: return "inconsistent rows / cols / ld / group_size";
    case EQ_E_PARAM: return "parameter out of range";
    case EQ_E_ALIGN: return "pointer not sufficiently aligned";
    case EQ_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case EQ_E_UNSUPPORTED: return "row too long for on-chip staging";
    case EQ_E_HIP: return "HIP runtime call failed";
    case EQ_E_SCRATCH: return "matrix and outlier capacity exceed the built-in scratch memory of the allocation-free entry point";
    default: return "unknown error code";
  }
}

int eq_last_hip_error(void) { return g_last_hip_error; }

double eq_test_div_f64(double a, double b) { return div_known_rcp(a, b, 1.0 / b); }
float eq_test_div_f32(float a, float b) { return div_known_rcp(a, b, 1.0f / b); }

int eq_test_set_override(int which, int64_t value) {
  if (which < 0 || which >= EQ_OVR_COUNT) return EQ_E_PARAM;
  g_override[which].store(value, std::memory_order_relaxed);
  return EQ_OK;
}

int64_t eq_test_plan_items(int32_t n, const int64_t* rows, const int64_t* cols, const int64_t* out_capacity,
                           const eq_params* p, int32_t* items, int32_t* launch_of_item, int64_t max_items) {
  if (n < 0 || !p || (n > 0 && (!rows || !cols || !out_capacity))) return EQ_E_NULL;
  if (!params_ok(p)) return EQ_E_PARAM;
  for (int32_t i = 0; i < n; ++i)
    if (rows[i] < 0 || cols[i] < 0 || rows[i] > 0x7FFFFFFF) return EQ_E_SHAPE;
  const Plan pl = make_plan(n, rows, cols, out_capacity, p, true);
  for (size_t c = 0; c < pl.classes.size(); ++c) {
    const LaneClass& lc = pl.classes[c];
    for (size_t i = lc.first_item; i < lc.first_item + lc.n_items && (int64_t)i < max_items; ++i) {
      if (items) {
        items[5 * i + 0] = pl.work[i].mat;
        items[5 * i + 1] = pl.work[i].row0;
        items[5 * i + 2] = pl.work[i].nrows;
        items[5 * i + 3] = pl.work[i].stride;
        items[5 * i + 4] = (int32_t)lc.rows_per_step;
      }
      if (launch_of_item) launch_of_item[i] = (int32_t)c;
    }
  }
  return (int64_t)pl.work.size();
}

int64_t eq_test_plan_sort_segments(int32_t n, const int64_t* rows, const int64_t* cols, const int64_t* out_capacity,
                                   const eq_params* p, int64_t* segs, int64_t max_segs, int64_t* record_region_bytes) {
  if (n < 0 || !p || (n > 0 && (!rows || !cols || !out_capacity))) return EQ_E_NULL;
  if (!params_ok(p)) return EQ_E_PARAM;
  for (int32_t i = 0; i < n; ++i)
    if (rows[i] < 0 || cols[i] < 0 || rows[i] > 0x7FFFFFFF) return EQ_E_SHAPE;
  const Plan pl = make_plan(n, rows, cols, out_capacity, p, true);
  for (size_t c = 0; c < pl.chunks.size(); ++c) {
    const SortChunk& ch = pl.chunks[c];
    for (size_t i = ch.first_seg; i < ch.first_seg + ch.n_segs && (int64_t)i < max_segs; ++i) {
      if (!segs) break;
      const SortSeg& sg = pl.segs[i];
      int64_t* o = segs + 7 * i;
      o[0] = (int64_t)c; o[1] = sg.mat; o[2] = sg.row0; o[3] = sg.nrows; o[4] = sg.first_group; o[5] = sg.first_row; o[6] = sg.ws_off;
    }
  }
  if (record_region_bytes) *record_region_bytes = (int64_t)pl.sort_ws_bytes;
  return (int64_t)pl.segs.size();
}

int eq_profile_enable(int on) {
  g_profile = on != 0;
  return EQ_OK;
}

int eq_profile_read(double* kernel_ms, int32_t* launches) {
  double total = 0.0;
  int32_t cnt = 0;
  int rc = EQ_OK;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> events;
  {
    std::lock_guard<std::mutex> hold(g_events_lock);
    events.swap(g_events);
  }
  for (auto& ev : events) {
    float ms = 0.0f;
    hipError_t e = hipEventSynchronize(ev.second);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.first, ev.second);
    if (e != hipSuccess) { g_last_hip_error = (int)e; rc = EQ_E_HIP; }
    total += ms;
    ++cnt;
    (void)hipEventDestroy(ev.first);
    (void)hipEventDestroy(ev.second);
  }
  if (kernel_ms) *kernel_ms = total;
  if (launches) *launches = cnt;
  return rc;
}

int64_t eq_code_words_per_row(int64_t cols, int32_t bits) {
  if (cols < 0 || bits < 1 || bits > 32) return 0;
  return (cols * bits + 31) / 32;
}

int64_t eq_outlier_capacity_bound(int64_t rows, int64_t cols, float n_sigma) {
  if (rows <= 0 || cols <= 0) return 0;
  if (!(n_sigma > 1.0f)) return rows * cols;
  const double per_row = std::floor((double)cols / ((double)n_sigma * (double)n_sigma)) + 1.0;
  const double v = std::fmin(per_row, (double)cols) * (double)rows;
  return (int64_t)v;
}

size_t eq_workspace_bytes(int32_t n, const int64_t* rows, const int64_t* cols, const int64_t* out_capacity,
                          const eq_params* p) {
  if (n < 0 || !p || (n > 0 && (!rows || !cols || !out_capacity))) return 0;
  if (!params_ok(p)) return 0;
  for (int32_t i = 0; i < n; ++i)
    if (rows[i] < 0 || cols[i] < 0 || rows[i] > 0x7FFFFFFF) return 0;
  return make_plan(n, rows, cols, out_capacity, p, true).total + 256;
}

int eq_quantize_batch(int32_t n, const void* const* W, const int64_t* rows, const int64_t* cols, const int64_t* ld,
                      const eq_params* p, const eq_qmatrix* outs, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  if (n < 0 || n > 65535) return EQ_E_SHAPE;
  if (n == 0) return EQ_OK;
  Plan pl;
  std::vector<MatDesc> h;
  int rc = check_and_plan(n, W, rows, cols, ld, p, outs, true, pl);
  if (rc != EQ_OK) return rc;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < pl.total) return EQ_E_WORKSPACE;
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  rc = fill_descriptors(n, W, rows, cols, ld, p, outs, pl, ws, h);
  if (rc != EQ_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  MatDesc* dmats = reinterpret_cast<MatDesc*>(ws + pl.descs);
  WorkItem* ditems = reinterpret_cast<WorkItem*>(ws + pl.items);
  double* dtab = reinterpret_cast<double*>(ws + pl.adam);
  // Descriptors, work items and Adam's table lead the workspace in that order: they are packed
  // with the same offsets into one pinned host block and go up in a single copy.
  const std::vector<double> tab = make_adam_table(p);
  static_assert(sizeof(int32_t) == 4, "");
  const size_t head_bytes = pl.adam + sizeof(double) * tab.size();
  PinnedBlock* blk = acquire_pinned(head_bytes);
  if (!blk) return EQ_E_HIP;
  unsigned char* hb = static_cast<unsigned char*>(blk->host);
  std::memcpy(hb + pl.descs, h.data(), sizeof(MatDesc) * (size_t)n);
  if (!pl.work.empty()) std::memcpy(hb + pl.items, pl.work.data(), sizeof(WorkItem) * pl.work.size());
  std::memcpy(hb + pl.ids, pl.finish_ids.data(), sizeof(int32_t) * pl.finish_ids.size());
  if (!pl.segs.empty()) std::memcpy(hb + pl.segs_off, pl.segs.data(), sizeof(SortSeg) * pl.segs.size());
  std::memcpy(hb + pl.adam, tab.data(), sizeof(double) * tab.size());
  hipError_t ce = hipMemcpyAsync(ws, hb, head_bytes, hipMemcpyHostToDevice, st);
  release_pinned(blk, st, ce == hipSuccess);
  EQ_HIP(ce);
  KParams kp = make_kparams(p);
  kp.adam_tab = dev(dtab);
  const int32_t* dids = reinterpret_cast<const int32_t*>(ws + pl.ids);
  const SortSeg* dsegs = reinterpret_cast<const SortSeg*>(ws + pl.segs_off);
  unsigned char* dsort = ws + pl.sort_ws;
  return p->dtype == EQ_F16 ? launch_all<EQ_F16>(n, dmats, ditems, dids, dsegs, dsort, h, pl, kp, st)
                            : launch_all<EQ_BF16>(n, dmats, ditems, dids, dsegs, dsort, h, pl, kp, st);
}

int eq_quantize_matrix_noalloc(const void* W, int64_t rows, int64_t cols, int64_t ld, const eq_params* p,
                               const eq_qmatrix* out, void* hip_stream) {
  if (!out) return EQ_E_NULL;
  Plan pl;
  std::vector<MatDesc> h;
  // (the sorted evaluation of per-channel rows needs gigabytes of records: not from this entry point)
  int rc = check_and_plan(1, &W, &rows, &cols, &ld, p, out, false, pl);
  if (rc != EQ_OK) return rc;
  if (pl.total > (size_t)EQ_STATIC_SCRATCH_BYTES) return EQ_E_SCRATCH;
  if (p->iters > kNoallocMaxIters) return EQ_E_UNSUPPORTED;
  unsigned char* ws = nullptr;
  rc = static_scratch_of_current_device(&ws);
  if (rc != EQ_OK) return rc;
  rc = fill_descriptors(1, &W, &rows, &cols, &ld, p, out, pl, ws, h);
  if (rc != EQ_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // a matrix is served by one launch class at most, whose work items are a regular cut of its rows
  SingleSetup su;
  su.md = h[0];
  su.dmats = reinterpret_cast<MatDesc*>(ws + pl.descs);
  su.ditems = reinterpret_cast<WorkItem*>(ws + pl.items);
  su.dtab = dev(reinterpret_cast<double*>(ws + pl.adam));
  su.n_items = (int32_t)pl.work.size();
  su.rows_per_item = pl.classes.empty() ? 0 : pl.classes[0].rows_per_item;
  su.rows_per_step = pl.classes.empty() ? 0 : pl.classes[0].rows_per_step;
  su.item_stride = pl.work.empty() ? 0 : pl.work[0].stride;
  su.iters = p->iters;
  su.b1 = (double)p->beta1;
  su.b2 = (double)p->beta2;
  // the kernel regenerates the plan's items from (rows, rows_per_item): make sure they are that regular
  if (pl.classes.size() > 1) return EQ_E_UNSUPPORTED;
  for (size_t i = 0; i < pl.work.size(); ++i) {
    const int64_t r0 = su.item_stride ? (int64_t)i * su.rows_per_step : (int64_t)i * su.rows_per_item;
    const WorkItem& w = pl.work[i];
    const int64_t nr = su.item_stride ? rows - r0 : std::min<int64_t>(su.rows_per_item, rows - r0);
    if (w.mat != 0 || w.row0 != r0 || w.nrows != nr || w.stride != su.item_stride) return EQ_E_UNSUPPORTED;
  }
  hipLaunchKernelGGL(setup_single_matrix, dim3((unsigned)((su.n_items + kThreads - 1) / kThreads + 1)), dim3(kThreads), 0, st, su);
  EQ_HIP(hipGetLastError());
  KParams kp = make_kparams(p);
  kp.adam_tab = su.dtab;
  return p->dtype == EQ_F16 ? launch_all<EQ_F16>(1, su.dmats, su.ditems, nullptr, nullptr, nullptr, h, pl, kp, st)
                            : launch_all<EQ_BF16>(1, su.dmats, su.ditems, nullptr, nullptr, nullptr, h, pl, kp, st);
}

int eq_quantize_matrix(const void* W, int64_t rows, int64_t cols, int64_t ld, const eq_params* p,
                       const eq_qmatrix* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!out) return EQ_E_NULL;
  return eq_quantize_batch(1, &W, &rows, &cols, &ld, p, out, workspace, workspace_bytes, hip_stream);
}

int eq_dequantize(const eq_qmatrix* q, int64_t rows, int64_t cols, const eq_params* p, void* W_out, int64_t ld_out,
                  void* hip_stream) {
  DeqDesc d;
  const int rc = make_deq_desc(q, rows, cols, p, &d);
  if (rc != EQ_OK) return rc;
  if (ld_out < cols || ld_out % 8) return EQ_E_SHAPE;
  if (rows == 0 || cols == 0) return EQ_OK;
  if (!W_out) return EQ_E_NULL;
  if ((uintptr_t)W_out & 15) return EQ_E_ALIGN;
  d.W = dev(static_cast<uint16_t*>(W_out));
  d.ld = ld_out;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  {
    ScopedKernelTimer tm(st);
    const dim3 grid((unsigned)rows), block(kThreads);
    if (p->dtype == EQ_F16 && p->bits == 4) hipLaunchKernelGGL((dequantize_rows<EQ_F16, true>), grid, block, 0, st, d);
    else if (p->dtype == EQ_F16) hipLaunchKernelGGL((dequantize_rows<EQ_F16, false>), grid, block, 0, st, d);
    else if (p->bits == 4) hipLaunchKernelGGL((dequantize_rows<EQ_BF16, true>), grid, block, 0, st, d);
    else hipLaunchKernelGGL((dequantize_rows<EQ_BF16, false>), grid, block, 0, st, d);
  }
  EQ_HIP(hipGetLastError());
  return EQ_OK;
}

int eq_dequant_matvec(const eq_qmatrix* q, int64_t rows, int64_t cols, const eq_params* p, const void* x, float* y,
                      void* hip_stream) {
  DeqDesc d;
  const int rc = make_deq_desc(q, rows, cols, p, &d);
  if (rc != EQ_OK) return rc;
  if (rows == 0) return EQ_OK;
  if (!y || (cols > 0 && !x)) return EQ_E_NULL;
  if (((uintptr_t)x & 15) || ((uintptr_t)y & 3)) return EQ_E_ALIGN;
  d.W = nullptr;
  d.ld = 0;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const unsigned blocks = (unsigned)((rows + kMvRows - 1) / kMvRows);
  {
    ScopedKernelTimer tm(st);
    const EQ_GLOBAL uint16_t* xd = dev(static_cast<const uint16_t*>(x));
    EQ_GLOBAL float* yd = dev(y);
    const dim3 grid(blocks), block(kThreads);
    // per-group tables (modes 3 and 4) need groups of at least 64 elements that tile the kernel's
    // 4096-column segments or are tiled by them
    const int64_t seg_cols = (int64_t)kMvChunks * kThreads * 8;
    const bool tables = d.G >= 64 && (d.G & (d.G - 1)) == 0 && (seg_cols % d.G == 0 || d.G % seg_cols == 0) &&
                        override_of(EQ_OVR_MATVEC_ARITHMETIC) != 1;   // test / measurement override
    const int mode = p->bits != 4 ? 0 : d.upr == 1 ? 2 : tables ? (d.G == 64 ? 4 : 3) : 1;
    if (mode == 2 && cols % 32 == 0) {
      // the paper's format: one range per row (a kernel of its own, 128-bit code loads)
      const int64_t lk = override_of(EQ_OVR_MATVEC_LOOKUP);
#define EQ_MVR(DT_, LK_) hipLaunchKernelGGL((dequant_matvec_rows4<DT_, LK_>), grid, block, 0, st, d, xd, yd)
      if (p->dtype == EQ_F16) {
        if (lk == 1) EQ_MVR(EQ_F16, kLookupMixed); else if (lk == 2) EQ_MVR(EQ_F16, kLookupSingles); else EQ_MVR(EQ_F16, kLookupPairs);
      } else {
        if (lk == 1) EQ_MVR(EQ_BF16, kLookupMixed); else if (lk == 2) EQ_MVR(EQ_BF16, kLookupSingles); else EQ_MVR(EQ_BF16, kLookupPairs);
      }
#undef EQ_MVR
      EQ_HIP(hipGetLastError());
      return EQ_OK;
    }
#define EQ_MV(DT_, MODE_) hipLaunchKernelGGL((dequant_matvec<DT_, MODE_>), grid, block, 0, st, d, xd, yd)
    if (p->dtype == EQ_F16) {
      if (mode == 4) EQ_MV(EQ_F16, 4); else if (mode == 3) EQ_MV(EQ_F16, 3); else if (mode == 2) EQ_MV(EQ_F16, 2);
      else if (mode == 1) EQ_MV(EQ_F16, 1); else EQ_MV(EQ_F16, 0);
    } else {
      if (mode == 4) EQ_MV(EQ_BF16, 4); else if (mode == 3) EQ_MV(EQ_BF16, 3); else if (mode == 2) EQ_MV(EQ_BF16, 2);
      else if (mode == 1) EQ_MV(EQ_BF16, 1); else EQ_MV(EQ_BF16, 0);
    }
#undef EQ_MV
  }
  EQ_HIP(hipGetLastError());
  return EQ_OK;
}

}  // extern "C"
