// What the host side and the translation units that hold the lane kernels share: the description
// of one launch, and one selector per kernel family.  Each family is compiled in a file of its
// own (eq_tu_units.hip, eq_tu_channels.hip, eq_tu_rtn.hip, eq_tu_sorted.hip), once per input type, so that the
// library builds in parallel; a selector returns the instantiation that serves a launch, or
// nothing if there is none.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

#include "eq_common.h"

namespace eq {

struct WorkItem;

// One launch of the unit-per-lane kernel: all matrices of a batch that share a row length.
struct LaneClass {
  int32_t kind = 1;                     // 1: one lane per group of 128, 2: per-channel rows spread over lanes,
                                        // 3: group of 128 without optimisation steps (load-pipelined kernel),
                                        // 5: per-channel rows cut into equal pieces over all lanes,
                                        // 6: per-channel rows without optimisation steps (kernel of kind 3, one range per row),
                                        // 7: kind 2 for rows of exactly 2048, 4096 or 8192 elements and at most 4 bits
  int32_t cols = 0, upr = 0;
  int32_t threads = kThreads;           // workgroup size = units per round
  int32_t chunks_per_thread = 1;        // 16-byte chunks of a row per thread, rounded up to 1, 2, 4 or 8
  int32_t rows_per_batch = 0;           // rows staged at once by the kind-1 kernel; 0 = 16 / chunks_per_thread
  uint32_t pool_slots = 0;
  size_t lds_bytes = 0;
  size_t first_item = 0, n_items = 0;
  int64_t rows_per_item = 0;            // every matrix of the class is cut into items of this many rows (the last one shorter),
  int64_t item_stride = 0;              // or (item_stride != 0) into interleaved items: item g takes the batches of
  int64_t rows_per_step = 0;            // rows_per_step rows that start at rows g * rows_per_step + k * item_stride
  // kind 6 after an optimisation from sorted rows (eq_sorted.h): the class's rows are cut into chunks
  // whose records fit the workspace; each chunk is prepared and iterated, then the kind-6 launch emits
  bool sorted = false;
  size_t first_chunk = 0, n_chunks = 0;
};

// One chunk of a sorted class: segments [first_seg, first_seg + n_segs) of the plan's list.
struct SortChunk {
  size_t first_seg = 0, n_segs = 0;
  int64_t rows = 0;
  int64_t groups = 0;                   // groups of 4 rows, counted per segment
};

typedef void (*LaneLaunch)(const LaneClass&, const MatDesc*, const WorkItem*, const KParams&, hipStream_t);
struct LaneKernel {
  const void* fn = nullptr;       // for hipFuncSetAttribute
  LaneLaunch launch = nullptr;
  size_t lds_bytes = 0;           // dynamic LDS of the launch if the family sizes it itself (else LaneClass::lds_bytes)
};

// The two kernels of the sorted evaluation for a class (eq_tu_sorted.hip).
struct SortLaunchArgs {
  const MatDesc* mats;
  const SortSeg* segs;                  // device: the chunk's segments
  int32_t nsegs;
  int64_t rows;
  int64_t groups;
  unsigned char* ws;                    // device: the records of the chunk
};
typedef void (*SortLaunch)(const LaneClass&, const SortLaunchArgs&, const KParams&, hipStream_t);
struct SortKernels {
  const void* prepare_fn = nullptr;     // for hipFuncSetAttribute
  size_t prepare_lds = 0;
  SortLaunch prepare = nullptr, iterate = nullptr;
};
template <int DT> SortKernels pick_sorted_kernels(const LaneClass& lc);

template <int DT> LaneKernel pick_units_kernel(const LaneClass& lc);     // kind 1
template <int DT> LaneKernel pick_channel_kernel(const LaneClass& lc);   // kinds 2, 5 and 7
template <int DT> LaneKernel pick_rtn_kernel(const LaneClass& lc);       // kinds 3 and 6

}  // namespace eq
