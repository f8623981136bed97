// Instantiations of the sorted evaluation of rows with one range each, for one input type, EQ_TU_DT.
#ifndef EQ_TU_DT
#define EQ_TU_DT 0   // the build compiles this file once per input type (0: fp16, 1: bf16)
#endif
#include "eq_launch.h"
#include "eq_sorted.h"

namespace eq {

// workgroups of sorted_prepare: as many as the chip holds at once (its LDS decides), each walking
// through rows j, j + G, j + 2 G, ... of the chunk
static unsigned prepare_grid(int64_t rows, size_t lds) {
  const int64_t per_cu = (int64_t)std::max<size_t>(1, std::min<size_t>(8, (160u * 1024u) / lds));
  return (unsigned)std::min<int64_t>(rows, 256 * per_cu);
}

template <int DT>
SortKernels pick_sorted_kernels(const LaneClass& lc) {
  SortKernels k;
  const int64_t nchunks = (int64_t)lc.cols / 8;
  // rows of which two fit the LDS of a compute unit (up to some 14 000 elements): 512 threads, two
  // workgroups; longer ones: 1024 threads, one workgroup; four wavefronts per SIMD either way
  const bool two_fit = lc.cols <= 16384 && 2 * sort_prepare_lds(sort_header_bytes<512>(), lc.cols, 8192) <= 160u * 1024u - 128u;
  const int nt = lc.cols <= 8192 ? 256 : two_fit ? 512 : 1024;
  const int64_t per_thread = (nchunks + nt - 1) / nt;
#define EQ_SORT_VARIANT(NT_, K_, NB_)                                                                                  \
  {                                                                                                                  \
    k.prepare_fn = reinterpret_cast<const void*>(&sorted_prepare<DT, NT_, K_, NB_>);                                      \
    k.prepare_lds = sort_prepare_lds(sort_header_bytes<NT_>(), lc.cols, NB_);                                             \
    k.prepare = [](const LaneClass& c, const SortLaunchArgs& a, const KParams& kp, hipStream_t s) {                  \
      const size_t lds = sort_prepare_lds(sort_header_bytes<NT_>(), c.cols, NB_);                                         \
      hipLaunchKernelGGL((sorted_prepare<DT, NT_, K_, NB_>), dim3(prepare_grid(a.rows, lds)), dim3(NT_), lds, s,          \
                         a.mats, a.segs, (int)a.nsegs, a.rows, (EQ_GLOBAL unsigned char*)a.ws, kp);                  \
    };                                                                                                               \
  }
  if (nt == 256) {
    if (per_thread <= 1) EQ_SORT_VARIANT(256, 1, 4096)
    else if (per_thread <= 2) EQ_SORT_VARIANT(256, 2, 4096)
    else EQ_SORT_VARIANT(256, 4, 4096)
  } else if (nt == 512) {
    EQ_SORT_VARIANT(512, 4, 8192)
  } else {
    if (per_thread <= 2) EQ_SORT_VARIANT(1024, 2, 8192)
    else EQ_SORT_VARIANT(1024, 4, 8192)
  }
#undef EQ_SORT_VARIANT
  k.iterate = [](const LaneClass&, const SortLaunchArgs& a, const KParams& kp, hipStream_t s) {
    hipLaunchKernelGGL((sorted_iterate<DT>), dim3((unsigned)a.groups), dim3(kWave), 0, s, a.mats, a.segs, (int)a.nsegs,
                       (int)a.groups, (const EQ_GLOBAL unsigned char*)a.ws, kp);
  };
  return k;
}

template SortKernels pick_sorted_kernels<EQ_TU_DT>(const LaneClass&);

}  // namespace eq
