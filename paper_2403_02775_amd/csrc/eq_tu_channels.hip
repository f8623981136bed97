// Instantiations of the per-channel lane kernels for one input type, EQ_TU_DT.
#ifndef EQ_TU_DT
#define EQ_TU_DT 0   // the build compiles this file once per input type (0: fp16, 1: bf16)
#endif
#include "eq_channel128.h"
#include "eq_channel_split.h"
#include "eq_launch.h"

namespace eq {

template <int DT>
LaneKernel pick_channel_kernel(const LaneClass& lc) {
  LaneKernel k;
  if (lc.kind == 5) {
    // rows cut into equal pieces; chunks_per_thread carries the variant chosen by the plan
#define EQ_SPLIT_VARIANT(ID_, P_, LPR_)                                                                         \
  if (lc.chunks_per_thread == ID_) {                                                                            \
    k.fn = reinterpret_cast<const void*>(&quantize_channels_split<DT, P_, LPR_>);                               \
    k.launch = [](const LaneClass& c, const MatDesc* dm, const WorkItem* di, const KParams& kp, hipStream_t s) { \
      hipLaunchKernelGGL((quantize_channels_split<DT, P_, LPR_>), dim3((unsigned)c.n_items), dim3(kChanThreads), \
                         c.lds_bytes, s, dm, di + c.first_item, kp);                                            \
    };                                                                                                          \
  }
    EQ_SPLIT_VARIANT(1, 43, 256) EQ_SPLIT_VARIANT(2, 43, 128) EQ_SPLIT_VARIANT(3, 27, 256) EQ_SPLIT_VARIANT(4, 35, 256)
#undef EQ_SPLIT_VARIANT
    return k;
  }
#define EQ_CHAN_VARIANT(K_, FULL_)                                                                              \
  if (lc.chunks_per_thread == K_ && (lc.kind == 7) == FULL_) {                                                  \
    k.fn = reinterpret_cast<const void*>(&quantize_channels128<DT, K_, FULL_>);                                 \
    k.launch = [](const LaneClass& c, const MatDesc* dm, const WorkItem* di, const KParams& kp, hipStream_t s) { \
      hipLaunchKernelGGL((quantize_channels128<DT, K_, FULL_>), dim3((unsigned)c.n_items), dim3(kChanThreads),  \
                         c.lds_bytes, s, dm, di + c.first_item, kp);                                            \
    };                                                                                                          \
  }
  EQ_CHAN_VARIANT(1, false) EQ_CHAN_VARIANT(2, false) EQ_CHAN_VARIANT(4, false) EQ_CHAN_VARIANT(8, false) EQ_CHAN_VARIANT(16, false)
  EQ_CHAN_VARIANT(1, true) EQ_CHAN_VARIANT(2, true) EQ_CHAN_VARIANT(4, true)
#undef EQ_CHAN_VARIANT
  return k;
}

template LaneKernel pick_channel_kernel<EQ_TU_DT>(const LaneClass&);

}  // namespace eq
