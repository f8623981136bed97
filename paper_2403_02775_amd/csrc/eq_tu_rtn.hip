// Instantiations of the kernel without optimisation steps (group size 128) for one input type, EQ_TU_DT.
#ifndef EQ_TU_DT
#define EQ_TU_DT 0   // the build compiles this file once per input type (0: fp16, 1: bf16)
#endif
#include "eq_launch.h"
#include "eq_rtn128.h"

namespace eq {

template <int DT>
LaneKernel pick_rtn_kernel(const LaneClass& lc) {
  LaneKernel k;
#define EQ_RTN_VARIANT(NT_, K_)                                                                                 \
  if (lc.threads == NT_ && lc.chunks_per_thread == K_) {                                                        \
    k.lds_bytes = rtn_header_bytes<NT_, K_>() + (size_t)lc.pool_slots * kSlotBytes;                             \
    if (lc.kind == 6) {                                                                                         \
      k.fn = reinterpret_cast<const void*>(&quantize_rtn128<DT, NT_, K_, true>);                                \
      k.launch = [](const LaneClass& c, const MatDesc* dm, const WorkItem* di, const KParams& kp, hipStream_t s) { \
        hipLaunchKernelGGL((quantize_rtn128<DT, NT_, K_, true>), dim3((unsigned)c.n_items), dim3(NT_), (rtn_header_bytes<NT_, K_>() + (size_t)c.pool_slots * kSlotBytes), s, \
                           dm, di + c.first_item, kp);                                                          \
      };                                                                                                        \
    } else {                                                                                                    \
      k.fn = reinterpret_cast<const void*>(&quantize_rtn128<DT, NT_, K_, false>);                               \
      k.launch = [](const LaneClass& c, const MatDesc* dm, const WorkItem* di, const KParams& kp, hipStream_t s) { \
        hipLaunchKernelGGL((quantize_rtn128<DT, NT_, K_, false>), dim3((unsigned)c.n_items), dim3(NT_), (rtn_header_bytes<NT_, K_>() + (size_t)c.pool_slots * kSlotBytes), s, \
                           dm, di + c.first_item, kp);                                                          \
      };                                                                                                        \
    }                                                                                                           \
  }
  EQ_RTN_VARIANT(64, 1) EQ_RTN_VARIANT(64, 2) EQ_RTN_VARIANT(64, 4) EQ_RTN_VARIANT(64, 8) EQ_RTN_VARIANT(64, 16)
  EQ_RTN_VARIANT(128, 1) EQ_RTN_VARIANT(128, 2) EQ_RTN_VARIANT(128, 4) EQ_RTN_VARIANT(128, 8)
  EQ_RTN_VARIANT(256, 1) EQ_RTN_VARIANT(256, 2) EQ_RTN_VARIANT(256, 4) EQ_RTN_VARIANT(256, 8) EQ_RTN_VARIANT(256, 16)
  EQ_RTN_VARIANT(192, 8) EQ_RTN_VARIANT(192, 16)
  EQ_RTN_VARIANT(512, 4) EQ_RTN_VARIANT(512, 8)
#undef EQ_RTN_VARIANT
  return k;
}

template LaneKernel pick_rtn_kernel<EQ_TU_DT>(const LaneClass&);

}  // namespace eq
