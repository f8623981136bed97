// Instantiations of the unit-per-lane kernel (group size 128) for one input type, EQ_TU_DT.
#ifndef EQ_TU_DT
#define EQ_TU_DT 0   // the build compiles this file once per input type (0: fp16, 1: bf16)
#endif
#include "eq_fused128.h"
#include "eq_launch.h"

namespace eq {

template <int DT>
LaneKernel pick_units_kernel(const LaneClass& lc) {
  LaneKernel k;
#define EQ_VARIANT(NT_, K_)                                                                                     \
  if (lc.threads == NT_ && lc.chunks_per_thread == K_) {                                                        \
    k.fn = reinterpret_cast<const void*>(&quantize_units128<DT, NT_, K_>);                                      \
    k.launch = [](const LaneClass& c, const MatDesc* dm, const WorkItem* di, const KParams& kp, hipStream_t s) { \
      hipLaunchKernelGGL((quantize_units128<DT, NT_, K_>), dim3((unsigned)c.n_items), dim3(NT_), c.lds_bytes, s, \
                         dm, di + c.first_item, kp, c.pool_slots);                                             \
    };                                                                                                          \
  }
  EQ_VARIANT(256, 1) EQ_VARIANT(256, 2) EQ_VARIANT(256, 4) EQ_VARIANT(256, 8)
  EQ_VARIANT(512, 2) EQ_VARIANT(512, 4) EQ_VARIANT(512, 8)
#undef EQ_VARIANT
  return k;
}

template LaneKernel pick_units_kernel<EQ_TU_DT>(const LaneClass&);

}  // namespace eq
