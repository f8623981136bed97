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
#define EQ_VARIANT_RB(NT_, K_, RB_)                                                                             \
  if (lc.threads == NT_ && lc.chunks_per_thread == K_ && (lc.rows_per_batch ? lc.rows_per_batch : 16 / K_) == RB_) { \
    k.fn = reinterpret_cast<const void*>(&quantize_units128<DT, NT_, K_, RB_>);                                 \
    k.launch = [](const LaneClass& c, const MatDesc* dm, const WorkItem* di, const KParams& kp, hipStream_t s) { \
      hipLaunchKernelGGL((quantize_units128<DT, NT_, K_, RB_>), dim3((unsigned)c.n_items), dim3(NT_), c.lds_bytes, s, \
                         dm, di + c.first_item, kp, c.pool_slots);                                             \
    };                                                                                                          \
  }
#define EQ_VARIANT(NT_, K_) EQ_VARIANT_RB(NT_, K_, 16 / K_)
  EQ_VARIANT(256, 1) EQ_VARIANT(256, 2) EQ_VARIANT(256, 4) EQ_VARIANT(256, 8) EQ_VARIANT_RB(256, 8, 3)
  EQ_VARIANT(512, 2) EQ_VARIANT(512, 4) EQ_VARIANT(512, 8) EQ_VARIANT_RB(512, 8, 3)
#undef EQ_VARIANT
#undef EQ_VARIANT_RB
  return k;
}

template LaneKernel pick_units_kernel<EQ_TU_DT>(const LaneClass&);

}  // namespace eq
