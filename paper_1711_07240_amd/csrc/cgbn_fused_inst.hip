// Explicit instantiations of the NCHW single-launch kernels, one translation unit per
// (element type, direction, activation) so that they compile side by side.  The build
// passes CGBN_INST_T (float or bf16_t), CGBN_INST_F32 (1 for float), CGBN_INST_FWD (0/1) and CGBN_INST_ACT (0/1/2).
#include "cgbn_fused.h"
#include "cgbn_fused_list.h"

namespace cgbn {
#if CGBN_INST_FWD
#define CGBN_X(LB_, LPPC_) template __global__ void nchw_fused_forward<CGBN_INST_T, LB_, LPPC_, CGBN_INST_ACT, 0>(FusedArgs);
CGBN_FUSED_COMMON(CGBN_X)
CGBN_FUSED_FORWARD_ONLY(CGBN_X)
template __global__ void nchw_fused_forward<CGBN_INST_T, 16, 0, CGBN_INST_ACT, 1>(FusedArgs);      // big-LDS variants
template __global__ void nchw_fused_forward<CGBN_INST_T, 16, -2, CGBN_INST_ACT, 1>(FusedArgs);
#define CGBN_X1(LB_, LPPC_) template __global__ void nchw_fused_forward<CGBN_INST_T, LB_, LPPC_, CGBN_INST_ACT, 1>(FusedArgs);
CGBN_FUSED_WGP_FORWARD(CGBN_X1)
#undef CGBN_X1
#define CGBN_X2(LB_, LPPC_) template __global__ void nchw_fused_forward<CGBN_INST_T, LB_, LPPC_, CGBN_INST_ACT, 2>(FusedArgs);
CGBN_FUSED_BIG_SMALL(CGBN_X2)
#else
#define CGBN_X(LB_, LPPC_) template __global__ void nchw_fused_backward<CGBN_INST_T, LB_, LPPC_, CGBN_INST_ACT, 0>(FusedArgs);
#define CGBN_X2(LB_, LPPC_) template __global__ void nchw_fused_backward<CGBN_INST_T, LB_, LPPC_, CGBN_INST_ACT, 2>(FusedArgs);
template __global__ void nchw_fused_backward<CGBN_INST_T, 16, 0, CGBN_INST_ACT, 1>(FusedArgs);     // big-LDS variants
template __global__ void nchw_fused_backward<CGBN_INST_T, 16, -2, CGBN_INST_ACT, 1>(FusedArgs);
#define CGBN_X1(LB_, LPPC_) template __global__ void nchw_fused_backward<CGBN_INST_T, LB_, LPPC_, CGBN_INST_ACT, 1>(FusedArgs);
CGBN_FUSED_WGP_BACKWARD(CGBN_X1)
#undef CGBN_X1
#if CGBN_INST_F32 && CGBN_INST_ACT == 1
// (the float ReLU backward with 4-byte accesses: see CGBN_FUSED_RELU_BWD_F32_NARROW)
CGBN_FUSED_COMMON_WIDE(CGBN_X)
CGBN_FUSED_BACKWARD_ONLY_WIDE(CGBN_X)
CGBN_FUSED_RELU_BWD_F32_NARROW(CGBN_X)
CGBN_FUSED_BIG_SMALL_WIDE(CGBN_X2)
#else
CGBN_FUSED_COMMON(CGBN_X)
CGBN_FUSED_BACKWARD_ONLY(CGBN_X)
CGBN_FUSED_BIG_SMALL(CGBN_X2)
#endif
#endif
#undef CGBN_X
#undef CGBN_X2
}  // namespace cgbn
