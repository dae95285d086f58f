// MFMA-regime projection kernels for candidate lists of length 2.
#include "vt_gemm_impl.h"

namespace vt {
hipError_t launch_gemm_kp2(const Plan& p, const GemmArgs& ga, hipStream_t s) { return launch_gemm_kp<2>(p, ga, s); }
}  // namespace vt
