// MFMA-regime projection kernels for candidate lists of length 4.
#include "vt_gemm_impl.h"

namespace vt {
hipError_t launch_gemm_kp4(const Plan& p, const GemmArgs& ga, hipStream_t s) { return launch_gemm_kp<4>(p, ga, s); }
}  // namespace vt
