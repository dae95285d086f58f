// MFMA-regime projection kernels for candidate lists of length 16.
#include "vt_gemm_impl.h"

namespace vt {
hipError_t launch_gemm_kp16(const Plan& p, const GemmArgs& ga, hipStream_t s) { return launch_gemm_kp<16>(p, ga, s); }
}  // namespace vt
