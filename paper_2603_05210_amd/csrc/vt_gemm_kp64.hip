// MFMA-regime projection kernels for candidate lists of length 64.
#include "vt_gemm_impl.h"

namespace vt {
hipError_t launch_gemm_kp64(const Plan& p, const GemmArgs& ga, hipStream_t s) { return launch_gemm_kp<64>(p, ga, s); }
}  // namespace vt
