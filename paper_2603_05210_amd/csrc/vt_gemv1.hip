// The one-row draft step over a bf16 W_sub: instantiations of the generic one-row kernel.
#include "vt_onerow.h"

namespace vt {

hipError_t launch_gemv_one_row(const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    if (!one_row_launch_ok(p, ga))
        return hipErrorInvalidValue;
    switch (ga.nchunk) {  // 16-byte pieces per row: H = 8 * nchunk = 512 * T
    case 64: return launch_one_row_t<FmtBf16, 1>(p, ga, s);
    case 128: return launch_one_row_t<FmtBf16, 2>(p, ga, s);
    case 256: return launch_one_row_t<FmtBf16, 4>(p, ga, s);
    case 512: return launch_one_row_t<FmtBf16, 8>(p, ga, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace vt
