// Internal interface of the vocabulary-size selection kernels (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "vt.h"

namespace vt {

struct SelectParams {
    long long d;            // hidden size of the head (Section 2.3: 2*d*k FLOPs)
    double F_fixed;         // FLOPs of the draft model that do not depend on k
    double alpha, c_min;    // Eq. 4 weight, Eq. 5 coverage threshold
    long long k_min, k_max; // Eq. 1 range
};

struct SelectLayout {
    int N2;  // V rounded up to a power of two (at least one sort chunk)
    size_t off_keys, off_mark, off_result, off_seg, off_err, total;
};

SelectLayout select_layout(int64_t V);
hipError_t launch_select(const int32_t* tokens, int64_t n, int V, const SelectParams& prm, uint32_t* freq,
                         int32_t* rank_ids, int32_t* token_ids, char* ws, const SelectLayout& L, hipStream_t s);

}  // namespace vt
