// Internal interface of the t2d / coverage kernels (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace vt {

struct CoverageLayout {
    size_t off_seen, off_inv, off_counters, off_err, total;
};

CoverageLayout coverage_layout(int64_t V);
hipError_t launch_build_t2d(const int32_t* d2t, int Vd, int V, int32_t* t2d, int* err, hipStream_t s);
hipError_t launch_coverage(const int32_t* tokens, int64_t n, const int32_t* t2d, int V, int32_t* draft_ids, char* ws,
                           const CoverageLayout& L, hipStream_t s);

}  // namespace vt
