// Host-side plan of one vt_draft_head call and the launchers of the kernel families.
// Everything here is internal to the library (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "vt_plan.h"

namespace vt {

struct HeadArgs {
    const uint16_t* h;
    const uint16_t* W;
    const void* scales;  // compressed W_sub only
    const uint16_t* gamma;  // fused RMSNorm: weight [H] (bf16), or NULL when h is already normalised
    float eps;
    const float* parent;    // cumulative log-probability of each row's node, added to the outputs (or NULL)
    uint16_t* h_out;        // test hook: the normalised hidden state [rows][H] (or NULL)
    const int32_t* d2t;
    int32_t* out_ids;
    float* out_logp;
    unsigned int* arrive;  // arrival counter in the workspace header
    float* part_val;   // [rows][P][KP]
    int32_t* part_idx; // [rows][P][KP]
    float2* part_stat; // [rows][P]  (max, sum exp(z - max))
    float* logits_out; // optional [rows][Vd]
    float* lse_out;    // optional [rows]
};

struct GemmArgs {
    const void* h;
    const void* W;
    int rows, nchunk, Vd, P;
    int n_vtiles, n_rtiles;
    float* part_val;
    int32_t* part_idx;
    float2* part_stat;
    float* logits_out;
    uint16_t* store_out;  // projection-only use: the product as a bf16 matrix [rows][Vd] instead of partial results
};

#define VT_DECL_GEMM_KP(N) hipError_t launch_gemm_kp##N(const Plan& p, const GemmArgs& ga, hipStream_t s);
VT_DECL_GEMM_KP(1)
VT_DECL_GEMM_KP(2)
VT_DECL_GEMM_KP(4)
VT_DECL_GEMM_KP(8)
VT_DECL_GEMM_KP(16)
VT_DECL_GEMM_KP(32)
VT_DECL_GEMM_KP(64)
#undef VT_DECL_GEMM_KP

hipError_t launch_gemv(const Plan& p, const HeadArgs& a, hipStream_t s);
hipError_t launch_gemm(const Plan& p, const HeadArgs& a, hipStream_t s);
hipError_t launch_merge(const Plan& p, const HeadArgs& a, hipStream_t s);
hipError_t launch_quant_gather(int fmt, const uint16_t* W, int H, const int32_t* ids, int Vd, uint8_t* codes,
                               void* scales, int32_t* d2t, hipStream_t s);
hipError_t launch_rmsnorm(const uint16_t* g, const uint16_t* gamma, float eps, int rows, int H, uint16_t* h_out, hipStream_t s);
hipError_t launch_feature_fusion(const uint16_t* x, int rows, int d_in, const uint16_t* W_fc, int d_out, uint16_t* g_out,
                                 hipStream_t s);
hipError_t launch_clear_words(uint32_t* p, int n, hipStream_t s);
hipError_t launch_check_ids(const int32_t* ids, int Vd, int V, uint32_t* bitmap, int* err, hipStream_t s);
hipError_t launch_gather(const uint16_t* W, int H, const int32_t* ids, int Vd, uint16_t* W_sub, int32_t* d2t,
                         hipStream_t s);

}  // namespace vt
