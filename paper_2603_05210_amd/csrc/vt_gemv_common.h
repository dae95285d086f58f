// Pieces shared by the streaming-regime kernels (vt_gemv.hip, vt_gemv1.hip): the kernel
// argument block, device-coherent accesses for partial results, the bf16 dot-product step and
// the final merge that the last workgroup of a single-launch step runs.
#pragma once

#include "vt.h"
#include "vt_device.h"
#include "vt_internal.h"

namespace vt {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct GemvArgs {
    const u32x4* h;
    const u32x4* W;
    const void* scales;  // compressed W_sub only: fp32 per row (FP8) or exponent byte per 32 weights (MXFP4)
    const uint16_t* gamma;  // fused RMSNorm weight, or NULL
    float eps;
    const float* parent;    // per-row score added to the emitted log-probabilities, or NULL
    uint16_t* h_out;        // test hook: normalised hidden state, or NULL
    int rows, nchunk, Vd, P, k, KP, rpb;  // rpb: W_sub rows per workgroup (multiple of J)
    int ks;  // slices of the hidden dimension whose partial logits sit side by side in LDS (1: none)
    int nsg; // kernel for a few rows: groups of 16 hidden states, each served by workgroups of its own
    float* part_val;
    int32_t* part_idx;
    float2* part_stat;
    float* logits_out;
    // fused final merge (done by the last workgroup to finish) -- used when `fused` is set
    int fused;
    unsigned int* arrive;  // this call's arrival counter (workspace header), zero between calls
    const int32_t* d2t;
    int32_t* out_ids;
    float* out_logp;
    float* lse_out;
};

// The arrival counter of the fused merge lives in the header of the call's own workspace (which
// concurrent calls never share): zero between calls, the last workgroup of a call puts it back.
//
// No cache-wide fences are used: the partial results are a few hundred bytes per workgroup and
// travel through device-coherent accesses (relaxed agent-scope atomics: they bypass the
// per-XCD caches), ordered by "stores acknowledged -> workgroup barrier -> ticket".
__device__ __forceinline__ void st_dev(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev(int* p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_dev(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ int ld_dev(const int* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

hipError_t launch_gemv_one_row(const Plan& p, const GemvArgs& ga, hipStream_t s);
hipError_t launch_gemv_few_rows(const Plan& p, const GemvArgs& ga, hipStream_t s);
hipError_t launch_gemv_few_rows_q(int fmt, const Plan& p, const GemvArgs& ga, hipStream_t s);
hipError_t launch_gemv_one_row_q(int fmt, const Plan& p, const GemvArgs& ga, hipStream_t s);
hipError_t launch_gemv_q(int fmt, const Plan& p, const HeadArgs& a, hipStream_t s);

// Final merge by the last workgroup: the partial lists of every row are fetched into LDS (all
// threads, coalesced), 256 threads per hidden-state row reduce the row's softmax partials, then
// one wave per row merges the row's lists by walking their heads (k rounds) and emits ids
// (through d2t) and log-probabilities.
constexpr int kFusedMaxRows = kGemvThreads / 256;
template <int KP>
__device__ __forceinline__ void fused_final_merge(const GemvArgs& a, char* lds, int tid)
{
    constexpr int S = KP + 1;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int row = tid >> 8;
    const int p = tid & 255;
    float* lv = reinterpret_cast<float*>(lds);                 // [rows][256][S]
    int* li = reinterpret_cast<int*>(lv + a.rows * 256 * S);   // [rows][256][S]
    float2* wstat = reinterpret_cast<float2*>(li + a.rows * 256 * S);  // [waves]

    // lists: consecutive threads fetch consecutive words of the row's [P][KP] arrays
    const int kp_shift = ilog2(KP);
    for (int r = 0; r < a.rows; ++r) {
        const size_t off = (size_t)r * a.P * KP;
        for (int e = tid; e < a.P * KP; e += kGemvThreads) {
            const float v = ld_dev(a.part_val + off + e);
            const int ix = ld_dev(a.part_idx + off + e);
            const int at = (r * 256 + (e >> kp_shift)) * S + (e & (KP - 1));
            lv[at] = v;
            li[at] = ix;
        }
    }
    const bool ok = row < a.rows && p < a.P;
    float m = neg_inf(), s = 0.0f;
    if (ok) {
        const size_t slot = (size_t)row * a.P + p;
        m = ld_dev(reinterpret_cast<const float*>(a.part_stat + slot));
        s = ld_dev(reinterpret_cast<const float*>(a.part_stat + slot) + 1);
    }
    wave_stat_merge(m, s, ok);  // the four waves of a row each reduce their share
    if (lane == 0)
        wstat[wave] = make_float2(m, s);
    __syncthreads();

    if ((wave & 3) == (row & 3) && row < a.rows) {  // one wave per row, each on a SIMD of its own
        float ov;
        int oi;
        wave_walk_merge<KP, 4, true>(lv + row * 256 * S, li + row * 256 * S, a.P, a.k, lane, ov, oi);
        const bool act = lane < 4;
        float mv = act ? wstat[(wave & ~3) + (lane & 3)].x : neg_inf();
        float sv = act ? wstat[(wave & ~3) + (lane & 3)].y : 0.0f;
        wave_stat_merge(mv, sv, act);
        const float lse = mv + __logf(sv);
        if (lane < a.k) {
            a.out_ids[(size_t)row * a.k + lane] = (oi != kIdxNone) ? a.d2t[oi] : -1;
            a.out_logp[(size_t)row * a.k + lane] = (ov - lse) + (a.parent != nullptr ? a.parent[row] : 0.0f);
        }
        if (lane == 0 && a.lse_out != nullptr)
            a.lse_out[row] = lse;
    }
}

template <bool DOT2>
__device__ __forceinline__ float dot8(const u32x4& w, const u32x4& x, float acc)
{
    if constexpr (DOT2) {
        // (cast the whole 128-bit vector, then pick pairs: a bit_cast of a single component of
        // an ext_vector reads component 0 with this compiler)
        const bf16x8 wb = __builtin_bit_cast(bf16x8, w);
        const bf16x8 xb = __builtin_bit_cast(bf16x8, x);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(wb, wb, 0, 1), __builtin_shufflevector(xb, xb, 0, 1), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(wb, wb, 2, 3), __builtin_shufflevector(xb, xb, 2, 3), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(wb, wb, 4, 5), __builtin_shufflevector(xb, xb, 4, 5), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(wb, wb, 6, 7), __builtin_shufflevector(xb, xb, 6, 7), acc, false);
    } else {
        acc = fmaf(bf16_lo(w.x), bf16_lo(x.x), acc);
        acc = fmaf(bf16_hi(w.x), bf16_hi(x.x), acc);
        acc = fmaf(bf16_lo(w.y), bf16_lo(x.y), acc);
        acc = fmaf(bf16_hi(w.y), bf16_hi(x.y), acc);
        acc = fmaf(bf16_lo(w.z), bf16_lo(x.z), acc);
        acc = fmaf(bf16_hi(w.z), bf16_hi(x.z), acc);
        acc = fmaf(bf16_lo(w.w), bf16_lo(x.w), acc);
        acc = fmaf(bf16_hi(w.w), bf16_hi(x.w), acc);
    }
    return acc;
}

}  // namespace vt
