// Target-to-draft index buffer and token coverage of a draft vocabulary on a token stream.
//
// Section 1 of the paper names the two index buffers of an EAGLE-3 style draft with a reduced
// vocabulary: d2t (draft index -> target id, used by the head) and t2d (target id -> draft
// index, used to mask and remap target tokens when the draft is trained or checked).  Section
// 5.1 / Table 4 measure a vocabulary on generated text by two ratios: the share of token
// occurrences it covers (Eq. 2 evaluated on that stream) and the share of distinct tokens.
// Everything here is integer work; the two ratios are one double division each, taken on the
// device by the call's last kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "vt.h"
#include "vt_coverage.h"

namespace vt {

__global__ void t2d_fill_kernel(int32_t* __restrict__ t2d, int V)
{
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v < V)
        t2d[v] = -1;
}

// err bit 0: an id outside [0,V); bit 1: an id that occurs twice
__global__ void t2d_scatter_kernel(const int32_t* __restrict__ d2t, int Vd, int V, int32_t* __restrict__ t2d,
                                   int* __restrict__ err)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= Vd)
        return;
    const int v = d2t[j];
    if (v < 0 || v >= V) {
        atomicOr(err, 1);
        return;
    }
    if (atomicCAS(&t2d[v], -1, j) != -1)
        atomicOr(err, 2);
}

// counters[0] = covered occurrences, counters[1] = distinct tokens, counters[2] = distinct covered
constexpr int kCovThreads = 256;

__global__ void __launch_bounds__(kCovThreads) coverage_kernel(const int32_t* __restrict__ tokens, int64_t n,
                                                               const int32_t* __restrict__ t2d, int V,
                                                               int32_t* __restrict__ draft_ids,
                                                               uint32_t* __restrict__ seen,
                                                               unsigned long long* __restrict__ counters,
                                                               int* __restrict__ err)
{
    unsigned long long covered = 0;
    const int64_t stride = (int64_t)gridDim.x * kCovThreads;
    for (int64_t i = (int64_t)blockIdx.x * kCovThreads + threadIdx.x; i < n; i += stride) {
        const int t = tokens[i];
        int j = -1;
        if (t < 0 || t >= V) {
            atomicOr(err, 1);
        } else {
            j = t2d[t];
            covered += j >= 0 ? 1u : 0u;
            const uint32_t bit = 1u << (t & 31);
            if ((seen[t >> 5] & bit) == 0u)  // most tokens have been seen before: skip the atomic
                atomicOr(&seen[t >> 5], bit);
        }
        if (draft_ids != nullptr)
            draft_ids[i] = j;
    }
    // one atomic per wave
    for (int off = 32; off > 0; off >>= 1)
        covered += __shfl_xor(covered, off, 64);
    if ((threadIdx.x & 63) == 0 && covered != 0)
        atomicAdd(&counters[0], covered);
}

// The same pass with both bitmaps in LDS, for vocabularies whose two V-bit maps fit there and
// calls that do not want the mapped stream: the in-vocabulary map is built once per call in
// memory and copied in, membership and "seen" are LDS bit operations, and the only per-token
// memory traffic is the stream itself.  A workgroup merges its "seen" words into the global
// bitmap when it is done.
constexpr int kCovLdsThreads = 1024;

__global__ void invocab_bitmap_kernel(const int32_t* __restrict__ t2d, int V, uint32_t* __restrict__ inv)
{
    const int w = blockIdx.x * blockDim.x + threadIdx.x;
    const int words = (V + 31) >> 5;
    if (w >= words)
        return;
    uint32_t bits = 0u;
    for (int b = 0; b < 32; ++b) {
        const int v = (w << 5) + b;
        if (v < V && t2d[v] >= 0)
            bits |= 1u << b;
    }
    inv[w] = bits;
}

__global__ void __launch_bounds__(kCovLdsThreads) coverage_lds_kernel(const int32_t* __restrict__ tokens, int64_t n,
                                                                      const uint32_t* __restrict__ inv, int V,
                                                                      uint32_t* __restrict__ seen,
                                                                      unsigned long long* __restrict__ counters,
                                                                      int* __restrict__ err)
{
    extern __shared__ uint32_t cov_lds[];
    const int words = (V + 31) >> 5;
    uint32_t* s_inv = cov_lds;
    uint32_t* s_seen = cov_lds + words;
    for (int w = threadIdx.x; w < words; w += kCovLdsThreads) {
        s_inv[w] = inv[w];
        s_seen[w] = 0u;
    }
    __syncthreads();
    unsigned long long covered = 0;
    auto take = [&](int t) {
        if (t < 0 || t >= V) {
            atomicOr(err, 1);
            return;
        }
        const uint32_t bit = 1u << (t & 31);
        covered += (s_inv[t >> 5] & bit) ? 1u : 0u;
        if ((s_seen[t >> 5] & bit) == 0u)
            atomicOr(&s_seen[t >> 5], bit);
    };
    // 16-byte loads over the 16-byte aligned middle of the stream, four per thread in flight; the few
    // tokens before and after it one by one
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    int64_t head = (int64_t)((16u - (unsigned int)(reinterpret_cast<uintptr_t>(tokens) & 15u)) & 15u) >> 2;
    head = head < n ? head : n;
    const i32x4* t4 = reinterpret_cast<const i32x4*>(tokens + head);
    const int64_t n4 = (n - head) >> 2;
    const int64_t stride = (int64_t)gridDim.x * kCovLdsThreads;
    for (int64_t j = (int64_t)blockIdx.x * kCovLdsThreads + threadIdx.x; j < head; j += stride)
        take(tokens[j]);
    int64_t i = (int64_t)blockIdx.x * kCovLdsThreads + threadIdx.x;
    for (; i + 3 * stride < n4; i += 4 * stride) {
        const i32x4 q0 = __builtin_nontemporal_load(t4 + i);
        const i32x4 q1 = __builtin_nontemporal_load(t4 + i + stride);
        const i32x4 q2 = __builtin_nontemporal_load(t4 + i + 2 * stride);
        const i32x4 q3 = __builtin_nontemporal_load(t4 + i + 3 * stride);
        take(q0.x), take(q0.y), take(q0.z), take(q0.w);
        take(q1.x), take(q1.y), take(q1.z), take(q1.w);
        take(q2.x), take(q2.y), take(q2.z), take(q2.w);
        take(q3.x), take(q3.y), take(q3.z), take(q3.w);
    }
    for (; i < n4; i += stride) {
        const i32x4 q = __builtin_nontemporal_load(t4 + i);
        take(q.x), take(q.y), take(q.z), take(q.w);
    }
    for (int64_t j = head + (n4 << 2) + (int64_t)blockIdx.x * kCovLdsThreads + threadIdx.x; j < n; j += stride)
        take(tokens[j]);
    for (int off = 32; off > 0; off >>= 1)
        covered += __shfl_xor(covered, off, 64);
    if ((threadIdx.x & 63) == 0 && covered != 0)
        atomicAdd(&counters[0], covered);
    __syncthreads();
    for (int w = threadIdx.x; w < words; w += kCovLdsThreads) {
        const uint32_t bits = s_seen[w];
        if (bits != 0u)
            atomicOr(&seen[w], bits);
    }
}

// distinct tokens, and distinct tokens with a draft index, from the bitmap of seen tokens
__global__ void __launch_bounds__(kCovThreads) unique_kernel(const uint32_t* __restrict__ seen,
                                                             const int32_t* __restrict__ t2d, int V,
                                                             unsigned long long* __restrict__ counters)
{
    unsigned long long uni = 0, uni_cov = 0;
    const int words = (V + 31) >> 5;
    for (int w = blockIdx.x * kCovThreads + threadIdx.x; w < words; w += gridDim.x * kCovThreads) {
        uint32_t bits = seen[w];
        uni += (unsigned)__popc(bits);
        while (bits != 0u) {
            const int b = __ffs((int)bits) - 1;
            bits &= bits - 1u;
            uni_cov += t2d[(w << 5) + b] >= 0 ? 1u : 0u;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        uni += __shfl_xor(uni, off, 64);
        uni_cov += __shfl_xor(uni_cov, off, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        if (uni != 0)
            atomicAdd(&counters[1], uni);
        if (uni_cov != 0)
            atomicAdd(&counters[2], uni_cov);
    }
}

// The table's two ratios (one IEEE double division each), written behind the three counters.
__global__ void coverage_ratio_kernel(const unsigned long long* __restrict__ counters, unsigned long long n,
                                      double* __restrict__ ratios)
{
    ratios[0] = (double)counters[0] / (double)n;
    ratios[1] = (double)counters[2] / (double)counters[1];
}

CoverageLayout coverage_layout(int64_t V)
{
    CoverageLayout L;
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    L.off_seen = 0;
    L.off_inv = up((size_t)((V + 31) / 32) * sizeof(uint32_t));
    L.off_counters = L.off_inv + up((size_t)((V + 31) / 32) * sizeof(uint32_t));
    L.off_err = L.off_counters + 256;
    L.total = L.off_err + 256;
    return L;
}

hipError_t launch_build_t2d(const int32_t* d2t, int Vd, int V, int32_t* t2d, int* err, hipStream_t s)
{
    hipError_t e = hipMemsetAsync(err, 0, sizeof(int), s);
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(t2d_fill_kernel, dim3((V + 255) / 256), dim3(256), 0, s, t2d, V);
    hipLaunchKernelGGL(t2d_scatter_kernel, dim3((Vd + 255) / 256), dim3(256), 0, s, d2t, Vd, V, t2d, err);
    return hipGetLastError();
}

hipError_t launch_coverage(const int32_t* tokens, int64_t n, const int32_t* t2d, int V, int32_t* draft_ids, char* ws,
                           const CoverageLayout& L, hipStream_t s)
{
    uint32_t* seen = reinterpret_cast<uint32_t*>(ws + L.off_seen);
    unsigned long long* counters = reinterpret_cast<unsigned long long*>(ws + L.off_counters);
    int* err = reinterpret_cast<int*>(ws + L.off_err);
    hipError_t e = hipMemsetAsync(ws, 0, L.total, s);
    if (e != hipSuccess)
        return e;
    const int words = (V + 31) >> 5;
    const size_t lds = (size_t)words * 2 * sizeof(uint32_t);
    if (draft_ids == nullptr && lds <= 128 * 1024 && n >= (int64_t)1 << 20) {
        // ratios only, long stream: bitmaps in LDS, one workgroup per compute unit
        uint32_t* inv = reinterpret_cast<uint32_t*>(ws + L.off_inv);
        hipLaunchKernelGGL(invocab_bitmap_kernel, dim3((words + 255) / 256), dim3(256), 0, s, t2d, V, inv);
        static std::atomic<size_t> lds_allowed{48 * 1024};  // raised once, then remembered
        if (lds > lds_allowed.load()) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(coverage_lds_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess)
                return e;
            lds_allowed.store(lds);
        }
        hipLaunchKernelGGL(coverage_lds_kernel, dim3(256), dim3(kCovLdsThreads), lds, s, tokens, n, inv, V, seen,
                           counters, err);
    } else {
        int64_t blocks = (n + kCovThreads * 16 - 1) / (kCovThreads * 16);
        if (blocks > 2048)
            blocks = 2048;
        hipLaunchKernelGGL(coverage_kernel, dim3((unsigned)blocks), dim3(kCovThreads), 0, s, tokens, n, t2d, V,
                           draft_ids, seen, counters, err);
    }
    int ub = (words + kCovThreads - 1) / kCovThreads;
    if (ub > 256)
        ub = 256;
    hipLaunchKernelGGL(unique_kernel, dim3(ub), dim3(kCovThreads), 0, s, seen, t2d, V, counters);
    hipLaunchKernelGGL(coverage_ratio_kernel, dim3(1), dim3(1), 0, s, counters, (unsigned long long)n,
                       reinterpret_cast<double*>(counters + 4));
    return hipGetLastError();
}

}  // namespace vt
