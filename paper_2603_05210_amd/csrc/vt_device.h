// Device-side building blocks shared by the head kernels: a total order on (logit, draft
// index), small sorted candidate lists kept in registers, wavefront (64-lane) reductions and
// the merge of per-lane lists across a wavefront.
//
// Order used everywhere: candidate a beats candidate b when a's logit is larger, or the
// logits are equal and a's draft index is smaller.  It is a strict total order on distinct
// indices, so every merge below yields the same k best whatever the partition of the
// vocabulary over lanes, waves and workgroups was.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vt {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kIdxNone = 0x7fffffff;
__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }

__device__ __forceinline__ bool better(float v1, int i1, float v2, int i2)
{
    return (v1 > v2) || (v1 == v2 && i1 < i2);
}

// Sorted (best first) list of KP candidates held in registers; all indexing is static.
template <int KP>
struct TopList {
    float v[KP];
    int i[KP];

    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int s = 0; s < KP; ++s) {
            v[s] = neg_inf();
            i[s] = kIdxNone;
        }
    }

    // Insert when candidates arrive in ascending index order: a newcomer displaces an entry
    // only when strictly larger, which is exactly the lower-index-wins rule.
    __device__ __forceinline__ void insert_ordered(float x, int ix)
    {
#pragma unroll
        for (int s = 0; s < KP; ++s) {
            const bool c = x > v[s];
            const float tv = c ? v[s] : x;
            const int ti = c ? i[s] : ix;
            v[s] = c ? x : v[s];
            i[s] = c ? ix : i[s];
            x = tv;
            ix = ti;
        }
    }

    // Insert with the full comparator (arrival order arbitrary).
    __device__ __forceinline__ void insert(float x, int ix)
    {
#pragma unroll
        for (int s = 0; s < KP; ++s) {
            const bool c = better(x, ix, v[s], i[s]);
            const float tv = c ? v[s] : x;
            const int ti = c ? i[s] : ix;
            v[s] = c ? x : v[s];
            i[s] = c ? ix : i[s];
            x = tv;
            ix = ti;
        }
    }

    __device__ __forceinline__ void pop()
    {
#pragma unroll
        for (int s = 0; s + 1 < KP; ++s) {
            v[s] = v[s + 1];
            i[s] = i[s + 1];
        }
        v[KP - 1] = neg_inf();
        i[KP - 1] = kIdxNone;
    }
};

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        x = fmaxf(x, __shfl_xor(x, off, kWave));
    return x;
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        x += __shfl_xor(x, off, kWave);
    return x;
}

// Softmax partial (m, s) with s = sum exp(z - m) over some set; the empty set is (-inf, 0).
__device__ __forceinline__ void stat_add(float& m, float& s, float z)
{
    const float mn = fmaxf(m, z);
    if (mn > neg_inf()) {
        s = s * __expf(m - mn) + __expf(z - mn);
        m = mn;
    }
}

__device__ __forceinline__ void stat_merge(float& m, float& s, float m2, float s2)
{
    const float mn = fmaxf(m, m2);
    if (mn > neg_inf()) {
        s = s * __expf(m - mn) + s2 * __expf(m2 - mn);
        m = mn;
    }
}

// Combine the partials of the active lanes of a wave; every lane returns the result.
__device__ __forceinline__ void wave_stat_merge(float& m, float& s, bool active)
{
    const float mm = active ? m : neg_inf();
    const float M = wave_max(mm);
    const float t = (active && mm > neg_inf()) ? s * __expf(mm - M) : 0.0f;
    s = wave_sum(t);
    m = M;
}

// Merge the sorted lists of the active lanes of a wave.  On return lane q (q < KP) holds the
// q-th best candidate of the union in (outv, outi).  The lists of active lanes are consumed.
// Indices must be distinct across lists (empty slots carry kIdxNone with -inf).
template <int KP>
__device__ __forceinline__ void wave_merge(TopList<KP>& L, bool active, int lane, float& outv, int& outi)
{
    outv = neg_inf();
    outi = kIdxNone;
#pragma unroll 1
    for (int q = 0; q < KP; ++q) {
        const float hv = active ? L.v[0] : neg_inf();
        const int hi = active ? L.i[0] : kIdxNone;
        float bv = hv;
        int bi = hi;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off, kWave);
            const int oi = __shfl_xor(bi, off, kWave);
            if (better(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
        }
        if (active && hi == bi && hv == bv)
            L.pop();
        if (lane == q) {
            outv = bv;
            outi = bi;
        }
    }
}

// Sum NP per-lane values across the wave so that lane l ends with the total of value number
// p(l) = l >> (6 - log2 NP): each exchange halves the number of live values instead of
// running a full butterfly per value.  NP is a power of two <= 64.
template <int N, int OFF>
struct PairReduce {
    template <int NP>
    static __device__ __forceinline__ void run(float (&v)[NP], int lane)
    {
        constexpr int half = N / 2;
        const bool up = (lane & OFF) != 0;
#pragma unroll
        for (int i = 0; i < half; ++i) {
            const float keep = up ? v[i + half] : v[i];
            const float send = up ? v[i] : v[i + half];
            v[i] = keep + __shfl_xor(send, OFF, kWave);
        }
        PairReduce<half, OFF / 2>::run(v, lane);
    }
};
template <int OFF>
struct PairReduce<1, OFF> {
    template <int NP>
    static __device__ __forceinline__ void run(float (&v)[NP], int)
    {
        float z = v[0];
#pragma unroll
        for (int off = OFF; off >= 1; off >>= 1)
            z += __shfl_xor(z, off, kWave);
        v[0] = z;
    }
};
template <>
struct PairReduce<1, 0> {
    template <int NP>
    static __device__ __forceinline__ void run(float (&)[NP], int) {}
};

template <int NP>
__device__ __forceinline__ float reduce_pairs(float (&v)[NP], int lane)
{
    PairReduce<NP, 32>::run(v, lane);
    return v[0];
}

constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x >> 1); }

// bf16 pair packed in a 32-bit word -> two fp32 values (exact widening).
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

}  // namespace vt
