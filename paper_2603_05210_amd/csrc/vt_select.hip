// Draft-vocabulary size selection on the device (Section 2 of the paper, Eq. 1-5):
//   f(v)  token frequencies over a stream of token ids                        (Section 2.2)
//   top-k the k most frequent tokens; equal frequencies: lower token id first
//   C(k) = sum_{top-k} f / sum f (Eq. 2), R(k) = 1 - (F_fixed + 2dk)/(F_fixed + 2dV) (Eq. 3),
//   U(k) = alpha C + (1 - alpha) R (Eq. 4), U~(k) = U(k) if C(k) >= c_min else -1 (Eq. 5),
//   k* = argmax over [k_min, k_max] of U~ (Eq. 1), smallest k among equals.
// The paper samples k with TPE (Section 2.5); the exact arg-max over every k of the range is
// what that search approximates and costs one pass over V values here.
//
// Kernels: a privatised histogram over the token stream (the only part that scales with the
// corpus), a bitonic sort of V 64-bit keys (frequency high, inverted id low), and single-
// workgroup passes for the prefix sums / utility / arg-max and for the ascending id list.
// The utility is evaluated in IEEE double, one rounding per operation in a fixed order
// (no contraction), so the arg-max is reproducible bit for bit.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "vt.h"
#include "vt_select.h"

namespace vt {

// ------------------------------------------------------------------ histogram
// Token frequencies are heavy-tailed, so plain global atomics would serialise on a few
// addresses.  Each workgroup keeps an open-addressed table of kHistSlots (id, count) pairs in
// LDS: a token whose slot is free or already its own is counted there, the rest go to memory;
// the table is flushed once at the end.
constexpr int kHistThreads = 1024;
constexpr int kHistSlots = 16384;  // 128 KiB of LDS: one workgroup per compute unit
constexpr int kHistEmpty = -1;

__global__ void __launch_bounds__(kHistThreads) hist_kernel(const int32_t* __restrict__ tokens, int64_t n, int V,
                                                            uint32_t* __restrict__ freq, int* __restrict__ err)
{
    extern __shared__ int hist_lds[];
    int* tab_id = hist_lds;
    uint32_t* tab_cnt = reinterpret_cast<uint32_t*>(hist_lds + kHistSlots);
    for (int i = threadIdx.x; i < kHistSlots; i += kHistThreads) {
        tab_id[i] = kHistEmpty;
        tab_cnt[i] = 0u;
    }
    __syncthreads();
    // claim-or-match at a slot: true when the token may be counted there
    auto try_slot = [&](int slot, int t) {
        int owner = tab_id[slot];
        if (owner == kHistEmpty)
            owner = atomicCAS(&tab_id[slot], kHistEmpty, t);
        return owner == kHistEmpty || owner == t;
    };
    auto count = [&](int t) {
        if (t < 0 || t >= V) {
            atomicOr(err, 1);
            return;
        }
        const int slot = (int)(((uint32_t)t * 2654435761u) >> 18);  // top 14 bits of a multiplicative hash
        if (try_slot(slot, t))
            atomicAdd(&tab_cnt[slot], 1u);
        else if (try_slot(slot ^ 1, t))
            atomicAdd(&tab_cnt[slot ^ 1], 1u);
        else
            atomicAdd(&freq[t], 1u);
    };
    // a contiguous share per workgroup, 128-bit loads over its aligned middle
    const int64_t per = (n + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * per;
    const int64_t hi = lo + per < n ? lo + per : n;
    if (lo < hi) {
        const int64_t a0 = (lo + 3) & ~(int64_t)3;  // tokens is 16-byte aligned: multiples of 4 are aligned
        const int64_t a1 = hi & ~(int64_t)3;
        if (a0 < a1) {
            for (int64_t i = lo + threadIdx.x; i < a0; i += kHistThreads)
                count(tokens[i]);
            typedef int i32x4 __attribute__((ext_vector_type(4)));
            const i32x4* t4 = reinterpret_cast<const i32x4*>(tokens);
            for (int64_t i = (a0 >> 2) + threadIdx.x; i < (a1 >> 2); i += kHistThreads) {
                const i32x4 q = __builtin_nontemporal_load(t4 + i);
                count(q.x);
                count(q.y);
                count(q.z);
                count(q.w);
            }
            for (int64_t i = a1 + threadIdx.x; i < hi; i += kHistThreads)
                count(tokens[i]);
        } else {
            for (int64_t i = lo + threadIdx.x; i < hi; i += kHistThreads)
                count(tokens[i]);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kHistSlots; i += kHistThreads) {
        const uint32_t c = tab_cnt[i];
        if (c != 0u)
            atomicAdd(&freq[tab_id[i]], c);
    }
}

// ------------------------------------------------------------------ sort by (frequency desc, id asc)
// key = frequency << 32 | (0xFFFFFFFF - id): descending keys are the wanted order; padding
// keys are 0 and sink to the end (a real key is never 0: its low word is >= 0x80000000).
constexpr int kSortThreads = 1024;
constexpr int kSortChunk = 4096;  // keys a workgroup sorts in LDS (32 KiB)

__global__ void make_keys_kernel(const uint32_t* __restrict__ freq, int V, int N2, uint64_t* __restrict__ keys)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N2)
        keys[i] = (i < V) ? (((uint64_t)freq[i] << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)i)) : 0ull;
}

// compare-exchange of positions i < j (global indices) in a bitonic network that ends descending
__device__ __forceinline__ void cmpx(uint64_t& a, uint64_t& b, bool descending)
{
    const bool swap = descending ? (a < b) : (a > b);
    if (swap) {
        const uint64_t t = a;
        a = b;
        b = t;
    }
}

// Runs the steps (size, stride) with stride < kSortChunk on a chunk held in LDS: every size
// from size_lo up to size_hi (size_lo == size_hi for the tail of a larger merge).
__global__ void __launch_bounds__(kSortThreads) bitonic_local_kernel(uint64_t* __restrict__ keys, int size_lo,
                                                                     int size_hi)
{
    __shared__ uint64_t s[kSortChunk];
    const int base = blockIdx.x * kSortChunk;
    for (int i = threadIdx.x; i < kSortChunk; i += kSortThreads)
        s[i] = keys[base + i];
    __syncthreads();
    for (int size = size_lo; size <= size_hi; size <<= 1) {
        int stride = size >> 1;
        if (stride >= kSortChunk)
            stride = kSortChunk >> 1;
        for (; stride > 0; stride >>= 1) {
            for (int p = threadIdx.x; p < kSortChunk / 2; p += kSortThreads) {
                const int i = ((p & ~(stride - 1)) << 1) | (p & (stride - 1));  // the pair's lower position
                const int j = i + stride;
                const bool desc = ((base + i) & size) == 0;
                uint64_t a = s[i], b = s[j];
                cmpx(a, b, desc);
                s[i] = a;
                s[j] = b;
            }
            __syncthreads();
        }
    }
    for (int i = threadIdx.x; i < kSortChunk; i += kSortThreads)
        keys[base + i] = s[i];
}

__global__ void bitonic_global_kernel(uint64_t* __restrict__ keys, int N2, int size, int stride)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= N2 / 2)
        return;
    const int i = ((p & ~(stride - 1)) << 1) | (p & (stride - 1));
    const int j = i + stride;
    uint64_t a = keys[i], b = keys[j];
    cmpx(a, b, (i & size) == 0);
    keys[i] = a;
    keys[j] = b;
}

// ------------------------------------------------------------------ prefix sums, utility, arg-max
constexpr int kScanThreads = 1024;

struct Best {
    double u;
    long long k;
};
__device__ __forceinline__ bool beats(const Best& a, const Best& b)  // larger utility, then smaller k
{
    return a.u > b.u || (a.u == b.u && a.k < b.k);
}

// One workgroup of 16 waves.  Wave w owns a contiguous segment of ranks and walks it in tiles of
// 64 (lane = rank within the tile: coalesced 512-byte loads).  Pass 1 sums the segment's
// frequencies and writes the ranking; the 16 sums give every wave its starting prefix; pass 2
// scans each tile across the lanes, evaluates Eq. 2-5 at every k of the range and keeps the best.
constexpr int kScanWaves = kScanThreads / 64;

__device__ __forceinline__ unsigned long long wave_incl_scan_u64(unsigned long long x, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned long long y = __shfl_up(x, off, 64);
        if (lane >= off)
            x += y;
    }
    return x;
}

__global__ void __launch_bounds__(kScanThreads) utility_kernel(const uint64_t* __restrict__ keys, int V, SelectParams prm,
                                                               int32_t* __restrict__ rank_ids, vt_selection* __restrict__ out)
{
#pragma clang fp contract(off)
    __shared__ unsigned long long wsum[kScanWaves];
    __shared__ Best best_s[kScanThreads];
    __shared__ int feas_s;
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int seg = ((V + kScanWaves - 1) / kScanWaves + 63) & ~63;  // ranks per wave, whole tiles
    const int r0 = wave * seg < V ? wave * seg : V;
    const int r1 = r0 + seg < V ? r0 + seg : V;
    if (t == 0)
        feas_s = 0;

    constexpr int TB = 8;  // tiles fetched together: the loop is bound by load latency otherwise
    unsigned long long lsum = 0;
    for (int rb = r0; rb < r1; rb += 64 * TB) {
        uint64_t kb[TB];
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int r = rb + 64 * u + lane;
            kb[u] = r < r1 ? keys[r] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int r = rb + 64 * u + lane;
            if (r < r1) {
                lsum += kb[u] >> 32;
                rank_ids[r] = (int32_t)(0xFFFFFFFFu - (uint32_t)kb[u]);
            }
        }
    }
    const unsigned long long wtot = __shfl(wave_incl_scan_u64(lsum, lane), 63, 64);
    if (lane == 0)
        wsum[wave] = wtot;
    __syncthreads();
    unsigned long long carry = 0, total = 0;
    for (int w = 0; w < kScanWaves; ++w) {
        const unsigned long long x = wsum[w];
        carry += w < wave ? x : 0ull;
        total += x;
    }

    const double tot = (double)total;
    const double two_d = 2.0 * (double)prm.d;
    const double den = prm.F_fixed + two_d * (double)V;
    const double one_minus_alpha = 1.0 - prm.alpha;
    Best best = {-2.0, (long long)V + 1};  // below every penalised utility
    double best_C = 0.0, best_R = 0.0, best_U = 0.0;
    bool feas = false;
    for (int rb0 = r0; rb0 < r1; rb0 += 64 * TB) {
        uint64_t kb[TB];
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int r = rb0 + 64 * u + lane;
            kb[u] = r < r1 ? keys[r] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < TB; ++u) {
        const int r = rb0 + 64 * u + lane;
        const unsigned long long cnt = kb[u] >> 32;
        const unsigned long long incl = wave_incl_scan_u64(cnt, lane);
        const unsigned long long prefix = carry + incl;  // sum of the r+1 largest frequencies
        carry += __shfl(incl, 63, 64);
        const long long k = (long long)r + 1;
        if (r < r1 && k >= prm.k_min && k <= prm.k_max) {
            const double C = (double)prefix / tot;
            const double num = prm.F_fixed + two_d * (double)k;
            const double R = 1.0 - num / den;
            const double U = prm.alpha * C + one_minus_alpha * R;
            const bool ok = C >= prm.c_min;
            feas |= ok;
            const Best cand = {ok ? U : -1.0, k};
            if (beats(cand, best)) {
                best = cand;
                // C, R, U at the best k so far travel with it (reported below)
                best_C = C;
                best_R = R;
                best_U = U;
            }
        }
        }
    }
    if (feas)
        atomicOr(&feas_s, 1);
    best_s[t] = best;
    __syncthreads();
    for (int off = kScanThreads / 2; off > 0; off >>= 1) {
        if (t < off && beats(best_s[t + off], best_s[t]))
            best_s[t] = best_s[t + off];
        __syncthreads();
    }
    // the thread whose own best is the overall best reports (k is unique to one thread)
    if (best.k == best_s[0].k) {
        out->k_star = best.k;
        out->feasible = feas_s;
        out->C = best_C;
        out->R = best_R;
        out->U = best_U;
        out->n_tokens = total;
    }
}

// ------------------------------------------------------------------ the selected ids, ascending
__global__ void mark_kernel(const int32_t* __restrict__ rank_ids, const vt_selection* __restrict__ sel,
                            uint32_t* __restrict__ mark, int V)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < V)
        mark[rank_ids[r]] = (r < sel->k_star) ? 1u : 0u;
}

// One workgroup; wave w owns a contiguous segment of ids, tiles of 64: a ballot of the marks
// gives both the tile's count and every marked lane's position.
__global__ void __launch_bounds__(kScanThreads) compact_kernel(const uint32_t* __restrict__ mark, int V,
                                                               int32_t* __restrict__ token_ids)
{
    __shared__ unsigned int wcnt[kScanWaves];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int seg = ((V + kScanWaves - 1) / kScanWaves + 63) & ~63;
    const int v0 = wave * seg < V ? wave * seg : V;
    const int v1 = v0 + seg < V ? v0 + seg : V;
    constexpr int TB = 8;  // tiles fetched together
    unsigned int cnt = 0;
    for (int vb = v0; vb < v1; vb += 64 * TB) {
        uint32_t mb[TB];
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int v = vb + 64 * u + lane;
            mb[u] = v < v1 ? mark[v] : 0u;
        }
#pragma unroll
        for (int u = 0; u < TB; ++u)
            cnt += (unsigned int)__popcll(__ballot(mb[u] != 0u));
    }
    if (lane == 0)
        wcnt[wave] = cnt;
    __syncthreads();
    unsigned int pos = 0;
    for (int w = 0; w < wave; ++w)
        pos += wcnt[w];
    for (int vb = v0; vb < v1; vb += 64 * TB) {
        uint32_t mb[TB];
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int v = vb + 64 * u + lane;
            mb[u] = v < v1 ? mark[v] : 0u;
        }
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const bool m = mb[u] != 0u;
            const unsigned long long b = __ballot(m);
            if (m)
                token_ids[pos + (unsigned int)__popcll(b & ((1ull << lane) - 1ull))] = vb + 64 * u + lane;
            pos += (unsigned int)__popcll(b);
        }
    }
}

// ------------------------------------------------------------------ host side
static int next_pow2_at_least(int x, int lo)
{
    int p = lo;
    while (p < x)
        p <<= 1;
    return p;
}

SelectLayout select_layout(int64_t V)
{
    SelectLayout L;
    L.N2 = next_pow2_at_least((int)V, kSortChunk);
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    L.off_keys = 0;
    L.off_mark = up((size_t)L.N2 * sizeof(uint64_t));
    L.off_result = L.off_mark + up((size_t)V * sizeof(uint32_t));
    L.off_err = L.off_result + 256;
    L.total = L.off_err + 256;
    return L;
}

hipError_t launch_select(const int32_t* tokens, int64_t n, int V, const SelectParams& prm, uint32_t* freq,
                         int32_t* rank_ids, int32_t* token_ids, char* ws, const SelectLayout& L, hipStream_t s)
{
    uint64_t* keys = reinterpret_cast<uint64_t*>(ws + L.off_keys);
    uint32_t* mark = reinterpret_cast<uint32_t*>(ws + L.off_mark);
    vt_selection* res = reinterpret_cast<vt_selection*>(ws + L.off_result);
    int* err = reinterpret_cast<int*>(ws + L.off_err);

    hipError_t e = hipMemsetAsync(freq, 0, (size_t)V * sizeof(uint32_t), s);
    if (e != hipSuccess)
        return e;
    e = hipMemsetAsync(err, 0, sizeof(int), s);
    if (e != hipSuccess)
        return e;
    // one workgroup per compute unit (128 KiB of LDS each), fewer for short streams
    constexpr size_t hist_lds = (size_t)kHistSlots * 8;
    static std::atomic<bool> lds_raised{false};
    if (!lds_raised.load()) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(hist_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)hist_lds);
        if (e != hipSuccess)
            return e;
        lds_raised.store(true);
    }
    int64_t hb = (n + (int64_t)kHistThreads * 64 - 1) / ((int64_t)kHistThreads * 64);
    if (hb > 256)
        hb = 256;
    hipLaunchKernelGGL(hist_kernel, dim3((unsigned)hb), dim3(kHistThreads), hist_lds, s, tokens, n, V, freq, err);

    hipLaunchKernelGGL(make_keys_kernel, dim3((L.N2 + 255) / 256), dim3(256), 0, s, freq, V, L.N2, keys);
    const int chunks = L.N2 / kSortChunk;
    hipLaunchKernelGGL(bitonic_local_kernel, dim3(chunks), dim3(kSortThreads), 0, s, keys, 2, kSortChunk);
    for (int size = 2 * kSortChunk; size <= L.N2; size <<= 1) {
        for (int stride = size >> 1; stride >= kSortChunk; stride >>= 1)
            hipLaunchKernelGGL(bitonic_global_kernel, dim3((L.N2 / 2 + 255) / 256), dim3(256), 0, s, keys, L.N2, size,
                               stride);
        hipLaunchKernelGGL(bitonic_local_kernel, dim3(chunks), dim3(kSortThreads), 0, s, keys, size, size);
    }
    hipLaunchKernelGGL(utility_kernel, dim3(1), dim3(kScanThreads), 0, s, keys, V, prm, rank_ids, res);
    hipLaunchKernelGGL(mark_kernel, dim3((V + 255) / 256), dim3(256), 0, s, rank_ids, res, mark, V);
    hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(kScanThreads), 0, s, mark, V, token_ids);
    return hipGetLastError();
}

}  // namespace vt
