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
constexpr int kHistProbes = 2;  // neighbouring slots tried before a token goes to memory (1: 331 us, 2: 274 us, 4: 277 us on 33.5 M tokens)

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
        bool done = false;
#pragma unroll
        for (int pr = 0; pr < kHistProbes; ++pr) {
            if (!done && try_slot(slot ^ pr, t)) {
                atomicAdd(&tab_cnt[slot ^ pr], 1u);
                done = true;
            }
        }
        if (!done)
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

// Long streams over a vocabulary of at most kRangeClasses * kRangeBins ids: the ids are cut into
// classes of kRangeBins consecutive ids, a workgroup owns one class and one slice of the stream and
// counts its class in a plain LDS histogram (no tags, no probing, one LDS atomic per token of the
// class; the other tokens are dropped).  Every slice is read by one workgroup per class; they are
// neighbours in launch order and sit on the same XCD (block number modulo 8), so the slice comes
// from HBM once and from that XCD's L2 for the rest.
constexpr int kRangeBins = 32768;   // 128 KiB of LDS
constexpr int kRangeClasses = 8;
constexpr int64_t kRangeMinTokens = 1 << 20;

__global__ void __launch_bounds__(kHistThreads) hist_range_kernel(const int32_t* __restrict__ tokens, int64_t n, int V,
                                                                  int ncls, uint32_t* __restrict__ freq,
                                                                  int* __restrict__ err)
{
    extern __shared__ int hist_lds[];
    uint32_t* bins = reinterpret_cast<uint32_t*>(hist_lds);
    for (int i = threadIdx.x; i < kRangeBins; i += kHistThreads)
        bins[i] = 0u;
    __syncthreads();
    const int nslices = gridDim.x / ncls;
    int cls, slice;
    if ((nslices & 7) == 0) {
        const int y = blockIdx.x >> 3;
        cls = y % ncls;
        slice = (y / ncls) * 8 + (blockIdx.x & 7);
    } else {
        cls = blockIdx.x % ncls;
        slice = blockIdx.x / ncls;
    }
    const int base = cls * kRangeBins;
    const bool checks = cls == 0;  // the class-0 workgroup of a slice reports ids outside [0, V)
    bool bad = false;
    auto count = [&](int t) {
        const unsigned int u = (unsigned int)(t - base);
        if (u < (unsigned int)kRangeBins && t < V)
            atomicAdd(&bins[u], 1u);
        if (checks)
            bad |= (t < 0 || t >= V);
    };
    const int64_t per = ((n + nslices - 1) / nslices + 3) & ~(int64_t)3;  // whole 16-byte pieces per slice
    const int64_t lo = (int64_t)slice * per;
    const int64_t hi = lo + per < n ? lo + per : n;
    if (lo < hi) {
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        const i32x4* t4 = reinterpret_cast<const i32x4*>(tokens);
        const int64_t a1 = hi & ~(int64_t)3;
        for (int64_t i = (lo >> 2) + threadIdx.x; i < (a1 >> 2); i += kHistThreads) {
            const i32x4 q = t4[i];
            count(q.x);
            count(q.y);
            count(q.z);
            count(q.w);
        }
        for (int64_t i = a1 + threadIdx.x; i < hi; i += kHistThreads)
            count(tokens[i]);
    }
    if (bad)
        atomicOr(err, 1);
    __syncthreads();
    for (int i = threadIdx.x; i < kRangeBins; i += kHistThreads) {
        const uint32_t c = bins[i];
        if (c != 0u)
            atomicAdd(&freq[base + i], c);
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

// The passes over the V sorted keys are spread over up to kSegBlocks workgroups: workgroup b owns
// the contiguous segment [b*seg, (b+1)*seg) of ranks (seg a multiple of 1024), walked in tiles
// of 1024 (thread = rank within the tile: coalesced loads).  Cross-workgroup prefixes come from
// a small array of per-segment sums written by a first kernel.
constexpr int kScanWaves = kScanThreads / 64;
constexpr int kSegBlocks = 256;

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

// Sum of one value per thread over the workgroup; every thread returns it.  `scratch` has
// kScanWaves entries and may be reused after the call.
__device__ __forceinline__ unsigned long long block_sum_u64(unsigned long long x, unsigned long long* scratch)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const unsigned long long w = __shfl(wave_incl_scan_u64(x, lane), 63, 64);
    __syncthreads();
    if (lane == 0)
        scratch[wave] = w;
    __syncthreads();
    unsigned long long tot = 0;
    for (int i = 0; i < kScanWaves; ++i)
        tot += scratch[i];
    return tot;
}

struct BlockBest {
    double u;       // penalised utility
    long long k;
    double C, R, U;
    int feasible;
};

// pass 1: the ranking, and the sum of the frequencies of every segment
__global__ void __launch_bounds__(kScanThreads) rank_sums_kernel(const uint64_t* __restrict__ keys, int V, int seg,
                                                                 int32_t* __restrict__ rank_ids,
                                                                 unsigned long long* __restrict__ seg_sum)
{
    __shared__ unsigned long long scratch[kScanWaves];
    const int r0 = blockIdx.x * seg;
    const int r1 = r0 + seg < V ? r0 + seg : V;
    unsigned long long sum = 0;
    for (int r = r0 + threadIdx.x; r < r1; r += kScanThreads) {
        const uint64_t key = keys[r];
        sum += key >> 32;
        rank_ids[r] = (int32_t)(0xFFFFFFFFu - (uint32_t)key);
    }
    sum = block_sum_u64(sum, scratch);
    if (threadIdx.x == 0)
        seg_sum[blockIdx.x] = sum;
}

// pass 2: prefix sums, Eq. 2-5 at every k of the range, and the segment's best k
__global__ void __launch_bounds__(kScanThreads) utility_kernel(const uint64_t* __restrict__ keys, int V, int seg,
                                                               SelectParams prm,
                                                               const unsigned long long* __restrict__ seg_sum,
                                                               BlockBest* __restrict__ seg_best)
{
#pragma clang fp contract(off)
    __shared__ unsigned long long scratch[kScanWaves];
    __shared__ Best best_s[kScanThreads];
    __shared__ int feas_s;
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int nseg = gridDim.x;
    if (t == 0)
        feas_s = 0;
    // frequencies before this segment, and in all segments
    unsigned long long before = 0, all = 0;
    for (int i = t; i < nseg; i += kScanThreads) {
        const unsigned long long x = seg_sum[i];
        all += x;
        before += i < (int)blockIdx.x ? x : 0ull;
    }
    const unsigned long long total = block_sum_u64(all, scratch);
    unsigned long long carry = block_sum_u64(before, scratch);

    const double tot = (double)total;
    const double two_d = 2.0 * (double)prm.d;
    const double den = prm.F_fixed + two_d * (double)V;
    const double one_minus_alpha = 1.0 - prm.alpha;
    Best best = {-2.0, (long long)V + 1};  // below every penalised utility
    double best_C = 0.0, best_R = 0.0, best_U = 0.0;
    bool feas = false;
    const int r0 = blockIdx.x * seg;
    const int r1 = r0 + seg < V ? r0 + seg : V;
    for (int rb = r0; rb < r1; rb += kScanThreads) {
        const int r = rb + t;
        const unsigned long long cnt = r < r1 ? (unsigned long long)(keys[r] >> 32) : 0ull;
        // inclusive scan over the tile: within the wave, then the waves before this one
        const unsigned long long incl = wave_incl_scan_u64(cnt, lane);
        __syncthreads();
        if (lane == 63)
            scratch[wave] = incl;
        __syncthreads();
        unsigned long long wbefore = 0, tile = 0;
        for (int i = 0; i < kScanWaves; ++i) {
            const unsigned long long x = scratch[i];
            wbefore += i < wave ? x : 0ull;
            tile += x;
        }
        const unsigned long long prefix = carry + wbefore + incl;  // sum of the r+1 largest frequencies
        carry += tile;
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
                best_C = C;
                best_R = R;
                best_U = U;
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
    // the thread whose own best is the segment's best reports (a k belongs to one thread); a
    // segment outside the range reports the initial value, which loses against everything
    if (best.k == best_s[0].k && (best.k <= V || t == 0)) {
        BlockBest bb;
        bb.u = best.u;
        bb.k = best.k;
        bb.C = best_C;
        bb.R = best_R;
        bb.U = best_U;
        bb.feasible = feas_s;
        seg_best[blockIdx.x] = bb;
    }
}

// pass 3: the best over the segments
__global__ void __launch_bounds__(kSegBlocks) utility_final_kernel(const BlockBest* __restrict__ seg_best, int nseg,
                                                                   const unsigned long long* __restrict__ seg_sum,
                                                                   vt_selection* __restrict__ out)
{
    __shared__ Best best_s[kSegBlocks];
    __shared__ int feas_s;
    const int t = threadIdx.x;
    if (t == 0)
        feas_s = 0;
    __syncthreads();
    Best mine = {-3.0, (long long)1 << 62};
    if (t < nseg) {
        mine.u = seg_best[t].u;
        mine.k = seg_best[t].k;
        if (seg_best[t].feasible)
            atomicOr(&feas_s, 1);
    }
    best_s[t] = mine;
    __syncthreads();
    for (int off = kSegBlocks / 2; off > 0; off >>= 1) {
        if (t < off && beats(best_s[t + off], best_s[t]))
            best_s[t] = best_s[t + off];
        __syncthreads();
    }
    if (t < nseg && mine.k == best_s[0].k) {
        unsigned long long total = 0;
        for (int i = 0; i < nseg; ++i)
            total += seg_sum[i];
        out->k_star = mine.k;
        out->feasible = feas_s;
        out->C = seg_best[t].C;
        out->R = seg_best[t].R;
        out->U = seg_best[t].U;
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

// Workgroup b owns the ids [b*seg, (b+1)*seg); a ballot of the marks gives a tile's count and
// every marked lane's position.  First the counts per segment, then the writes.
__global__ void __launch_bounds__(kScanThreads) mark_count_kernel(const uint32_t* __restrict__ mark, int V, int seg,
                                                                  unsigned long long* __restrict__ seg_cnt)
{
    __shared__ unsigned long long scratch[kScanWaves];
    const int v0 = blockIdx.x * seg;
    const int v1 = v0 + seg < V ? v0 + seg : V;
    unsigned long long cnt = 0;
    for (int v = v0 + threadIdx.x; v < v1; v += kScanThreads)
        cnt += mark[v] != 0u ? 1u : 0u;
    cnt = block_sum_u64(cnt, scratch);
    if (threadIdx.x == 0)
        seg_cnt[blockIdx.x] = cnt;
}

__global__ void __launch_bounds__(kScanThreads) compact_kernel(const uint32_t* __restrict__ mark, int V, int seg,
                                                               const unsigned long long* __restrict__ seg_cnt,
                                                               int32_t* __restrict__ token_ids)
{
    __shared__ unsigned long long scratch[kScanWaves];
    __shared__ unsigned int wcnt[kScanWaves];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    unsigned long long before = 0;
    for (int i = t; i < (int)blockIdx.x; i += kScanThreads)
        before += seg_cnt[i];
    unsigned int pos = (unsigned int)block_sum_u64(before, scratch);
    const int v0 = blockIdx.x * seg;
    const int v1 = v0 + seg < V ? v0 + seg : V;
    for (int vb = v0; vb < v1; vb += kScanThreads) {
        const int v = vb + t;
        const bool m = v < v1 && mark[v] != 0u;
        const unsigned long long b = __ballot(m);
        __syncthreads();
        if (lane == 0)
            wcnt[wave] = (unsigned int)__popcll(b);
        __syncthreads();
        unsigned int wbefore = 0, tile = 0;
        for (int i = 0; i < kScanWaves; ++i) {
            wbefore += i < wave ? wcnt[i] : 0u;
            tile += wcnt[i];
        }
        if (m)
            token_ids[pos + wbefore + (unsigned int)__popcll(b & ((1ull << lane) - 1ull))] = v;
        pos += tile;
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
    L.off_seg = L.off_result + 256;
    L.off_err = L.off_seg + up((size_t)kSegBlocks * (2 * sizeof(unsigned long long) + sizeof(BlockBest)));
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
    const int ncls = (V + kRangeBins - 1) / kRangeBins;
    if (n >= kRangeMinTokens && ncls <= kRangeClasses) {
        constexpr size_t range_lds = (size_t)kRangeBins * sizeof(uint32_t);
        static std::atomic<bool> range_raised{false};
        if (!range_raised.load()) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(hist_range_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)range_lds);
            if (e != hipSuccess)
                return e;
            range_raised.store(true);
        }
        const int nslices = 256 / ncls / 8 * 8;  // a multiple of 8 slices: one workgroup per compute unit at most
        hipLaunchKernelGGL(hist_range_kernel, dim3((unsigned)(nslices * ncls)), dim3(kHistThreads), range_lds, s, tokens,
                           n, V, ncls, freq, err);
    } else {
        int64_t hb = (n + (int64_t)kHistThreads * 64 - 1) / ((int64_t)kHistThreads * 64);
        if (hb > 256)
            hb = 256;
        hipLaunchKernelGGL(hist_kernel, dim3((unsigned)hb), dim3(kHistThreads), hist_lds, s, tokens, n, V, freq, err);
    }

    hipLaunchKernelGGL(make_keys_kernel, dim3((L.N2 + 255) / 256), dim3(256), 0, s, freq, V, L.N2, keys);
    const int chunks = L.N2 / kSortChunk;
    hipLaunchKernelGGL(bitonic_local_kernel, dim3(chunks), dim3(kSortThreads), 0, s, keys, 2, kSortChunk);
    for (int size = 2 * kSortChunk; size <= L.N2; size <<= 1) {
        for (int stride = size >> 1; stride >= kSortChunk; stride >>= 1)
            hipLaunchKernelGGL(bitonic_global_kernel, dim3((L.N2 / 2 + 255) / 256), dim3(256), 0, s, keys, L.N2, size,
                               stride);
        hipLaunchKernelGGL(bitonic_local_kernel, dim3(chunks), dim3(kSortThreads), 0, s, keys, size, size);
    }
    // segments of whole 1024-rank tiles over at most kSegBlocks workgroups
    int seg = ((V + kSegBlocks - 1) / kSegBlocks + kScanThreads - 1) / kScanThreads * kScanThreads;
    const int nseg = (V + seg - 1) / seg;
    unsigned long long* seg_sum = reinterpret_cast<unsigned long long*>(ws + L.off_seg);
    unsigned long long* seg_cnt = seg_sum + kSegBlocks;
    BlockBest* seg_best = reinterpret_cast<BlockBest*>(seg_cnt + kSegBlocks);
    hipLaunchKernelGGL(rank_sums_kernel, dim3(nseg), dim3(kScanThreads), 0, s, keys, V, seg, rank_ids, seg_sum);
    hipLaunchKernelGGL(utility_kernel, dim3(nseg), dim3(kScanThreads), 0, s, keys, V, seg, prm, seg_sum, seg_best);
    hipLaunchKernelGGL(utility_final_kernel, dim3(1), dim3(kSegBlocks), 0, s, seg_best, nseg, seg_sum, res);
    hipLaunchKernelGGL(mark_kernel, dim3((V + 255) / 256), dim3(256), 0, s, rank_ids, res, mark, V);
    hipLaunchKernelGGL(mark_count_kernel, dim3(nseg), dim3(kScanThreads), 0, s, mark, V, seg, seg_cnt);
    hipLaunchKernelGGL(compact_kernel, dim3(nseg), dim3(kScanThreads), 0, s, mark, V, seg, seg_cnt, token_ids);
    return hipGetLastError();
}

}  // namespace vt
