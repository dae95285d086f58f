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

    // Bitonic sorting network over the KP slots (KP is a power of two): best first.
    template <int K, int J, int I>
    __device__ __forceinline__ void sort_step()
    {
        if constexpr (I < KP) {
            constexpr int l = I ^ J;
            if constexpr (l > I) {
                constexpr bool first_best = (I & K) == 0;
                const bool swap = first_best ? better(v[l], i[l], v[I], i[I]) : better(v[I], i[I], v[l], i[l]);
                const float tv = swap ? v[l] : v[I];
                const int ti = swap ? i[l] : i[I];
                v[l] = swap ? v[I] : v[l];
                i[l] = swap ? i[I] : i[l];
                v[I] = tv;
                i[I] = ti;
            }
            sort_step<K, J, I + 1>();
        }
    }
    template <int K, int J>
    __device__ __forceinline__ void sort_j()
    {
        if constexpr (J > 0) {
            sort_step<K, J, 0>();
            sort_j<K, J / 2>();
        }
    }
    template <int K>
    __device__ __forceinline__ void sort_k()
    {
        if constexpr (K <= KP) {
            sort_j<K, K / 2>();
            sort_k<K * 2>();
        }
    }
    __device__ __forceinline__ void sort() { sort_k<2>(); }

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

// ---- cross-lane exchange on the VALU (DPP / permlane swaps; no LDS round trip) ----
// xchg<OFF>(x) returns the value held by lane (l ^ OFF).  Lane mappings used (checked on
// gfx950): quad_perm for 1 and 2; quad reversal followed by row_half_mirror for 4;
// row_ror:8 for 8; v_permlane16_swap / v_permlane32_swap for 16 and 32.
template <int OFF>
__device__ __forceinline__ int xchg_i(int x, int lane)
{
    // (every lane has a source lane for distances 1, 2 and 8, so the plain DPP move serves: no
    // copy of the old value is needed)
    if constexpr (OFF == 1) {
        return __builtin_amdgcn_mov_dpp(x, 0xB1, 0xf, 0xf, true);
    } else if constexpr (OFF == 2) {
        return __builtin_amdgcn_mov_dpp(x, 0x4E, 0xf, 0xf, true);
    } else if constexpr (OFF == 4) {
        // l ^ 4 = (l ^ 3) ^ 7: reverse the quads, then mirror each half row of eight
        const int t = __builtin_amdgcn_mov_dpp(x, 0x1B, 0xf, 0xf, true);
        return __builtin_amdgcn_mov_dpp(t, 0x141, 0xf, 0xf, true);
    } else if constexpr (OFF == 8) {
        return __builtin_amdgcn_mov_dpp(x, 0x128, 0xf, 0xf, true);
    } else if constexpr (OFF == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        return (lane & 16) ? (int)r[0] : (int)r[1];
    } else {
        static_assert(OFF == 32, "exchange distance must be a power of two <= 32");
        const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
        return (lane & 32) ? (int)r[0] : (int)r[1];
    }
}
template <int OFF>
__device__ __forceinline__ float xchg_f(float x, int lane)
{
    return __int_as_float(xchg_i<OFF>(__float_as_int(x), lane));
}

// Order-preserving map of a (non-NaN) float onto int32: a > b <=> key(a) > key(b); -0 and +0
// share a key.  Integer max/min fold their DPP operand into one instruction and need no NaN
// quieting, so the arg-max rounds below run on keys.
__device__ __forceinline__ int f2key(float x)
{
    const int b = __float_as_int(x + 0.0f);
    return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float key2f(int k) { return __int_as_float(k ^ ((k >> 31) & 0x7fffffff)); }
constexpr int kKeyNone = (int)0x807fffff;  // key of -inf

// Reductions over the 16 lanes of a DPP row: pairs (quad_perm), quads, mirrored halves of 8,
// mirrored row.  Every lane returns the result.
__device__ __forceinline__ int row16_max_i(int x)
{
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0xB1, 0xf, 0xf, true));
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0x4E, 0xf, 0xf, true));
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0x141, 0xf, 0xf, true));
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0x140, 0xf, 0xf, true));
    return x;
}
__device__ __forceinline__ int row16_min_i(int x)
{
    x = min(x, __builtin_amdgcn_mov_dpp(x, 0xB1, 0xf, 0xf, true));
    x = min(x, __builtin_amdgcn_mov_dpp(x, 0x4E, 0xf, 0xf, true));
    x = min(x, __builtin_amdgcn_mov_dpp(x, 0x141, 0xf, 0xf, true));
    x = min(x, __builtin_amdgcn_mov_dpp(x, 0x140, 0xf, 0xf, true));
    return x;
}
__device__ __forceinline__ int wave_max_i(int x)
{
    x = row16_max_i(x);
    {
        const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        x = max((int)r[0], (int)r[1]);
    }
    {
        const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
        x = max((int)r[0], (int)r[1]);
    }
    return x;
}
__device__ __forceinline__ int wave_min_i(int x)
{
    x = row16_min_i(x);
    {
        const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        x = min((int)r[0], (int)r[1]);
    }
    {
        const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
        x = min((int)r[0], (int)r[1]);
    }
    return x;
}

__device__ __forceinline__ float wave_max(float x) { return key2f(wave_max_i(f2key(x))); }

// Sum over the wave; every lane returns the same bits (a fixed tree: xor 1, 2, 4, 8, 16, 32).
__device__ __forceinline__ float wave_sum(float x)
{
    const int lane = (int)__lane_id();
    x += xchg_f<1>(x, lane);
    x += xchg_f<2>(x, lane);
    x += xchg_f<4>(x, lane);
    x += xchg_f<8>(x, lane);
    {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_int(x), __float_as_int(x), false, false);
        x = __int_as_float(r[0]) + __int_as_float(r[1]);
    }
    {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
        x = __int_as_float(r[0]) + __int_as_float(r[1]);
    }
    return x;
}

// Best (logit, index) pair over the wave under the strict order; every lane returns it.
// Two cheap reductions instead of one over pairs: the largest logit, then the smallest index
// among the lanes that hold it.
__device__ __forceinline__ void wave_best_key(int& kv, int& i)
{
    const int bk = wave_max_i(kv);
    const int cand = (kv == bk) ? i : kIdxNone;
    i = wave_min_i(cand);
    kv = bk;
}
__device__ __forceinline__ void wave_best(float& v, int& i)
{
    int kv = f2key(v);
    wave_best_key(kv, i);
    v = key2f(kv);
}

// The same when lane order is index order (a lower lane never holds a higher index among
// equal keys): the best key comes back wave-uniform through four lane reads of the row maxima,
// and the winner is the lowest lane that holds it.  Needs all 64 lanes active.
__device__ __forceinline__ int wave_max_i_uniform(int x)
{
    x = row16_max_i(x);
    const int a = __builtin_amdgcn_readlane(x, 0);
    const int b = __builtin_amdgcn_readlane(x, 16);
    const int c = __builtin_amdgcn_readlane(x, 32);
    const int d = __builtin_amdgcn_readlane(x, 48);
    return max(max(a, b), max(c, d));
}
__device__ __forceinline__ void wave_best_ordered(int kv, int i, int& best_key, int& best_idx, int& winner)
{
    best_key = wave_max_i_uniform(kv);
    const unsigned long long tie = __ballot(kv == best_key);
    winner = (int)__builtin_ctzll(tie);
    best_idx = __builtin_amdgcn_readlane(i, winner);
}

// Softmax partial (m, s) with s = sum exp(z - m) over some set; the empty set is (-inf, 0).
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
__device__ __forceinline__ void wave_merge(TopList<KP>& L, bool active, int lane, float& outv, int& outi,
                                           int rounds = KP)
{
    outv = neg_inf();
    outi = kIdxNone;
#pragma unroll 1
    for (int q = 0; q < rounds; ++q) {
        const float hv = active ? L.v[0] : neg_inf();
        const int hi = active ? L.i[0] : kIdxNone;
        float bv = hv;
        int bi = hi;
        wave_best(bv, bi);
        if (active && hi == bi && hv == bv)
            L.pop();
        if (lane == q) {
            outv = bv;
            outi = bi;
        }
    }
}

// k-way merge by one wave of up to NSLOT*64 sorted candidate lists parked in LDS: list t
// occupies lv/li[t * (KP + 1) .. + KP) (odd stride: conflict-free column access), an empty list
// has the empty marker at its head.  A lane keeps only the current heads of its NSLOT lists in
// registers; a round takes the wave-wide best head and the owning lane advances that list's
// read position.  Candidate indices are distinct across lists, so exactly one lane owns the
// winner.  Lane q returns the q-th best (q < rounds).
//
// ORDERED: every index in list t is below every index in list t+1.  Lane l then looks after
// lists NSLOT*l .. NSLOT*l+NSLOT-1, ties resolve by position alone and the cheaper
// wave_best_ordered applies.  Otherwise lane l has lists l, l+64, ... and ties compare indices.
template <int KP, int NSLOT, bool ORDERED>
__device__ __forceinline__ void wave_walk_merge(const float* lv, const int* li, int nlists, int rounds, int lane,
                                                float& outv, int& outi)
{
    constexpr int S = KP + 1;
    int hk[NSLOT];  // heads as order-preserving keys
    int hi[NSLOT];
#pragma unroll
    for (int sl = 0; sl < NSLOT; ++sl) {
        const int t = ORDERED ? lane * NSLOT + sl : sl * kWave + lane;
        const bool ok = t < nlists;
        hk[sl] = ok ? f2key(lv[t * S]) : kKeyNone;
        hi[sl] = ok ? li[t * S] : kIdxNone;
    }
    int pos = 0;  // read positions of the NSLOT lists, 8 bits each
    int outk = kKeyNone;
    outi = kIdxNone;
#pragma unroll 1
    for (int q = 0; q < rounds; ++q) {
        int bk = hk[0];
        int bi = hi[0];
        int bs = 0;
#pragma unroll
        for (int sl = 1; sl < NSLOT; ++sl) {
            const bool c = ORDERED ? (hk[sl] > bk) : ((hk[sl] > bk) || (hk[sl] == bk && hi[sl] < bi));
            bk = c ? hk[sl] : bk;
            bi = c ? hi[sl] : bi;
            bs = c ? sl : bs;
        }
        int wk, wi;
        bool mine;
        if constexpr (ORDERED) {
            int winner;
            wave_best_ordered(bk, bi, wk, wi, winner);
            mine = lane == winner;
        } else {
            wk = bk;
            wi = bi;
            wave_best_key(wk, wi);
            mine = bi == wi;
        }
        if (lane == q) {
            outk = wk;
            outi = wi;
        }
        if (wi == kIdxNone)  // wave-uniform: nothing left anywhere
            break;
        if (mine) {
            pos += 1 << (8 * bs);
            const int np = (pos >> (8 * bs)) & 0xff;
            const int t = ORDERED ? lane * NSLOT + bs : bs * kWave + lane;
            int nk = kKeyNone;
            int ni = kIdxNone;
            if (np < KP) {
                nk = f2key(lv[t * S + np]);
                ni = li[t * S + np];
            }
#pragma unroll
            for (int sl = 0; sl < NSLOT; ++sl) {
                hk[sl] = (sl == bs) ? nk : hk[sl];
                hi[sl] = (sl == bs) ? ni : hi[sl];
            }
        }
    }
    outv = key2f(outk);
}

// ---- 64-bit order keys: a candidate (logit, draft index) as one integer, larger = better ----
// high word: the order-preserving key of the logit; low word: 0x7fffffff - index, so that of
// two equal logits the lower index is the larger key.  Distinct candidates have distinct keys
// (the empty marker, key of -inf with index kIdxNone, is the smallest of all and may repeat).
typedef long long k64;
__device__ __forceinline__ k64 k64_make(int key, int idx)
{
    return (k64)(((unsigned long long)(unsigned int)key << 32) | (unsigned int)(kIdxNone - idx));
}
__device__ __forceinline__ int k64_key(k64 x) { return (int)(x >> 32); }
__device__ __forceinline__ int k64_idx(k64 x) { return kIdxNone - (int)(unsigned int)x; }

__device__ __forceinline__ k64 k64_row_mirror(k64 x)  // lane q of a 16-lane row <- lane 15-q
{
    const int lo = __builtin_amdgcn_mov_dpp((int)(unsigned int)x, 0x140, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_mov_dpp((int)(x >> 32), 0x140, 0xf, 0xf, true);
    return (k64)(((unsigned long long)(unsigned int)hi << 32) | (unsigned int)lo);
}
template <int OFF>
__device__ __forceinline__ k64 k64_xchg(k64 x, int lane)  // value of lane l ^ OFF
{
    const int lo = xchg_i<OFF>((int)(unsigned int)x, lane);
    const int hi = xchg_i<OFF>((int)(x >> 32), lane);
    return (k64)(((unsigned long long)(unsigned int)hi << 32) | (unsigned int)lo);
}
// One stage of the bitonic sorter inside a 16-lane row: the lower lane of a pair keeps the
// larger key.
template <int OFF>
__device__ __forceinline__ k64 k64_stage(k64 c, int lane)
{
    const k64 p = k64_xchg<OFF>(c, lane);
    const bool lower = (lane & OFF) == 0;
    return ((p > c) == lower) ? p : c;
}
// a, b: lists of 16 keys sorted best first, one per 16-lane row (lane q holds the q-th).
// Returns the 16 best of their union, sorted best first: max(a, reversed b) is a bitonic
// sequence holding exactly those 16, which four compare-exchange stages sort.
__device__ __forceinline__ k64 k64_merge16(k64 a, k64 b, int lane)
{
    const k64 br = k64_row_mirror(b);
    k64 c = a > br ? a : br;
    c = k64_stage<8>(c, lane);
    c = k64_stage<4>(c, lane);
    c = k64_stage<2>(c, lane);
    c = k64_stage<1>(c, lane);
    return c;
}
// 16 sorted lists of 16 keys, stored back to back at `lists` (LDS), merged by one wave: every
// 16-lane row returns the 16 best of all 256, sorted best first.
__device__ __forceinline__ k64 k64_merge_16_lists(const k64* lists, int lane)
{
    const k64 s0 = lists[lane], s1 = lists[64 + lane], s2 = lists[128 + lane], s3 = lists[192 + lane];
    const k64 m01 = k64_merge16(s0, s1, lane);
    const k64 m23 = k64_merge16(s2, s3, lane);
    k64 m = k64_merge16(m01, m23, lane);          // row r now holds the best of lists r, 4+r, 8+r, 12+r
    m = k64_merge16(m, k64_xchg<16>(m, lane), lane);  // rows 0|1 and 2|3
    m = k64_merge16(m, k64_xchg<32>(m, lane), lane);  // all four rows
    return m;
}

// Largest key of the wave, in every lane.
__device__ __forceinline__ k64 k64_wave_max(k64 c, int lane)
{
    k64 p;
    p = k64_xchg<1>(c, lane), c = p > c ? p : c;
    p = k64_xchg<2>(c, lane), c = p > c ? p : c;
    p = k64_xchg<4>(c, lane), c = p > c ? p : c;
    p = k64_xchg<8>(c, lane), c = p > c ? p : c;
    p = k64_xchg<16>(c, lane), c = p > c ? p : c;
    p = k64_xchg<32>(c, lane), c = p > c ? p : c;
    return c;
}

// Sorts the 16 keys of every 16-lane row best first (bitonic sorting network, ten stages).
template <int S, int OFF>
__device__ __forceinline__ k64 k64_sort_stage(k64 c, int lane)
{
    const k64 p = k64_xchg<OFF>(c, lane);
    const bool lower = (lane & OFF) == 0;
    const bool desc = (lane & S) == 0 || S == 16;  // blocks alternate direction until the last pass
    return ((p > c) == (lower == desc)) ? p : c;
}
__device__ __forceinline__ k64 k64_row_sort16(k64 c, int lane)
{
    c = k64_sort_stage<2, 1>(c, lane);
    c = k64_sort_stage<4, 2>(c, lane);
    c = k64_sort_stage<4, 1>(c, lane);
    c = k64_sort_stage<8, 4>(c, lane);
    c = k64_sort_stage<8, 2>(c, lane);
    c = k64_sort_stage<8, 1>(c, lane);
    c = k64_sort_stage<16, 8>(c, lane);
    c = k64_sort_stage<16, 4>(c, lane);
    c = k64_sort_stage<16, 2>(c, lane);
    c = k64_sort_stage<16, 1>(c, lane);
    return c;
}

// ---- the same reduction inside one DPP row (16 consecutive lanes), DPP only ----
__device__ __forceinline__ float row16_max(float x) { return key2f(row16_max_i(f2key(x))); }

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
            v[i] = keep + xchg_f<OFF>(send, lane);
        }
        PairReduce<half, OFF / 2>::run(v, lane);
    }
};
template <int OFF>
struct PairReduce<1, OFF> {
    template <int NP>
    static __device__ __forceinline__ void run(float (&v)[NP], int lane)
    {
        float z = v[0];
        if constexpr (OFF >= 32) z += xchg_f<32>(z, lane);
        if constexpr (OFF >= 16) z += xchg_f<16>(z, lane);
        if constexpr (OFF >= 8) z += xchg_f<8>(z, lane);
        if constexpr (OFF >= 4) z += xchg_f<4>(z, lane);
        if constexpr (OFF >= 2) z += xchg_f<2>(z, lane);
        if constexpr (OFF >= 1) z += xchg_f<1>(z, lane);
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

// fp32 -> bf16 bit pattern, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

}  // namespace vt
