// Streaming regime of the draft head (1..16 hidden-state rows): the projection of Section
// 2.3 of the paper, z[r,j] = sum_i h[r,i] W_sub[j,i], is bound by reading W_sub once from
// HBM (2*H*V_draft bytes, the same number as the paper's 2dk FLOP count), so the kernel is a
// row-split dot product.
//
// A workgroup of 16 waves owns a contiguous range of at most kGemvMaxRowsPerBlock W_sub rows.
// A wave reads J consecutive rows at a time, one coalesced 128-bit load per lane per KiB,
// multiplies them against the hidden states held in LDS (bf16 pairs through v_dot2_f32_bf16,
// fp32 accumulation) and reduces across its 64 lanes on the VALU (DPP / permlane swaps).  The
// logits of the range are parked in LDS, never in memory (except in the test hook).  When the
// range is done, wave r reduces hidden-state row r: softmax statistics and the k best logits
// of the range by k rounds of a wave-wide arg-max under the (logit, lower index) order.  One
// partial per (row, workgroup) goes to the merge kernel.
#include <atomic>
#include <type_traits>

#include "vt_device.h"
#include "vt_internal.h"

namespace vt {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct GemvArgs {
    const u32x4* h;
    const u32x4* W;
    int rows, nchunk, Vd, P, k, KP, rpb;  // rpb: W_sub rows per workgroup (multiple of J)
    float* part_val;
    int32_t* part_idx;
    float2* part_stat;
    float* logits_out;
    // fused final merge (done by the last workgroup to finish) -- used when `fused` is set
    int fused, ticket_slot;
    const int32_t* d2t;
    int32_t* out_ids;
    float* out_logp;
    float* lse_out;
};

// Arrival counters for the fused merge, one per in-flight call (the host hands out slots
// round-robin); zero when idle: the last workgroup of a call puts its slot back to zero.
//
// No cache-wide fences are used: the partial results are a few hundred bytes per workgroup and
// travel through device-coherent accesses (relaxed agent-scope atomics: they bypass the
// per-XCD caches), ordered by "stores acknowledged -> workgroup barrier -> ticket".
constexpr int kTicketSlots = 1024;
__device__ __forceinline__ void st_dev(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev(int* p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_dev(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ int ld_dev(const int* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
static __device__ unsigned int g_ticket[kTicketSlots];

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
            a.out_logp[(size_t)row * a.k + lane] = ov - lse;
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

template <int NR, int J, bool DOT2>
__global__ void __launch_bounds__(kGemvThreads) gemv_head_kernel(GemvArgs a)
{
    constexpr int NP = NR * J;      // (hidden row, W_sub row) pairs reduced together
    constexpr int CL = kWave / NP;  // lanes that end up holding the same pair
    static_assert(kGemvMaxRowsPerBlock <= 8 * kWave, "at most 8 logits per lane in the selection");
    static_assert(NP <= kWave && (NP & (NP - 1)) == 0, "pairs per group must be a power of two <= 64");
    static_assert(NR <= kGemvWaves, "one wave per hidden-state row in the selection");
    extern __shared__ u32x4 smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nchunk = a.nchunk;
    float* zbuf = reinterpret_cast<float*>(smem + NR * nchunk);  // [NR][rpb]

    const int p_l = (NP > 1) ? (lane >> (6 - ilog2(NP))) : 0;  // pair this lane ends up with
    const int r_l = p_l / J;
    const int jj_l = p_l - r_l * J;
    const bool owner = (lane & (CL - 1)) == 0;

    const int j_lo = blockIdx.x * a.rpb;
    const int j_hi = (j_lo + a.rpb < a.Vd) ? j_lo + a.rpb : a.Vd;
    const int n_local = j_hi - j_lo;
    const int ngroups = (n_local + J - 1) / J;

    // The wave walks positions (group g of J rows, 1 KiB column step t) in order and keeps the
    // loads of the next position in flight while it multiplies the current one, also across
    // the boundary between two groups.
    const int T = (nchunk + kWave - 1) / kWave;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    auto load_pos = [&](int gg, int tt, u32x4(&buf)[J]) {
        const int c = lane + tt * kWave;
        const int j0 = j_lo + gg * J;
#pragma unroll
        for (int jj = 0; jj < J; ++jj) {
            const int j = (j0 + jj < a.Vd) ? j0 + jj : a.Vd - 1;
            buf[jj] = (c < nchunk) ? __builtin_nontemporal_load(a.W + (size_t)j * nchunk + c) : zero4;
        }
    };
    float acc[NR][J];
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int jj = 0; jj < J; ++jj)
            acc[r][jj] = 0.0f;

    int g = wave, t = 0;
    auto step = [&](u32x4(&cur)[J], u32x4(&nxt)[J]) {
        int tn = t + 1, gn = g;
        if (tn == T) {
            tn = 0;
            gn = g + kGemvWaves;
        }
        if (gn < ngroups)
            load_pos(gn, tn, nxt);
        int c = lane + t * kWave;
        c = c < nchunk ? c : nchunk - 1;  // lanes past the row end hold zeros in cur
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const u32x4 x = smem[r * nchunk + c];
#pragma unroll
            for (int jj = 0; jj < J; ++jj)
                acc[r][jj] = dot8<DOT2>(cur[jj], x, acc[r][jj]);
        }
        if (t == T - 1) {
            float pv[NP];
#pragma unroll
            for (int r = 0; r < NR; ++r)
#pragma unroll
                for (int jj = 0; jj < J; ++jj) {
                    pv[r * J + jj] = acc[r][jj];
                    acc[r][jj] = 0.0f;
                }
            const float z = reduce_pairs<NP>(pv, lane);
            const int j = j_lo + g * J + jj_l;
            if (owner && j < j_hi && r_l < a.rows) {
                zbuf[r_l * a.rpb + (j - j_lo)] = z;
                if (a.logits_out != nullptr)
                    a.logits_out[(size_t)r_l * a.Vd + j] = z;
            }
        }
        t = tn;
        g = gn;
    };
    u32x4 bufA[J], bufB[J];
    if (g < ngroups)
        load_pos(g, 0, bufA);  // the first W_sub loads are in flight while the hidden states are staged

    // hidden states -> LDS (rows beyond `rows` repeat the last one; their results are dropped)
    for (int x = tid; x < NR * nchunk; x += kGemvThreads) {
        const int r = x / nchunk;
        const int c = x - r * nchunk;
        const int rr = r < a.rows ? r : a.rows - 1;
        smem[x] = a.h[(size_t)rr * nchunk + c];
    }
    __syncthreads();
    while (g < ngroups) {
        step(bufA, bufB);
        if (g >= ngroups)
            break;
        step(bufB, bufA);
    }
    __syncthreads();

    // ---- selection over this workgroup's range: wave r handles hidden-state row r ----
    if (wave < a.rows) {
        const int r = wave;
        float m = 0.0f, s = 0.0f;
        float outv = neg_inf();
        int outi = kIdxNone;
        // VPL = logits per lane: the smallest of 1, 2, 4, 8 that covers the workgroup's range
        auto select = [&](auto vpl_c) {
            constexpr int VPL = decltype(vpl_c)::value;
            // lane l takes logits l*VPL .. l*VPL+VPL-1 of the range: lane order is index order
            float v[VPL];
            float mloc = neg_inf();
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                const int e = lane * VPL + i;
                v[i] = (e < n_local) ? zbuf[r * a.rpb + e] : neg_inf();
                mloc = fmaxf(mloc, v[i]);
            }
            m = wave_max(mloc);
            float sloc = 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i)
                sloc += __expf(v[i] - m);  // n_local >= 1, so m is finite
            s = wave_sum(sloc);

            // k rounds of a wave-wide arg-max on order-preserving integer keys
            int kv[VPL];
#pragma unroll
            for (int i = 0; i < VPL; ++i)
                kv[i] = f2key(v[i]);
            int outk = kKeyNone;
#pragma unroll 1
            for (int q = 0; q < a.k; ++q) {
                // best of this lane's logits: the first maximum has the lowest index
                int bk = kv[0];
                int bi = 0;
#pragma unroll
                for (int i = 1; i < VPL; ++i) {
                    const bool c = kv[i] > bk;
                    bk = c ? kv[i] : bk;
                    bi = c ? i : bi;
                }
                const int gi = (bk != kKeyNone) ? (j_lo + lane * VPL + bi) : kIdxNone;
                int wk, wi, winner;
                wave_best_ordered(bk, gi, wk, wi, winner);
                if (lane == q) {
                    outk = wk;
                    outi = wi;
                }
                // the owner retires the winner
                const int gone = (lane == winner) ? bi : -1;
#pragma unroll
                for (int i = 0; i < VPL; ++i)
                    kv[i] = (gone == i) ? kKeyNone : kv[i];
            }
            outv = key2f(outk);
        };
        const int per_lane = (a.rpb + kWave - 1) / kWave;
        if (per_lane <= 1)
            select(std::integral_constant<int, 1>{});
        else if (per_lane <= 2)
            select(std::integral_constant<int, 2>{});
        else if (per_lane <= 4)
            select(std::integral_constant<int, 4>{});
        else
            select(std::integral_constant<int, 8>{});
        const size_t slot = (size_t)r * a.P + blockIdx.x;
        if (lane < a.KP) {  // slots k..KP-1 carry the empty marker
            st_dev(a.part_val + slot * a.KP + lane, outv);
            st_dev(a.part_idx + slot * a.KP + lane, outi);
        }
        if (lane == 0) {
            st_dev(reinterpret_cast<float*>(a.part_stat + slot), m);
            st_dev(reinterpret_cast<float*>(a.part_stat + slot) + 1, s);
        }
        // vmcnt(0): this wave's coherent stores are acknowledged before it reaches the barrier
        // that precedes the ticket (expcnt / lgkmcnt fields left at their maxima)
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }

    if (!a.fused)
        return;
    // ---- fused final merge: the last workgroup to arrive finishes the call ----
    __shared__ int s_last;
    __syncthreads();
    if (tid == 0) {
        const unsigned int t =
            __hip_atomic_fetch_add(&g_ticket[a.ticket_slot], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (t == gridDim.x - 1) ? 1 : 0;
    }
    __syncthreads();
    if (!s_last)
        return;
    char* lds = reinterpret_cast<char*>(smem);
    switch (a.KP) {
    case 1: fused_final_merge<1>(a, lds, tid); break;
    case 2: fused_final_merge<2>(a, lds, tid); break;
    case 4: fused_final_merge<4>(a, lds, tid); break;
    case 8: fused_final_merge<8>(a, lds, tid); break;
    default: fused_final_merge<16>(a, lds, tid); break;
    }
    if (tid == 0)
        __hip_atomic_store(&g_ticket[a.ticket_slot], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int NR, int J, bool DOT2>
static hipError_t launch_one(const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    size_t lds = (size_t)NR * ga.nchunk * sizeof(u32x4) + (size_t)NR * ga.rpb * sizeof(float);
    if (ga.fused) {  // the fused merge parks up to 256 lists per row in LDS, plus per-wave statistics
        if (ga.rows > kFusedMaxRows || ga.P > 256 || ga.KP > 16)
            return hipErrorInvalidValue;
        const size_t l1 = (size_t)ga.rows * 256 * ((size_t)ga.KP + 1) * 8 + kGemvWaves * sizeof(float2);
        lds = lds > l1 ? lds : l1;
    }
    auto kern = gemv_head_kernel<NR, J, DOT2>;
    if (lds > (size_t)kGemvLdsLimit)
        return hipErrorInvalidValue;
    static size_t lds_allowed = 48 * 1024;  // per instantiation: raised once, then remembered
    if (lds > lds_allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return e;
        lds_allowed = lds;
    }
    hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(kGemvThreads), lds, s, ga);
    return hipGetLastError();
}

hipError_t launch_gemv(const Plan& p, const HeadArgs& a, hipStream_t s)
{
    GemvArgs ga;
    ga.h = reinterpret_cast<const u32x4*>(a.h);
    ga.W = reinterpret_cast<const u32x4*>(a.W);
    ga.rows = p.rows;
    ga.nchunk = p.H / 8;
    ga.Vd = p.Vd;
    ga.P = p.P;
    ga.k = p.k;
    ga.KP = p.KP;
    ga.rpb = p.rpb;
    ga.part_val = a.part_val;
    ga.part_idx = a.part_idx;
    ga.part_stat = a.part_stat;
    ga.logits_out = a.logits_out;
    ga.fused = p.fused;
    static std::atomic<unsigned int> next_slot{0};
    ga.ticket_slot = p.fused ? (int)(next_slot.fetch_add(1u) % (unsigned int)kTicketSlots) : 0;
    ga.d2t = a.d2t;
    ga.out_ids = a.out_ids;
    ga.out_logp = a.out_logp;
    ga.lse_out = a.lse_out;
    // rows of W_sub a wave reduces together (J): measured best 1 for a single hidden row, 2 otherwise
    switch (p.NR) {
    case 1: return launch_one<1, 1, true>(p, ga, s);
    case 2: return launch_one<2, 2, true>(p, ga, s);
    case 4: return launch_one<4, 2, true>(p, ga, s);
    case 8: return launch_one<8, 2, true>(p, ga, s);
    case 16: return launch_one<16, 2, true>(p, ga, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace vt
