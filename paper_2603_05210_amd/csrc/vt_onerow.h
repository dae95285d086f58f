// The one-row draft step, generic over how W_sub is stored (bf16, FP8 E4M3 with a scale per
// row, MXFP4 with an exponent per 32 weights): the kernel template, its list-merge network
// and its launch-side constants.  vt_gemv1.hip instantiates it for bf16, vt_gemvq.hip for the
// compressed forms.
//
// The step (Section 2.3's projection over a few thousand to 128 K draft tokens for one hidden
// state) is bound by reading W_sub once, and at the vocabulary sizes the paper selects (Sections
// 2.6, 3.2) the whole read takes only a few microseconds, so everything around the stream is
// latency:
//
//   - a workgroup owns a contiguous run of W_sub rows and hands them out to its 16 waves in
//     order from an LDS counter (a wave that is served faster by memory takes more rows); a wave
//     keeps 8 KiB of loads in flight and turns each 1 KiB piece over as soon as it has arrived;
//   - lane l always multiplies the same column pieces of a row, so it keeps exactly those
//     pieces of h in registers (h passes through LDS once, behind a bare barrier that does not
//     drain the W_sub loads already in flight);
//   - a row's logit comes out of a DPP / permlane butterfly wave-uniform and is inserted there
//     and then into the wave's running list of the 16 best (lane q of every 16-lane row holds
//     the q-th best; one shifted copy and two compares per row), under the latency of the loads
//     in flight; the logit also goes to its place in LDS so that the softmax statistics are
//     summed in a fixed order whatever wave happened to take the row;
//   - lists are merged by a bitonic network on 64-bit order keys (logit key, then lower draft
//     index) held one list per 16-lane row: no rounds, no data-dependent control flow, the same
//     primitive for the workgroup's 16 wave lists and for the final merge of all workgroups'
//     lists by the last workgroup to arrive (single launch per step).
#pragma once

#include <type_traits>

#include "vt_gemv_common.h"

namespace vt {

constexpr int kKeyMax = 0x7fffffff;

// Value of lane l-1 of the same 16-lane row; lane 0 of a row gets `fill`.
__device__ __forceinline__ int row_shr1(int x, int fill)
{
    return __builtin_amdgcn_update_dpp(fill, x, 0x111, 0xf, 0xf, false);
}

// Device-coherent loads of what other workgroups published, issued back to back and awaited
// once (the compiler's own atomic loads wait for each load separately).  The wait takes the
// destinations as operands, so no use can be scheduled ahead of it.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void coherent_load_issue(f32x4& dst, const float* p)
{
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=&v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void coherent_load_issue(i32x4& dst, const int* p)
{
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=&v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void coherent_load_issue(float2& dst, const float2* p)
{
    asm volatile("global_load_dwordx2 %0, %1, off sc1" : "=&v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void coherent_load_issue(float& dst, const float* p)
{
    asm volatile("global_load_dword %0, %1, off sc1" : "=&v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void coherent_load_issue(int& dst, const int* p)
{
    asm volatile("global_load_dword %0, %1, off sc1" : "=&v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void coherent_load_wait(float& a, int& b, float2& c)
{
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c) : : "memory");
}
__device__ __forceinline__ void coherent_load_wait(f32x4& a, i32x4& b, float2& c)
{
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c) : : "memory");
}

constexpr int kOneRowMaxRowsPerBlock = 1024;  // W_sub rows a workgroup may own (LDS place per logit)

// LDS map of the kernel (bytes)
constexpr int kLdsZ = 0;                                        // float[1024]  logits of the workgroup's rows
constexpr int kLdsWl = kLdsZ + kOneRowMaxRowsPerBlock * 4;      // k64[16][16]  wave lists
constexpr int kLdsWst = kLdsWl + 16 * 16 * 8;                   // float2[16]   slice statistics
constexpr int kLdsCand = kLdsWst + 16 * 8;                      // k64[256][16] all workgroups' lists (final merge)
constexpr int kLdsWl2 = kLdsCand + 256 * 16 * 8;                // k64[16][16]  per-wave results of the final merge
constexpr int kLdsFst = kLdsWl2 + 16 * 16 * 8;                  // float2[16]
constexpr int kLdsTotal = kLdsFst + 16 * 8;
constexpr int kLdsH = kLdsCand;  // u32x4[512]: the hidden state on its way to the waves' registers (dead before the final merge)
constexpr int kLdsPs = kLdsCand + 8192;  // uint8[16][512]: per wave, the block exponents of its hand-out (dead before the final merge)


// ---- storage formats of W_sub ----
// A format says how many weights a 16-byte piece holds, how the piece is multiplied with the
// matching pieces of h (kept as bf16 pairs in kHRegs registers per piece) and which scales go
// with it.  Products of bf16 numbers with bf16 / E4M3 / E2M1 numbers are exact in fp32; sums are
// fp32.
struct FmtBf16 {
    static constexpr int kElems = 8;        // weights per 16-byte piece
    static constexpr int kHRegs = 4;        // registers of h per piece (two bf16 each)
    static constexpr bool kRowScale = false;
    static constexpr bool kPieceScale = false;
    static __device__ __forceinline__ float dot(const u32x4& w, const uint32_t* hp, float acc, uint32_t)
    {
        const u32x4 x = {hp[0], hp[1], hp[2], hp[3]};
        return dot8<true>(w, x, acc);
    }
};

// T: 1 KiB pieces per W_sub row (H = 64 * T * F::kElems); 8 KiB in flight per wave.
template <class F, int T>
__global__ void __launch_bounds__(kGemvThreads) gemv_one_row_kernel(GemvArgs a)
{
    constexpr int D = 8;
    constexpr int G = D / T;  // W_sub rows per hand-out (one loop iteration)
    constexpr int HR = F::kHRegs;
    static_assert(D % T == 0, "a loop iteration covers whole rows");
    static_assert(T * HR <= 32, "h pieces of a lane must fit 32 registers");
    extern __shared__ u32x4 smem[];
    __shared__ int s_last;
    __shared__ unsigned int s_next;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int nchunk = T * 64;          // 16-byte pieces per row
    constexpr int H = nchunk * F::kElems;   // hidden size
    char* lds = reinterpret_cast<char*>(smem);
    float* zbuf = reinterpret_cast<float*>(lds + kLdsZ);
    k64* wl = reinterpret_cast<k64*>(lds + kLdsWl);
    float2* wst = reinterpret_cast<float2*>(lds + kLdsWst);

    // rows of this workgroup: an even split of V_draft over the grid, in order
    const int nb = gridDim.x;
    const int b = blockIdx.x;
    const int base = a.Vd / nb;
    const int rem = a.Vd - base * nb;
    const int n_wg = base + (b < rem ? 1 : 0);
    const int j0 = b * base + (b < rem ? b : rem);
    const int ngroups = (n_wg + G - 1) / G;
    const int nfull = n_wg / G;  // groups below this index have all G rows

    const u32x4* wp = a.W + (size_t)j0 * nchunk + lane;
    auto slot_ptr = [&](int grp, int i) { return wp + (size_t)(grp * G + i / T) * nchunk + (i % T) * kWave; };
    // scales: one fp32 per row (kRowScale) or one exponent byte per piece (kPieceScale).  The bytes of a
    // hand-out are contiguous (D * 64 of them): the wave fetches them with one 8-byte load per lane and
    // passes them through its own 512 bytes of LDS, where lane l picks up byte i * 64 + l for piece i.
    const float* rsp = reinterpret_cast<const float*>(a.scales) + j0;
    constexpr int kPsBytes = D * kWave;
    const uint8_t* psg = reinterpret_cast<const uint8_t*>(a.scales) + (size_t)j0 * nchunk;
    uint8_t* psl = reinterpret_cast<uint8_t*>(lds + kLdsPs) + wave * kPsBytes;
    auto load_ps = [&](int grp, bool full) {
        u32x2 v = {0x7f7f7f7fu, 0x7f7f7f7fu};
        if (full || grp * G + (8 * lane) / nchunk < n_wg)  // rows past the workgroup's run are not read
            v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(psg + (size_t)grp * kPsBytes) + lane);
        return v;
    };

    // the hidden state: one 8-byte piece (four bf16) per thread, requested before anything else
    const int hpiece = tid < H / 4 ? tid : H / 4 - 1;
    uint2 hval = reinterpret_cast<const uint2*>(a.h)[hpiece];
    const bool norm = a.gamma != nullptr;  // h is the state before the final RMSNorm: normalise it on the way in
    uint2 gval = make_uint2(0u, 0u);
    if (norm)
        gval = reinterpret_cast<const uint2*>(a.gamma)[hpiece];
    __builtin_amdgcn_sched_barrier(0);
    // the first hand-out is the wave's own number; later ones come from the counter
    if (tid == 0)
        s_next = kGemvWaves;
    int gc = wave;
    u32x4 buf[D];
    uint32_t sbuf[F::kPieceScale ? D : 1];  // exponent bytes of the current hand-out's pieces
    auto put_ps = [&](const u32x2& v) {
        reinterpret_cast<u32x2*>(psl)[lane] = v;  // LDS operations of one wave complete in order
#pragma unroll
        for (int i = 0; i < D; ++i)
            sbuf[i] = psl[i * kWave + lane];
    };
    float rsbuf[F::kRowScale ? G : 1];      // row scales of the rows in flight
    // The first pieces of W_sub are requested, then h goes through LDS to every wave.  When the
    // wave's first hand-out is full its loads are unconditional, so the compiler knows how many
    // loads follow the h piece and waits for that piece alone (loads return in order).  The
    // counter is set before any wave draws from it.  A bare barrier behind the LDS writes: a full
    // __syncthreads would drain the W_sub loads in flight.
    uint32_t hreg[T * HR];
    auto stage_h = [&]() {
        if (norm) {
            // RMSNorm on the way in: every thread squares its four elements, the 16 wave sums meet in LDS
            // and every thread adds them up in the same order; h = bf16(g * rsqrt(mean g^2 + eps) * gamma)
            const float g0 = bf16_lo(hval.x), g1 = bf16_hi(hval.x), g2 = bf16_lo(hval.y), g3 = bf16_hi(hval.y);
            float ss = tid < H / 4 ? ((g0 * g0 + g1 * g1) + (g2 * g2 + g3 * g3)) : 0.0f;
            ss = wave_sum(ss);
            float* nrm = reinterpret_cast<float*>(lds + kLdsWst);
            if (lane == 0)
                nrm[wave] = ss;
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
            float tot = 0.0f;
#pragma unroll
            for (int w = 0; w < kGemvWaves; ++w)
                tot += nrm[w];
            const float r = 1.0f / __builtin_sqrtf(tot / (float)H + a.eps);
            const float n0 = (g0 * r) * bf16_lo(gval.x), n1 = (g1 * r) * bf16_hi(gval.x);
            const float n2 = (g2 * r) * bf16_lo(gval.y), n3 = (g3 * r) * bf16_hi(gval.y);
            hval = make_uint2(f32_to_bf16_bits(n0) | (f32_to_bf16_bits(n1) << 16),
                              f32_to_bf16_bits(n2) | (f32_to_bf16_bits(n3) << 16));
            if (a.h_out != nullptr && blockIdx.x == 0 && tid < H / 4)
                reinterpret_cast<uint2*>(a.h_out)[tid] = hval;
        }
        reinterpret_cast<uint2*>(lds + kLdsH)[hpiece] = hval;
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0) only
        __builtin_amdgcn_s_barrier();        // every wave passes exactly one of the two barriers below
#pragma unroll
        for (int t = 0; t < T; ++t) {
            // lane's piece t covers elements (t*64 + lane) * kElems ..: HR registers = HR/4 reads of 16 bytes
            const u32x4* src = reinterpret_cast<const u32x4*>(lds + kLdsH) + (size_t)(t * kWave + lane) * (HR / 4);
#pragma unroll
            for (int q = 0; q < HR / 4; ++q) {
                const u32x4 x = src[q];
                hreg[t * HR + 4 * q] = x.x;
                hreg[t * HR + 4 * q + 1] = x.y;
                hreg[t * HR + 4 * q + 2] = x.z;
                hreg[t * HR + 4 * q + 3] = x.w;
            }
        }
    };
    auto load_slot = [&](int grp, int i) {
        buf[i] = __builtin_nontemporal_load(slot_ptr(grp, i));
        if constexpr (F::kRowScale) {
            if (i % T == 0)
                rsbuf[i / T] = __builtin_nontemporal_load(rsp + grp * G + i / T);
        }
    };
    if (gc < nfull) {
        u32x2 ps0 = {0u, 0u};
        if constexpr (F::kPieceScale)
            ps0 = load_ps(gc, true);
#pragma unroll
        for (int i = 0; i < D; ++i)
            load_slot(gc, i);
        stage_h();
        if constexpr (F::kPieceScale)
            put_ps(ps0);
        asm volatile("; first hand-out full");  // keeps the two copies apart (exact load count in this one)
    } else {
        u32x2 ps0 = {0u, 0u};
        if constexpr (F::kPieceScale)
            ps0 = load_ps(gc, false);
#pragma unroll
        for (int i = 0; i < D; ++i) {
            if (gc * G + i / T < n_wg)
                load_slot(gc, i);
        }
        stage_h();
        if constexpr (F::kPieceScale)
            put_ps(ps0);
        asm volatile("; first hand-out partial or none");
    }
    auto grab = [&]() {
        unsigned int v = 0;
        if (lane == 0)
            v = atomicAdd(&s_next, 1u);
        return v;
    };
    int gn = (int)__builtin_amdgcn_readfirstlane(grab());

    int lkey = kKeyNone, lidx = kIdxNone;  // the wave's 16 best so far: lane q of each 16-lane row holds the q-th
    float acc = 0.0f;
    float row_scale = 1.0f;
    // One iteration = the D pieces (G whole rows) of hand-out gc; the pieces of hand-out gn are
    // requested one by one as the current ones are consumed.  STEADY: both hand-outs are full,
    // so every load and every row is unconditional and the compiler counts the loads in flight
    // exactly; otherwise rows and loads are guarded.
    auto iteration = [&](auto steady_c) {
        constexpr bool STEADY = decltype(steady_c)::value;
        const unsigned int gnn_raw = grab();  // the hand-out after next: its LDS round trip hides under this iteration
        u32x2 psn = {0u, 0u};
        if constexpr (F::kPieceScale)
            psn = load_ps(gn, STEADY);
#pragma unroll
        for (int i = 0; i < D; ++i) {
            const int rr = gc * G + i / T;  // row within the workgroup's run
            if (STEADY || rr < n_wg) {
                const u32x4 cur = buf[i];
                const uint32_t cur_ps = F::kPieceScale ? sbuf[i] : 0u;
                if constexpr (F::kRowScale) {
                    if (i % T == 0)
                        row_scale = rsbuf[i / T];
                }
                if (STEADY || gn * G + i / T < n_wg)
                    load_slot(gn, i);
                acc = F::dot(cur, &hreg[(i % T) * HR], acc, cur_ps);
                if (i % T == T - 1) {
                    float pv[1] = {acc};
                    float z = reduce_pairs<1>(pv, lane);
                    if constexpr (F::kRowScale)
                        z *= row_scale;
                    acc = 0.0f;
                    const int zk = f2key(z);
                    const int j = j0 + rr;
                    const int sk = row_shr1(lkey, kKeyMax);
                    const int si = row_shr1(lidx, kIdxNone);
                    const bool c0 = zk > lkey;  // a wave's rows ascend: ties keep the earlier (lower) index ahead
                    const bool c1 = zk > sk;
                    lkey = c0 ? (c1 ? sk : zk) : lkey;
                    lidx = c0 ? (c1 ? si : j) : lidx;
                    if (lane == 0) {
                        zbuf[rr] = z;
                        if (a.logits_out != nullptr)
                            a.logits_out[j] = z;
                    }
                }
            }
            if (STEADY)
                __builtin_amdgcn_sched_barrier(0);  // keep "consume piece i, request its successor" in this order
        }
        if constexpr (F::kPieceScale)
            put_ps(psn);  // the next hand-out's exponents: they arrived before its first piece
        gc = gn;
        gn = (int)__builtin_amdgcn_readfirstlane(gnn_raw);
    };
    while (gc < ngroups) {
        if (gc < nfull && gn < nfull)
            iteration(std::true_type{});
        else
            iteration(std::false_type{});
    }

    // ---- the wave's list goes to LDS ----
    if (lane < 16)
        wl[wave * 16 + lane] = k64_make(lkey, lidx);
    __syncthreads();

    // ---- wave 0 merges the 16 lists; waves 1..15 sum the softmax statistics over fixed slices ----
    k64 best = 0;
    const bool single = a.k == 1;  // one candidate per list: plain maxima instead of the merge networks
    if (wave == 0) {
        best = single ? k64_wave_max(lane < kGemvWaves ? wl[lane * 16] : k64_make(kKeyNone, kIdxNone), lane)
                      : k64_merge_16_lists(wl, lane);
    } else {
        const int per = (n_wg + 14) / 15;  // at most 69 logits per slice: two per lane
        const int lo = (wave - 1) * per;
        const int hi = lo + per < n_wg ? lo + per : n_wg;
        const int e0 = lo + lane, e1 = lo + kWave + lane;
        const float v0 = e0 < hi ? zbuf[e0] : neg_inf();
        const float v1 = e1 < hi ? zbuf[e1] : neg_inf();
        float m = neg_inf(), s = 0.0f;
        if (lo < hi) {
            m = wave_max(fmaxf(v0, v1));
            s = wave_sum((e0 < hi ? __expf(v0 - m) : 0.0f) + (e1 < hi ? __expf(v1 - m) : 0.0f));
        }
        if (lane == 0)
            wst[wave - 1] = make_float2(m, s);
    }
    __syncthreads();

    // ---- wave 0 publishes the workgroup's partial result and takes the arrival ticket ----
    if (wave == 0) {
        const bool act = lane < 15;
        float m = act ? wst[act ? lane : 0].x : neg_inf();
        float s = act ? wst[act ? lane : 0].y : 0.0f;
        wave_stat_merge(m, s, act);
        const size_t slot = blockIdx.x;
        if (lane < 16) {
            st_dev(a.part_val + slot * 16 + lane, key2f(k64_key(best)));
            st_dev(a.part_idx + slot * 16 + lane, k64_idx(best));
        }
        if (lane == 0) {
            st_dev(reinterpret_cast<float*>(a.part_stat + slot), m);
            st_dev(reinterpret_cast<float*>(a.part_stat + slot) + 1, s);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the coherent stores are acknowledged
        if (lane == 0) {
            // arrival in two levels (groups of 16 workgroups, then the groups): at small V_draft all
            // workgroups arrive within a fraction of a microsecond, and 256 atomics on one word
            // queue up for longer than two uncontended round trips take.  Every counter is put back
            // to zero by whoever sees it full.
            const int grp = blockIdx.x >> 4;
            const int ngrp = (gridDim.x + 15) >> 4;
            const int in_grp = (grp == ngrp - 1) ? (int)gridDim.x - grp * 16 : 16;
            int last = 0;
            const unsigned int t1 = __hip_atomic_fetch_add(a.arrive + (1 + grp) * kArriveStrideWords, 1u, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT);
            if ((int)t1 == in_grp - 1) {
                __hip_atomic_store(a.arrive + (1 + grp) * kArriveStrideWords, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const unsigned int t2 = __hip_atomic_fetch_add(a.arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                last = ((int)t2 == ngrp - 1) ? 1 : 0;
            }
            s_last = last;
        }
    }
    __syncthreads();
    if (!s_last)
        return;

    // ---- the last workgroup to arrive finishes the call ----
    k64* cand = reinterpret_cast<k64*>(lds + kLdsCand);
    k64* wl2 = reinterpret_cast<k64*>(lds + kLdsWl2);
    float2* fst = reinterpret_cast<float2*>(lds + kLdsFst);
    const int P = gridDim.x;
    if (single) {
        // k = 1: the head of every workgroup's list and its statistics, one workgroup per thread
        float v = neg_inf();
        int ix = kIdxNone;
        float2 st = make_float2(neg_inf(), 0.0f);
        const bool okp = tid < P;
        if (okp) {
            coherent_load_issue(v, a.part_val + 16 * tid);
            coherent_load_issue(ix, a.part_idx + 16 * tid);
            coherent_load_issue(st, a.part_stat + tid);
        }
        coherent_load_wait(v, ix, st);
        float m = st.x, s = st.y;
        if (wave < 4) {
            const k64 top = k64_wave_max(k64_make(f2key(v), ix), lane);
            wave_stat_merge(m, s, okp);
            if (lane == 0) {
                wl2[wave] = top;
                fst[wave] = make_float2(m, s);
            }
        }
        __syncthreads();
        if (wave == 0) {
            const k64 fin = k64_wave_max(lane < 4 ? wl2[lane] : k64_make(kKeyNone, kIdxNone), lane);
            const bool act = lane < 4;
            float mv = act ? fst[act ? lane : 0].x : neg_inf();
            float sv = act ? fst[act ? lane : 0].y : 0.0f;
            wave_stat_merge(mv, sv, act);
            const float lse = mv + __logf(sv);
            if (lane == 0) {
                const int oi = k64_idx(fin);
                a.out_ids[0] = (oi != kIdxNone) ? a.d2t[oi] : -1;
                a.out_logp[0] = (key2f(k64_key(fin)) - lse) + (a.parent != nullptr ? a.parent[0] : 0.0f);
                if (a.lse_out != nullptr)
                    a.lse_out[0] = lse;
                __hip_atomic_store(a.arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        return;
    }
    {
        // all lists into LDS as keys: thread t takes entries 4t .. 4t+3 with two 128-bit device-coherent
        // loads, and one workgroup's statistics; every load is in flight before the first is awaited
        // (lists beyond P are empty)
        f32x4 v = {neg_inf(), neg_inf(), neg_inf(), neg_inf()};
        i32x4 ix = {kIdxNone, kIdxNone, kIdxNone, kIdxNone};
        float2 st = make_float2(neg_inf(), 0.0f);
        const bool ok = tid < 4 * P;
        const bool okp = tid < P;
        if (ok) {
            coherent_load_issue(v, a.part_val + 4 * tid);
            coherent_load_issue(ix, a.part_idx + 4 * tid);
        }
        if (okp)
            coherent_load_issue(st, a.part_stat + tid);
        coherent_load_wait(v, ix, st);
        float m = st.x, s = st.y;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            cand[4 * tid + q] = k64_make(f2key(v[q]), ix[q]);
        if (wave < 4) {  // the statistics of up to 256 workgroups sit in the first four waves
            wave_stat_merge(m, s, okp);
            if (lane == 0)
                fst[wave] = make_float2(m, s);
        }
    }
    __syncthreads();
    {
        const k64 mine = k64_merge_16_lists(cand + wave * 256, lane);  // wave w: lists 16w .. 16w+15
        if (lane < 16)
            wl2[wave * 16 + lane] = mine;
    }
    __syncthreads();
    if (wave == 0) {
        const k64 fin = k64_merge_16_lists(wl2, lane);
        const bool act = lane < 4;
        float mv = act ? fst[act ? lane : 0].x : neg_inf();
        float sv = act ? fst[act ? lane : 0].y : 0.0f;
        wave_stat_merge(mv, sv, act);
        const float lse = mv + __logf(sv);
        if (lane < a.k) {
            const int oi = k64_idx(fin);
            a.out_ids[lane] = (oi != kIdxNone) ? a.d2t[oi] : -1;
            a.out_logp[lane] = (key2f(k64_key(fin)) - lse) + (a.parent != nullptr ? a.parent[0] : 0.0f);
        }
        if (lane == 0) {
            if (a.lse_out != nullptr)
                a.lse_out[0] = lse;
            __hip_atomic_store(a.arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// What the kernel assumes of a launch: one row, lists of 16 in the workspace, at most 256
// workgroups (partial results) of at most kOneRowMaxRowsPerBlock W_sub rows each.
inline bool one_row_launch_ok(const Plan& p, const GemvArgs& ga)
{
    return ga.rows == 1 && ga.KP == 16 && ga.k <= 16 && p.blocks <= 256 && p.blocks >= 1 && ga.P == p.blocks &&
           (long long)ga.Vd <= (long long)p.blocks * kOneRowMaxRowsPerBlock && ga.fused;
}

template <class F, int T>
inline hipError_t launch_one_row_t(const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    static_assert(kLdsTotal <= 48 * 1024, "fits the default dynamic LDS limit");
    hipLaunchKernelGGL((gemv_one_row_kernel<F, T>), dim3(p.blocks), dim3(kGemvThreads), kLdsTotal, s, ga);
    return hipGetLastError();
}

}  // namespace vt
