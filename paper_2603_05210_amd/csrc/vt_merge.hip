// Final stage of a draft step and the one-time subset construction.
//
// merge_kernel: per hidden-state row, combines the P partial results (softmax statistics and
// candidate lists of KP entries; lists longer than 16 arrive sorted, shorter ones in any order)
// that the projection kernel left in the workspace into the row's log-sum-exp over V_d and its
// k best draft tokens, then maps them through the draft-to-target buffer (Section 1 of the
// paper: EAGLE-3 style d2t) and emits log-probabilities.  The merge uses the strict
// (logit, index) order, so its result does not depend on how the vocabulary was split.
//
// check_ids / gather kernels: Section 2.1's V_d as a list of token ids -> W_sub and d2t.
#include "vt_device.h"
#include "vt_internal.h"

namespace vt {

template <int KP>
__global__ void __launch_bounds__(kMergeThreads) merge_kernel(const float* __restrict__ part_val,
                                                              const int32_t* __restrict__ part_idx,
                                                              const float2* __restrict__ part_stat, int P, int k,
                                                              int lists_sorted, const int32_t* __restrict__ d2t,
                                                              int32_t* __restrict__ out_ids,
                                                              float* __restrict__ out_logp,
                                                              float* __restrict__ lse_out,
                                                              const float* __restrict__ parent)
{
    constexpr int NW = kMergeThreads / kWave;
    __shared__ float sm_val[KP > 16 ? NW : 1][KP];  // per-wave results (long lists only)
    __shared__ int sm_idx[KP > 16 ? NW : 1][KP];
    __shared__ float2 sm_stat[NW];
    __shared__ int sm_qn;  // lists queued for the merge (short lists only)
    // one LDS area, two uses: the surviving lists as 64-bit keys (up to kNetLists lists of 16, plus 16
    // group results), or, when more lists survive, the per-thread sorted lists of the walking merge
    constexpr int kNetLists = 256;
    constexpr size_t kRawBytes = KP < 16 ? kMergeThreads * (KP + 1) * 8 : KP == 16 ? ((kNetLists + 16) * 16 * 8 > kMergeThreads * (KP + 1) * 8 ? (kNetLists + 16) * 16 * 8 : kMergeThreads * (KP + 1) * 8) : 16;
    __shared__ __align__(16) unsigned char sm_raw[kRawBytes];

    const int r = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // Pass A over the P partial statistics only (8 bytes each): softmax partials, and a bound
    // below which no candidate can be among the row's k best.  Split the lists into 16 classes
    // (list index mod 16); `bound` = the smallest of the 16 class maxima of the lists' best
    // logits.  16 >= KP distinct candidates are >= bound, so a list whose best logit is strictly
    // below it cannot contribute and its entries are never read.
    __shared__ float sm_cls[NW][16];
    constexpr int CH = 8;  // statistics fetched per thread and batch (independent loads in flight together)
    float m = neg_inf(), s = 0.0f;
    float cls = neg_inf();  // this thread's lists all fall in class tid % 16 (stride 256)
    float best0[CH];        // best logits of the first batch, kept for pass B
#pragma unroll
    for (int c = 0; c < CH; ++c)
        best0[c] = neg_inf();
    for (int base = 0; base < P; base += CH * kMergeThreads) {
        float2 st[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int p = base + c * kMergeThreads + tid;
            st[c] = (p < P) ? part_stat[(size_t)r * P + p] : make_float2(neg_inf(), 0.0f);
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            stat_merge(m, s, st[c].x, st[c].y);
            cls = fmaxf(cls, st[c].x);
            if (base == 0)
                best0[c] = st[c].x;
        }
    }
    float bound = neg_inf();
    if (KP <= 16 && P >= 64) {
        // class maxima: over the four 16-lane rows of a wave, then over the waves
        {
            const auto r16 = __builtin_amdgcn_permlane16_swap(__float_as_int(cls), __float_as_int(cls), false, false);
            cls = fmaxf(__int_as_float(r16[0]), __int_as_float(r16[1]));
            const auto r32 = __builtin_amdgcn_permlane32_swap(__float_as_int(cls), __float_as_int(cls), false, false);
            cls = fmaxf(__int_as_float(r32[0]), __int_as_float(r32[1]));
        }
        if (lane < 16)
            sm_cls[wave][lane] = cls;
        __syncthreads();
        float c = sm_cls[0][lane & 15];
#pragma unroll
        for (int w = 1; w < NW; ++w)
            c = fmaxf(c, sm_cls[w][lane & 15]);
        bound = -row16_max(-c);  // min over the 16 classes
    }

    TopList<KP> L;
    L.clear();
    bool first = true;
    auto take_list = [&](int p) {
        const size_t slot = (size_t)r * P + p;
        const float* pv = part_val + slot * KP;
        const int32_t* pi = part_idx + slot * KP;
        if (first) {  // the first list a thread keeps is taken whole
            if constexpr (KP % 4 == 0) {  // workspace and its sections are 16-byte aligned: 128-bit loads
#pragma unroll
                for (int q = 0; q < KP; q += 4) {
                    const float4 xv = *reinterpret_cast<const float4*>(pv + q);
                    const int4 xi = *reinterpret_cast<const int4*>(pi + q);
                    L.v[q] = xv.x, L.v[q + 1] = xv.y, L.v[q + 2] = xv.z, L.v[q + 3] = xv.w;
                    L.i[q] = xi.x, L.i[q + 1] = xi.y, L.i[q + 2] = xi.z, L.i[q + 3] = xi.w;
                }
            } else {
#pragma unroll
                for (int q = 0; q < KP; ++q) {
                    L.v[q] = pv[q];
                    L.i[q] = pi[q];
                }
            }
            if (KP <= 16 && !lists_sorted)
                L.sort();  // short lists arrive unsorted from the matrix-core GEMM kernels
            first = false;
        } else {  // later lists (rare): entry by entry; long lists are sorted, so they may stop early
#pragma unroll 1
            for (int q = 0; q < KP; ++q) {
                const float x = pv[q];
                const int ix = pi[q];
                if (!better(x, ix, L.v[KP - 1], L.i[KP - 1])) {
                    if constexpr (KP > 16)
                        break;
                    else
                        continue;
                }
                L.insert(x, ix);
            }
        }
    };
    if constexpr (KP <= 16) {
        // The lists that pass the bound (a few dozen as a rule) are queued in LDS and dealt out
        // again one per thread, so their loads are all in flight together instead of one list
        // after the other in the threads that happened to own several.  A list that does not fit
        // the queue is merged on the spot by its owner.
        constexpr int QCAP = 2048;
        __shared__ int sm_queue[QCAP];
        if (tid == 0)
            sm_qn = 0;
        __syncthreads();
        auto offer = [&](int p, float best) {
            if (best < bound)
                return;
            const int slot = atomicAdd(&sm_qn, 1);
            if (slot < QCAP)
                sm_queue[slot] = p;
            else
                take_list(p);
        };
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int p = c * kMergeThreads + tid;
            if (p < P)
                offer(p, best0[c]);
        }
        for (int p = CH * kMergeThreads + tid; p < P; p += kMergeThreads)  // beyond the first batch (very large P)
            offer(p, part_stat[(size_t)r * P + p].x);
        __syncthreads();
        const int qn = sm_qn < QCAP ? sm_qn : QCAP;
        if (KP == 16 && sm_qn <= kNetLists) {  // measured: shorter lists are faster through the register sort + walking merge below
            // The usual case: at most 256 lists survive the bound.  They go to LDS as 64-bit order keys,
            // 16 per list (shorter lists padded with the empty marker), are sorted four at a time by
            // a wave (one list per 16-lane row) unless they arrive sorted, and are merged by the same
            // bitonic network as in the one-row kernel: groups of 16 lists per wave, then the group
            // results by wave 0.  No rounds, no data-dependent control flow.
            k64* sk = reinterpret_cast<k64*>(sm_raw);                 // [up to 256 lists][16]
            k64* res = sk + kNetLists * 16;                          // [16 groups][16]
            const int ngrp = (qn + 15) >> 4;
            for (int q = tid; q < ngrp * 16; q += kMergeThreads) {
                const k64 none = k64_make(kKeyNone, kIdxNone);
                k64* dst = sk + q * 16;
                if (q < qn) {
                    const size_t slot = (size_t)r * P + sm_queue[q];
                    const float* pv = part_val + slot * KP;
                    const int32_t* pi = part_idx + slot * KP;
                    if constexpr (KP % 4 == 0) {
#pragma unroll
                        for (int t = 0; t < KP; t += 4) {
                            const float4 xv = *reinterpret_cast<const float4*>(pv + t);
                            const int4 xi = *reinterpret_cast<const int4*>(pi + t);
                            dst[t] = k64_make(f2key(xv.x), xi.x), dst[t + 1] = k64_make(f2key(xv.y), xi.y);
                            dst[t + 2] = k64_make(f2key(xv.z), xi.z), dst[t + 3] = k64_make(f2key(xv.w), xi.w);
                        }
                    } else {
#pragma unroll
                        for (int t = 0; t < KP; ++t)
                            dst[t] = k64_make(f2key(pv[t]), pi[t]);
                    }
#pragma unroll
                    for (int t = KP; t < 16; ++t)
                        dst[t] = none;
                } else {
#pragma unroll
                    for (int t = 0; t < 16; ++t)
                        dst[t] = none;
                }
            }
            res[tid] = k64_make(kKeyNone, kIdxNone);  // unused group results are empty lists (256 entries, 256 threads)
            __syncthreads();
            if (!lists_sorted) {
                for (int g4 = wave; g4 * 4 < ngrp * 16; g4 += NW)
                    sk[g4 * 64 + lane] = k64_row_sort16(sk[g4 * 64 + lane], lane);
                __syncthreads();
            }
            for (int g = wave; g < ngrp; g += NW) {
                const k64 m16 = k64_merge_16_lists(sk + g * 256, lane);
                if (lane < 16)
                    res[g * 16 + lane] = m16;
            }
            wave_stat_merge(m, s, true);
            if (lane == 0)
                sm_stat[wave] = make_float2(m, s);
            __syncthreads();
            if (wave != 0)
                return;
            const k64 fin = ngrp > 1 ? k64_merge_16_lists(res, lane) : res[lane & 15];
            const bool act = lane < NW;
            float mv = act ? sm_stat[act ? lane : 0].x : neg_inf();
            float sv = act ? sm_stat[act ? lane : 0].y : 0.0f;
            wave_stat_merge(mv, sv, act);
            const float lse = mv + __logf(sv);
            if (lane < k) {
                const int oi = k64_idx(fin);
                out_ids[(size_t)r * k + lane] = (oi != kIdxNone) ? d2t[oi] : -1;
                out_logp[(size_t)r * k + lane] = (key2f(k64_key(fin)) - lse) + (parent != nullptr ? parent[r] : 0.0f);
            }
            if (lane == 0 && lse_out != nullptr)
                lse_out[r] = lse;
            return;
        }
        for (int q = tid; q < qn; q += kMergeThreads)
            take_list(sm_queue[q]);
    } else {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int p = c * kMergeThreads + tid;
            if (p < P && !(best0[c] < L.v[KP - 1]))
                take_list(p);
        }
        for (int p = CH * kMergeThreads + tid; p < P; p += kMergeThreads) {  // beyond the first batch (very large P)
            const float best = part_stat[(size_t)r * P + p].x;
            if (!(best < L.v[KP - 1]))
                take_list(p);
        }
    }

    wave_stat_merge(m, s, true);
    if (lane == 0)
        sm_stat[wave] = make_float2(m, s);
    float ov;
    int oi;
    if constexpr (KP <= 16) {
        // Every thread parks its (sorted) list in LDS; wave 0 merges all of them in k rounds,
        // touching only list heads.
        constexpr int S = KP + 1;
        float* sl_val = reinterpret_cast<float*>(sm_raw);  // [kMergeThreads][S]
        int* sl_idx = reinterpret_cast<int*>(sm_raw) + kMergeThreads * S;
        sl_val[tid * S] = L.v[0];
        sl_idx[tid * S] = L.i[0];
        if (L.i[0] != kIdxNone) {
#pragma unroll
            for (int q = 1; q < KP; ++q) {
                sl_val[tid * S + q] = L.v[q];
                sl_idx[tid * S + q] = L.i[q];
            }
        }
        __syncthreads();
        if (wave != 0)
            return;
        // at most 64 queued lists sit in the first 64 threads: one head per lane then
        if (sm_qn <= kWave)
            wave_walk_merge<KP, 1, false>(sl_val, sl_idx, kWave, k, lane, ov, oi);
        else
            wave_walk_merge<KP, NW, false>(sl_val, sl_idx, kMergeThreads, k, lane, ov, oi);
    } else {
        wave_merge<KP>(L, true, lane, ov, oi, k);
        if (lane < KP) {
            sm_val[wave][lane] = ov;
            sm_idx[wave][lane] = oi;
        }
        __syncthreads();
        if (wave != 0)
            return;
        const bool act = lane < NW;
        TopList<KP> T;
        T.clear();
        if (act) {
#pragma unroll
            for (int q = 0; q < KP; ++q) {  // slots k..KP-1 were not produced: leave them empty
                if (q < k) {
                    T.v[q] = sm_val[lane][q];
                    T.i[q] = sm_idx[lane][q];
                }
            }
        }
        wave_merge<KP>(T, act, lane, ov, oi, k);
    }

    {
        const bool act = lane < NW;
        float mv = act ? sm_stat[act ? lane : 0].x : neg_inf();
        float sv = act ? sm_stat[act ? lane : 0].y : 0.0f;
        wave_stat_merge(mv, sv, act);
        const float lse = mv + __logf(sv);
        if (lane < k) {
            out_ids[(size_t)r * k + lane] = (oi != kIdxNone) ? d2t[oi] : -1;
            out_logp[(size_t)r * k + lane] = (ov - lse) + (parent != nullptr ? parent[r] : 0.0f);
        }
        if (lane == 0 && lse_out != nullptr)
            lse_out[r] = lse;
    }
}

hipError_t launch_merge(const Plan& p, const HeadArgs& a, hipStream_t s)
{
    // the streaming kernels and long lists arrive sorted; the GEMM epilogue leaves short lists as they come
    const int sorted = (p.regime == 0 || p.KP > 16) ? 1 : 0;
#define VT_MERGE_CASE(KPV)                                                                                   \
    case KPV:                                                                                                \
        hipLaunchKernelGGL(merge_kernel<KPV>, dim3(p.rows), dim3(kMergeThreads), 0, s, a.part_val, a.part_idx, \
                           a.part_stat, p.P, p.k, sorted, a.d2t, a.out_ids, a.out_logp, a.lse_out, a.parent);  \
        break;
    switch (p.KP) {
        VT_MERGE_CASE(1)
        VT_MERGE_CASE(2)
        VT_MERGE_CASE(4)
        VT_MERGE_CASE(8)
        VT_MERGE_CASE(16)
        VT_MERGE_CASE(32)
        VT_MERGE_CASE(64)
    default:
        return hipErrorInvalidValue;
    }
#undef VT_MERGE_CASE
    return hipGetLastError();
}

// RMSNorm of the hidden states ahead of the head, for the shapes whose projection kernel does not
// normalise on the way in: h[r,i] = bf16(g[r,i] * rsqrt(mean_i g[r,i]^2 + eps) * gamma[i]); one
// workgroup per row, sums in a fixed order.
__global__ void __launch_bounds__(256) rmsnorm_kernel(const uint32_t* __restrict__ g, const uint32_t* __restrict__ gamma,
                                                      float eps, int H, uint32_t* __restrict__ h_out)
{
    __shared__ float part[4];
    const int r = blockIdx.x;
    const int tid = threadIdx.x;
    const uint32_t* gr = g + (size_t)r * (H / 2);
    float ss = 0.0f;
    for (int c = tid; c < H / 2; c += 256) {
        const uint32_t w = gr[c];
        const float a = bf16_lo(w), b = bf16_hi(w);
        ss += a * a + b * b;
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0)
        part[tid >> 6] = ss;
    __syncthreads();
    const float tot = (part[0] + part[1]) + (part[2] + part[3]);
    const float rs = 1.0f / __builtin_sqrtf(tot / (float)H + eps);
    for (int c = tid; c < H / 2; c += 256) {
        const uint32_t w = gr[c], gm = gamma[c];
        const float a = (bf16_lo(w) * rs) * bf16_lo(gm), b = (bf16_hi(w) * rs) * bf16_hi(gm);
        h_out[(size_t)r * (H / 2) + c] = f32_to_bf16_bits(a) | (f32_to_bf16_bits(b) << 16);
    }
}

hipError_t launch_rmsnorm(const uint16_t* g, const uint16_t* gamma, float eps, int rows, int H, uint16_t* h_out, hipStream_t s)
{
    hipLaunchKernelGGL(rmsnorm_kernel, dim3(rows), dim3(256), 0, s, reinterpret_cast<const uint32_t*>(g),
                       reinterpret_cast<const uint32_t*>(gamma), eps, H, reinterpret_cast<uint32_t*>(h_out));
    return hipGetLastError();
}

// Zeroes n 32-bit words (workspace header); a kernel rather than a memset so that a caller may
// record it into a graph.
__global__ void clear_words_kernel(uint32_t* __restrict__ p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        p[i] = 0u;
}

hipError_t launch_clear_words(uint32_t* p, int n, hipStream_t s)
{
    hipLaunchKernelGGL(clear_words_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

// ------------------------------------------------------------------ subset construction

// err bit 0: an id outside [0,V); bit 1: an id seen twice.  bitmap has ceil(V/32) zeroed words.
__global__ void check_ids_kernel(const int32_t* __restrict__ ids, int Vd, int V, uint32_t* bitmap, int* err)
{
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < Vd; j += gridDim.x * blockDim.x) {
        const int id = ids[j];
        if (id < 0 || id >= V) {
            atomicOr(err, 1);
        } else {
            const uint32_t bit = 1u << (id & 31);
            const uint32_t old = atomicOr(&bitmap[id >> 5], bit);
            if (old & bit)
                atomicOr(err, 2);
        }
    }
}

// One wave per W_sub row: 128-bit copies of the source row, 1 KiB per wave instruction.
__global__ void __launch_bounds__(256) gather_kernel(const u32x4* __restrict__ W, int nchunk,
                                                     const int32_t* __restrict__ ids, int Vd,
                                                     u32x4* __restrict__ W_sub, int32_t* __restrict__ d2t)
{
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int nw = gridDim.x * (blockDim.x >> 6);
    for (int j = gw; j < Vd; j += nw) {
        const int id = ids[j];
        const u32x4* src = W + (size_t)id * nchunk;
        u32x4* dst = W_sub + (size_t)j * nchunk;
        for (int c = lane; c < nchunk; c += kWave)
            __builtin_nontemporal_store(__builtin_nontemporal_load(src + c), dst + c);
        if (lane == 0)
            d2t[j] = id;
    }
}

hipError_t launch_check_ids(const int32_t* ids, int Vd, int V, uint32_t* bitmap, int* err, hipStream_t s)
{
    int blocks = (Vd + 255) / 256;
    if (blocks > 1024)
        blocks = 1024;
    hipLaunchKernelGGL(check_ids_kernel, dim3(blocks), dim3(256), 0, s, ids, Vd, V, bitmap, err);
    return hipGetLastError();
}

hipError_t launch_gather(const uint16_t* W, int H, const int32_t* ids, int Vd, uint16_t* W_sub, int32_t* d2t,
                         hipStream_t s)
{
    int blocks = (Vd + 3) / 4;
    if (blocks > 8192)
        blocks = 8192;
    hipLaunchKernelGGL(gather_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<const u32x4*>(W), H / 8, ids,
                       Vd, reinterpret_cast<u32x4*>(W_sub), d2t);
    return hipGetLastError();
}

}  // namespace vt
