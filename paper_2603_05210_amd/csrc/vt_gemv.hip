// Streaming regime of the draft head (1..16 hidden-state rows): the projection of Section
// 2.3 of the paper, z[r,j] = sum_i h[r,i] W_sub[j,i], is bound by reading W_sub once from
// HBM (2*H*V_draft bytes, the same number as the paper's 2dk FLOP count), so the kernel is a
// row-split dot product: a wave reads J consecutive W_sub rows with one coalesced 128-bit
// load per lane per KiB, multiplies them against the hidden states held in LDS, and reduces
// across its 64 lanes with shuffles.  Softmax statistics and the k best candidates are kept
// per lane while streaming, merged per workgroup at the end, and one partial per (row,
// workgroup) goes to the merge kernel.  Logits never reach memory (except in the test hook).
#include "vt_device.h"
#include "vt_internal.h"

namespace vt {

struct GemvArgs {
    const u32x4* h;
    const u32x4* W;
    int rows, nchunk, Vd, P;
    float* part_val;
    int32_t* part_idx;
    float2* part_stat;
    float* logits_out;
};

__device__ __forceinline__ float dot8(const u32x4& w, const u32x4& x, float acc)
{
    acc = fmaf(bf16_lo(w.x), bf16_lo(x.x), acc);
    acc = fmaf(bf16_hi(w.x), bf16_hi(x.x), acc);
    acc = fmaf(bf16_lo(w.y), bf16_lo(x.y), acc);
    acc = fmaf(bf16_hi(w.y), bf16_hi(x.y), acc);
    acc = fmaf(bf16_lo(w.z), bf16_lo(x.z), acc);
    acc = fmaf(bf16_hi(w.z), bf16_hi(x.z), acc);
    acc = fmaf(bf16_lo(w.w), bf16_lo(x.w), acc);
    acc = fmaf(bf16_hi(w.w), bf16_hi(x.w), acc);
    return acc;
}

template <int NR, int J, int KP>
__global__ void __launch_bounds__(kGemvThreads) gemv_head_kernel(GemvArgs a)
{
    constexpr int NP = NR * J;               // (row, W_sub row) pairs reduced together
    constexpr int CL = kWave / NP;           // lanes that end up holding the same pair
    static_assert(NP <= kWave && (NP & (NP - 1)) == 0, "pairs per group must be a power of two <= 64");
    extern __shared__ u32x4 smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nchunk = a.nchunk;

    // hidden states -> LDS (rows beyond `rows` repeat the last one; their results are dropped)
    for (int x = tid; x < NR * nchunk; x += kGemvThreads) {
        const int r = x / nchunk;
        const int c = x - r * nchunk;
        const int rr = r < a.rows ? r : a.rows - 1;
        smem[x] = a.h[(size_t)rr * nchunk + c];
    }
    __syncthreads();

    const int p_l = (NP > 1) ? (lane >> (6 - ilog2(NP))) : 0;  // pair this lane ends up with
    const int r_l = p_l / J;
    const int jj_l = p_l - r_l * J;
    const bool owner = (lane & (CL - 1)) == 0;

    TopList<KP> L;
    L.clear();
    float m = neg_inf(), s = 0.0f;

    const int ngroups = (a.Vd + J - 1) / J;
    const int gw = blockIdx.x * kGemvWaves + wave;
    const int nw = gridDim.x * kGemvWaves;

    for (int g = gw; g < ngroups; g += nw) {
        const int j0 = g * J;
        const u32x4* wp[J];
#pragma unroll
        for (int jj = 0; jj < J; ++jj) {
            const int j = (j0 + jj < a.Vd) ? j0 + jj : a.Vd - 1;
            wp[jj] = a.W + (size_t)j * nchunk;
        }
        float acc[NR][J];
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int jj = 0; jj < J; ++jj)
                acc[r][jj] = 0.0f;

#pragma unroll 2
        for (int c = lane; c < nchunk; c += kWave) {
            u32x4 w[J];
#pragma unroll
            for (int jj = 0; jj < J; ++jj)
                w[jj] = __builtin_nontemporal_load(wp[jj] + c);
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const u32x4 x = smem[r * nchunk + c];
#pragma unroll
                for (int jj = 0; jj < J; ++jj)
                    acc[r][jj] = dot8(w[jj], x, acc[r][jj]);
            }
        }

        float pv[NP];
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int jj = 0; jj < J; ++jj)
                pv[r * J + jj] = acc[r][jj];
        float z = reduce_pairs<NP>(pv, lane);

        const int j = j0 + jj_l;
        const bool valid = (j < a.Vd) && (r_l < a.rows);
        if (!valid)
            z = neg_inf();
        if (a.logits_out != nullptr && valid && owner)
            a.logits_out[(size_t)r_l * a.Vd + j] = z;
        stat_add(m, s, z);
        L.insert_ordered(z, valid ? j : kIdxNone);
    }

    // ---- per-workgroup merge: lanes -> wave (registers), waves -> workgroup (LDS) ----
    __syncthreads();  // the hidden states in LDS are dead from here on
    float* sm_val = reinterpret_cast<float*>(smem);                  // [waves][NR][KP]
    int* sm_idx = reinterpret_cast<int*>(sm_val + kGemvWaves * NR * KP);
    float2* sm_stat = reinterpret_cast<float2*>(sm_idx + kGemvWaves * NR * KP);  // [waves][NR]

#pragma unroll 1
    for (int r = 0; r < NR; ++r) {
        const bool act = owner && (r_l == r);
        float mv = m, sv = s;
        wave_stat_merge(mv, sv, act);
        float ov;
        int oi;
        wave_merge<KP>(L, act, lane, ov, oi);
        if (lane < KP) {
            sm_val[(wave * NR + r) * KP + lane] = ov;
            sm_idx[(wave * NR + r) * KP + lane] = oi;
        }
        if (lane == 0)
            sm_stat[wave * NR + r] = make_float2(mv, sv);
    }
    __syncthreads();

    for (int r = wave; r < a.rows; r += kGemvWaves) {
        const bool act = lane < kGemvWaves;
        TopList<KP> T;
        T.clear();
        float mv = neg_inf(), sv = 0.0f;
        if (act) {
#pragma unroll
            for (int q = 0; q < KP; ++q) {
                T.v[q] = sm_val[(lane * NR + r) * KP + q];
                T.i[q] = sm_idx[(lane * NR + r) * KP + q];
            }
            const float2 st = sm_stat[lane * NR + r];
            mv = st.x;
            sv = st.y;
        }
        wave_stat_merge(mv, sv, act);
        float ov;
        int oi;
        wave_merge<KP>(T, act, lane, ov, oi);
        const size_t slot = (size_t)r * a.P + blockIdx.x;
        if (lane < KP) {
            a.part_val[slot * KP + lane] = ov;
            a.part_idx[slot * KP + lane] = oi;
        }
        if (lane == 0)
            a.part_stat[slot] = make_float2(mv, sv);
    }
}

template <int NR, int J, int KP>
static hipError_t launch_one(const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    const size_t lds_h = (size_t)NR * ga.nchunk * sizeof(u32x4);
    const size_t lds_merge = (size_t)kGemvWaves * NR * (KP * 8 + 8);
    const size_t lds = lds_h > lds_merge ? lds_h : lds_merge;
    auto kern = gemv_head_kernel<NR, J, KP>;
    if (lds > 160 * 1024)
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

template <int NR, int J>
static hipError_t launch_kp(const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    switch (p.KP) {
    case 1: return launch_one<NR, J, 1>(p, ga, s);
    case 2: return launch_one<NR, J, 2>(p, ga, s);
    case 4: return launch_one<NR, J, 4>(p, ga, s);
    case 8: return launch_one<NR, J, 8>(p, ga, s);
    case 16: return launch_one<NR, J, 16>(p, ga, s);
    case 32: return launch_one<NR, J, 32>(p, ga, s);
    case 64: return launch_one<NR, J, 64>(p, ga, s);
    }
    return hipErrorInvalidValue;
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
    ga.part_val = a.part_val;
    ga.part_idx = a.part_idx;
    ga.part_stat = a.part_stat;
    ga.logits_out = a.logits_out;
    switch (p.NR) {
    case 1: return launch_kp<1, 4>(p, ga, s);
    case 2: return launch_kp<2, 4>(p, ga, s);
    case 4: return launch_kp<4, 4>(p, ga, s);
    case 8: return launch_kp<8, 4>(p, ga, s);
    case 16: return launch_kp<16, 4>(p, ga, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace vt
