// The feature-fusion layer ahead of the draft's decoder layer (Section 2.3, component 1; Table 1's
// "Feature fusion" row): g[r,j] = sum_i x[r,i] * W_fc[j,i], a linear projection from the three
// concatenated target features (3d) to the hidden size d, 2*3d*d FLOPs per row.  bf16 in, fp32
// accumulation, bf16 out (round to nearest even).
//
// One to four rows: bound by reading W_fc once (2*3d*d bytes, 100.7 MB at d = 4096): a streaming
// row-split dot product like the head's.  More rows: the bf16 MFMA tile kernel of the head's
// tree-drafting regime with a store epilogue in place of the fused softmax / top-k one.
#include "vt_gemm_impl.h"

namespace vt {

typedef __bf16 bf16x2_f __attribute__((ext_vector_type(2)));

constexpr int kFcThreads = 1024;
constexpr int kFcDepth = 4;  // KiB in flight per wave

// One wave per W_fc row at a time (rows handed out statically, interleaved over the waves of the
// grid); x sits in LDS ([NR][d_in] bf16, at most four rows of 12288).
template <int NR>
__global__ void __launch_bounds__(kFcThreads) fc_gemv_kernel(const u32x4* __restrict__ x, int rows, int nchunk,
                                                             const u32x4* __restrict__ W, int d_out,
                                                             uint16_t* __restrict__ g_out)
{
    extern __shared__ u32x4 fc_smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nw = gridDim.x * (kFcThreads / 64);
    const int gw = blockIdx.x * (kFcThreads / 64) + wave;
    const int T = (nchunk + kWave - 1) / kWave;  // 1 KiB pieces per row (the last may be ragged)
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    int j = gw;
    u32x4 buf[kFcDepth];
    auto piece = [&](int jj, int t) {
        const int c = t * kWave + lane;
        return (jj < d_out && c < nchunk) ? __builtin_nontemporal_load(W + (size_t)jj * nchunk + c) : zero4;
    };
    // position = (row j, piece t); kFcDepth positions in flight, also across rows
    int pj = j, pt = 0;
    auto advance = [&](int& jj, int& tt) {
        if (++tt == T) {
            tt = 0;
            jj += nw;
        }
    };
#pragma unroll
    for (int i = 0; i < kFcDepth; ++i) {
        buf[i] = piece(pj, pt);
        advance(pj, pt);
    }
    for (int e = tid; e < NR * nchunk; e += kFcThreads) {
        const int r = e / nchunk;
        fc_smem[e] = x[(size_t)(r < rows ? r : rows - 1) * nchunk + (e - r * nchunk)];
    }
    __syncthreads();
    float acc[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r)
        acc[r] = 0.0f;
    int t = 0;
    while (j < d_out) {
#pragma unroll
        for (int i = 0; i < kFcDepth; ++i) {
            if (j < d_out) {  // wave-uniform
                const u32x4 cur = buf[i];
                buf[i] = piece(pj, pt);
                advance(pj, pt);
                int c = t * kWave + lane;
                c = c < nchunk ? c : nchunk - 1;  // lanes past the row end hold zeros in cur
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    const u32x4 xv = fc_smem[r * nchunk + c];
                    const bf16x8 wb = __builtin_bit_cast(bf16x8, cur);
                    const bf16x8 xb = __builtin_bit_cast(bf16x8, xv);
                    float s = acc[r];
                    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(wb, wb, 0, 1), __builtin_shufflevector(xb, xb, 0, 1), s, false);
                    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(wb, wb, 2, 3), __builtin_shufflevector(xb, xb, 2, 3), s, false);
                    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(wb, wb, 4, 5), __builtin_shufflevector(xb, xb, 4, 5), s, false);
                    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(wb, wb, 6, 7), __builtin_shufflevector(xb, xb, 6, 7), s, false);
                    acc[r] = s;
                }
                if (++t == T) {
                    t = 0;
#pragma unroll
                    for (int r = 0; r < NR; ++r) {
                        float v = acc[r];
                        v = wave_sum(v);
                        acc[r] = 0.0f;
                        if (lane == 0 && r < rows)
                            g_out[(size_t)r * d_out + j] = (uint16_t)f32_to_bf16_bits(v);
                    }
                    j += nw;
                }
            }
        }
    }
}

template <int NR>
static hipError_t launch_fc_gemv(const uint16_t* x, int rows, int d_in, const uint16_t* W, int d_out, uint16_t* g,
                                 hipStream_t s)
{
    const int nchunk = d_in / 8;
    const size_t lds = (size_t)NR * nchunk * sizeof(u32x4);
    if (lds > 150 * 1024)
        return hipErrorInvalidValue;
    int blocks = (d_out + (kFcThreads / 64) - 1) / (kFcThreads / 64);
    blocks = blocks > 256 ? 256 : blocks;
    auto kern = fc_gemv_kernel<NR>;
    static std::atomic<size_t> lds_allowed{48 * 1024};
    if (lds > lds_allowed.load()) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return e;
        lds_allowed.store(lds);
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(kFcThreads), lds, s, reinterpret_cast<const u32x4*>(x), rows, nchunk,
                       reinterpret_cast<const u32x4*>(W), d_out, g);
    return hipGetLastError();
}

hipError_t launch_feature_fusion(const uint16_t* x, int rows, int d_in, const uint16_t* W_fc, int d_out, uint16_t* g_out,
                                 hipStream_t s)
{
    if (rows <= 4 && (size_t)rows * d_in * 2 <= 150 * 1024) {
        switch (rows) {
        case 1: return launch_fc_gemv<1>(x, rows, d_in, W_fc, d_out, g_out, s);
        case 2: return launch_fc_gemv<2>(x, rows, d_in, W_fc, d_out, g_out, s);
        default: return launch_fc_gemv<4>(x, rows, d_in, W_fc, d_out, g_out, s);
        }
    }
    // matrix-core tiles: "vocabulary" = output features, hidden size = d_in
    Plan p{};
    p.rows = rows;
    p.H = d_in;
    p.Vd = d_out;
    // up to 128 rows: 32-feature tiles, so that d_out / 32 workgroups share the read of W_fc (128-feature tiles
    // would leave most compute units idle: d_out = 4096 gives 32 of them)
    p.tile = rows <= 128 ? 2 : (d_in % 64 == 0) ? 1 : 0;
    int BMV, BNR, ppv;
    gemm_tile_dims(p.tile, BMV, BNR, ppv);
    p.n_vtiles = (d_out + BMV - 1) / BMV;
    p.n_rtiles = (rows + BNR - 1) / BNR;
    p.blocks = ((p.n_vtiles * p.n_rtiles + 7) / 8) * 8;
    GemmArgs ga{};
    ga.h = x;
    ga.W = W_fc;
    ga.rows = rows;
    ga.nchunk = d_in / 8;
    ga.Vd = d_out;
    ga.n_vtiles = p.n_vtiles;
    ga.n_rtiles = p.n_rtiles;
    ga.store_out = g_out;
    if (p.tile == 1)
        return launch_tile<2, 4, 4, 2, 1, false, true>(p, ga, s);
    if (p.tile == 2)
        return launch_tile<1, 4, 1, 1, 1, true, true>(p, ga, s);
    return launch_tile<2, 2, 2, 2, 1, true, true>(p, ga, s);
}

}  // namespace vt
