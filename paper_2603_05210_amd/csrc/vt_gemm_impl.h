// Implementation of the MFMA-regime projection kernel; included by one translation unit per
// candidate-list length so that the instantiations compile in parallel.
#pragma once

#include <type_traits>

#include "vt_device.h"
#include "vt_internal.h"

namespace vt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Compile-time loop: the body receives an integral_constant, so every register-array index
// below is a constant before any optimisation pass runs (accumulators must stay in registers).
template <int N, typename F, int I = 0>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, F, I + 1>(static_cast<F&&>(f));
    }
}

template <int WV, int WR, int SV, int SR, int KP, bool GUARD_K>
__global__ void __launch_bounds__(WV* WR * 64) gemm_head_kernel(GemmArgs a)
{
    constexpr int BMV = WV * SV * 32;    // draft tokens per workgroup tile
    constexpr int BNR = WR * SR * 32;    // hidden-state rows per workgroup tile
    constexpr int NT = WV * WR * 64;
    constexpr int TROWS = BMV + BNR;     // LDS rows per stage (W_sub rows, then h rows)
    constexpr int STAGE = TROWS * 8;     // 16-byte pieces per stage
    constexpr int NLD = STAGE / NT;      // 16-byte global loads per thread per stage
    constexpr int NLD_W = BMV * 8 / NT;  // the first NLD_W of them read W_sub
    constexpr int RSTEP = NT / 8;        // tile rows between two loads of one thread
    static_assert(STAGE % NT == 0 && (BMV * 8) % NT == 0, "tile must split evenly over the threads");
    static_assert(RSTEP % 16 == 0, "row stride per load must keep the swizzle per-thread constant");
    extern __shared__ u32x4 smem[];

    // XCD-aware tile order: workgroup ids go round-robin over the 8 XCDs, so give each XCD a
    // contiguous run of tiles (all row tiles of a vocabulary tile share W_sub through one L2).
    const int total = a.n_vtiles * a.n_rtiles;
    const int per_xcd = (total + 7) >> 3;
    const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || lin >= total)
        return;
    const int vt_i = lin / a.n_rtiles;
    const int rt_i = lin - vt_i * a.n_rtiles;
    const int v0 = vt_i * BMV;
    const int r0 = rt_i * BNR;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wv = wave / WR;
    const int wr = wave - wv * WR;
    const int nchunk = a.nchunk;

    // ---- global -> register staging: thread t moves piece (t%8) of tile rows t/8 + i*RSTEP ----
    const int lrow = tid >> 3;
    const int lc = tid & 7;
    const u32x4* gsrc[NLD];
    const u32x4* Wp = static_cast<const u32x4*>(a.W);
    const u32x4* hp = static_cast<const u32x4*>(a.h);
    static_for<NLD>([&](auto I) {
        constexpr int i = decltype(I)::value;
        const int rowid = lrow + i * RSTEP;
        if constexpr (i < NLD_W) {
            int v = v0 + rowid;
            v = v < a.Vd ? v : a.Vd - 1;
            gsrc[i] = Wp + (size_t)v * nchunk + lc;
        } else {
            int r = r0 + rowid - BMV;
            r = r < a.rows ? r : a.rows - 1;
            gsrc[i] = hp + (size_t)r * nchunk + lc;
        }
    });
    const int st_off = lrow * 8 + (lc ^ ((lrow >> 1) & 7));

    u32x4 stage[NLD];
    auto load_stage = [&](int kt) {
        bool ok = true;
        if constexpr (GUARD_K)
            ok = (kt * 8 + lc) < nchunk;
        static_for<NLD>([&](auto I) {
            constexpr int i = decltype(I)::value;
            if constexpr (GUARD_K) {
                const u32x4 zero = {0u, 0u, 0u, 0u};
                stage[i] = ok ? gsrc[i][kt * 8] : zero;
            } else {
                stage[i] = gsrc[i][kt * 8];
            }
        });
    };
    auto store_stage = [&](int buf) {
        static_for<NLD>([&](auto I) {
            constexpr int i = decltype(I)::value;
            smem[buf * STAGE + st_off + i * RSTEP * 8] = stage[i];
        });
    };

    // ---- fragment addressing ----
    const int frow = lane & 31;
    const int fhalf = lane >> 5;
    const int fsw = (lane >> 1) & 7;
    const int a_base = (wv * SV * 32 + frow) * 8;
    const int b_base = (BMV + wr * SR * 32 + frow) * 8;

    f32x16 acc[SV * SR];
    static_for<SV * SR>([&](auto I) {
        constexpr int i = decltype(I)::value;
        static_for<16>([&](auto E) { acc[i][decltype(E)::value] = 0.0f; });
    });

    const int KT = (nchunk + 7) >> 3;
    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT)
            load_stage(kt + 1);
        static_for<4>([&](auto KS) {
            constexpr int ks = decltype(KS)::value;
            const int pc = ((ks * 2 + fhalf) ^ fsw);
            bf16x8 af[SV], bfr[SR];
            static_for<SV>([&](auto I) {
                constexpr int sv = decltype(I)::value;
                af[sv] = __builtin_bit_cast(bf16x8, smem[buf * STAGE + a_base + sv * 32 * 8 + pc]);
            });
            static_for<SR>([&](auto I) {
                constexpr int sr = decltype(I)::value;
                bfr[sr] = __builtin_bit_cast(bf16x8, smem[buf * STAGE + b_base + sr * 32 * 8 + pc]);
            });
            static_for<SV>([&](auto I) {
                constexpr int sv = decltype(I)::value;
                static_for<SR>([&](auto Jc) {
                    constexpr int sr = decltype(Jc)::value;
                    acc[sv * SR + sr] =
                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[sv], bfr[sr], acc[sv * SR + sr], 0, 0, 0);
                });
            });
        });
        if (kt + 1 < KT)
            store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- fused epilogue, lane-private on the accumulators ----
    // accumulator element e of sub-tile (sv, sr): draft token v0 + wv*SV*32 + sv*32 + 8*(e/4) + 4*(lane/32) + e%4,
    // hidden-state row r0 + wr*SR*32 + sr*32 + lane%32.
    const int tok_base = v0 + wv * SV * 32 + 4 * fhalf;
    const int part = (vt_i * WV + wv) * 2 + fhalf;
    const bool full_v = (v0 + BMV) <= a.Vd;  // no vocabulary tail inside this tile
    static_for<SR>([&](auto Jc) {
        constexpr int sr = decltype(Jc)::value;
        const int row = r0 + wr * SR * 32 + sr * 32 + frow;
        const bool row_ok = row < a.rows;
        float mx = neg_inf();
        static_for<SV>([&](auto I) {
            constexpr int sv = decltype(I)::value;
            static_for<16>([&](auto E) {
                constexpr int e = decltype(E)::value;
                const int tok = tok_base + sv * 32 + 8 * (e >> 2) + (e & 3);
                if (!full_v && tok >= a.Vd)
                    acc[sv * SR + sr][e] = neg_inf();
                mx = fmaxf(mx, acc[sv * SR + sr][e]);
            });
        });
        TopList<KP> L;
        L.clear();
        float s = 0.0f;
        const float mref = mx > neg_inf() ? mx : 0.0f;  // all-masked stream: exp(-inf - 0) = 0
        static_for<SV>([&](auto I) {
            constexpr int sv = decltype(I)::value;
            static_for<16>([&](auto E) {
                constexpr int e = decltype(E)::value;
                const int tok = tok_base + sv * 32 + 8 * (e >> 2) + (e & 3);
                const float z = acc[sv * SR + sr][e];
                s += __expf(z - mref);
                L.insert_ordered(z, (full_v || tok < a.Vd) ? tok : kIdxNone);
                if (a.logits_out != nullptr && row_ok && tok < a.Vd)
                    a.logits_out[(size_t)row * a.Vd + tok] = z;
            });
        });
        if (row_ok) {
            const size_t slot = (size_t)row * a.P + part;
            static_for<KP>([&](auto Q) {
                constexpr int q = decltype(Q)::value;
                a.part_val[slot * KP + q] = L.v[q];
                a.part_idx[slot * KP + q] = L.i[q];
            });
            a.part_stat[slot] = make_float2(mx, s);
        }
    });
}


template <int WV, int WR, int SV, int SR, int KP, bool ALLOW_GUARD>
static hipError_t launch_tile(const Plan& p, const GemmArgs& ga, hipStream_t s)
{
    constexpr int BMV = WV * SV * 32, BNR = WR * SR * 32, NT = WV * WR * 64;
    const size_t lds = (size_t)2 * (BMV + BNR) * 128;
    const bool guard = (p.H % 64) != 0;
    void (*kern)(GemmArgs) = gemm_head_kernel<WV, WR, SV, SR, KP, false>;
    if constexpr (ALLOW_GUARD) {
        if (guard)
            kern = gemm_head_kernel<WV, WR, SV, SR, KP, true>;
    } else {
        if (guard)
            return hipErrorInvalidValue;
    }
    static bool lds_raised[2] = {false, false};  // per instantiation and variant: raised once
    if (lds > 48 * 1024 && !lds_raised[guard]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return e;
        lds_raised[guard] = true;
    }
    hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(NT), lds, s, ga);
    return hipGetLastError();
}

template <int KP>
static hipError_t launch_gemm_kp(const Plan& p, const GemmArgs& ga, hipStream_t s)
{
    if (p.tile == 0)
        return launch_tile<2, 2, 2, 2, KP, true>(p, ga, s);
    if constexpr (KP <= 16) {
        if (p.tile == 1)
            return launch_tile<2, 2, 4, 4, KP, false>(p, ga, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace vt
