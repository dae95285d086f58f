// Compressed W_sub for the one-row draft step.  The paper (Sections 1, 2.3) cuts the head's cost
// 2*d*k by trimming k; at one row that cost is bytes read, so storing each weight in fewer bits
// cuts it further.  Two forms, both native number formats of this GPU:
//   FP8    E4M3 codes (OCP: bias 7, no infinities, largest value 448) with one fp32 scale per
//          row: scale = max|w| / 448, code = E4M3(w / scale), nearest, ties to even, saturating;
//   MXFP4  OCP microscaling: E2M1 codes, two per byte (even element in the low nibble), and one
//          power-of-two exponent byte (bias 127) per 32 consecutive weights:
//          exponent = floor(log2(max|w| of the block)) - 2, code = E2M1(w / 2^exponent).
// This file holds the set-up kernels that gather the rows of V_d (Section 2.1) and quantise
// them, and the two storage formats of the generic one-row kernel: codes are widened to bf16 in
// registers by the hardware conversions (exact) and multiplied against bf16 pairs of h with
// fp32 accumulation; scales are applied to fp32 partial sums (per row, or per 32-weight block).
#include "vt_onerow.h"

namespace vt {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

struct FmtFp8 {
    static constexpr int kElems = 16;
    static constexpr int kHRegs = 8;
    static constexpr bool kRowScale = true;
    static constexpr bool kPieceScale = false;
    static __device__ __forceinline__ float dot(const u32x4& w, const uint32_t* hp, float acc, uint32_t)
    {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            // bytes 0,1 and bytes 2,3 of the word -> two bf16 each (E4M3 values are exact in bf16)
            const bf16x2_t lo = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[d], 1.0f, false);
            const bf16x2_t hi = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[d], 1.0f, true);
            acc = __builtin_amdgcn_fdot2_f32_bf16(lo, __builtin_bit_cast(bf16x2_t, hp[2 * d]), acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(hi, __builtin_bit_cast(bf16x2_t, hp[2 * d + 1]), acc, false);
        }
        return acc;
    }
};

struct FmtFp4 {
    static constexpr int kElems = 32;
    static constexpr int kHRegs = 16;
    static constexpr bool kRowScale = false;
    static constexpr bool kPieceScale = true;
    // one 16-byte piece = one 32-weight block: its sum is scaled by the block's power of two (exact)
    static __device__ __forceinline__ float dot(const u32x4& w, const uint32_t* hp, float acc, uint32_t ebyte)
    {
        float part = 0.0f;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            part = __builtin_amdgcn_fdot2_f32_bf16(__builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[d], 1.0f, 0),
                                                   __builtin_bit_cast(bf16x2_t, hp[4 * d]), part, false);
            part = __builtin_amdgcn_fdot2_f32_bf16(__builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[d], 1.0f, 1),
                                                   __builtin_bit_cast(bf16x2_t, hp[4 * d + 1]), part, false);
            part = __builtin_amdgcn_fdot2_f32_bf16(__builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[d], 1.0f, 2),
                                                   __builtin_bit_cast(bf16x2_t, hp[4 * d + 2]), part, false);
            part = __builtin_amdgcn_fdot2_f32_bf16(__builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[d], 1.0f, 3),
                                                   __builtin_bit_cast(bf16x2_t, hp[4 * d + 3]), part, false);
        }
        return acc + __builtin_ldexpf(part, (int)ebyte - 127);
    }
};

hipError_t launch_gemv_one_row_q(int fmt, const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    if (!one_row_launch_ok(p, ga) || ga.scales == nullptr)
        return hipErrorInvalidValue;
    if (fmt == VT_Q_FP8_E4M3) {
        switch (p.H) {  // T = H / 1024 pieces of 1 KiB per row
        case 1024: return launch_one_row_t<FmtFp8, 1>(p, ga, s);
        case 2048: return launch_one_row_t<FmtFp8, 2>(p, ga, s);
        case 4096: return launch_one_row_t<FmtFp8, 4>(p, ga, s);
        }
    } else if (fmt == VT_Q_MXFP4) {
        switch (p.H) {  // T = H / 2048
        case 2048: return launch_one_row_t<FmtFp4, 1>(p, ga, s);
        case 4096: return launch_one_row_t<FmtFp4, 2>(p, ga, s);
        }
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------ quantising gather (set-up)

// |x| of a finite fp32 -> E4M3 magnitude code: nearest, ties to the even mantissa, saturating at 448.
__device__ __forceinline__ uint32_t e4m3_code(float a)
{
    const uint32_t u = __float_as_uint(a);
    if (u >= 0x3C800000u) {  // a >= 2^-6: a normal E4M3 number; keep three mantissa bits
        uint32_t r = u + 0x7FFFFu + ((u >> 20) & 1u);
        r >>= 20;                        // (fp32 exponent << 3) | mantissa
        r -= (127u - 7u) << 3;           // rebias
        return r < 0x7Eu ? r : 0x7Eu;
    }
    return (uint32_t)__builtin_rintf(a * 512.0f);  // multiples of 2^-9; 8 is the smallest normal
}

// One wave per W_sub row: row maximum, scale, codes.
__global__ void __launch_bounds__(256) quant_fp8_kernel(const u32x4* __restrict__ W, int nchunk,
                                                        const int32_t* __restrict__ ids, int Vd,
                                                        uint2* __restrict__ codes, float* __restrict__ scales,
                                                        int32_t* __restrict__ d2t)
{
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int nw = gridDim.x * (blockDim.x >> 6);
    for (int j = gw; j < Vd; j += nw) {
        const int id = ids[j];
        const u32x4* src = W + (size_t)id * nchunk;
        float amax = 0.0f;
        for (int c = lane; c < nchunk; c += kWave) {
            const u32x4 v = src[c];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                amax = fmaxf(amax, fabsf(bf16_lo(v[q])));
                amax = fmaxf(amax, fabsf(bf16_hi(v[q])));
            }
        }
        amax = wave_max(amax);
        const float scale = amax > 0.0f ? amax / 448.0f : 1.0f;
        for (int c = lane; c < nchunk; c += kWave) {
            const u32x4 v = src[c];  // second pass: the row is in the cache
            uint32_t out[2] = {0u, 0u};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float w = (e & 1) ? bf16_hi(v[e >> 1]) : bf16_lo(v[e >> 1]);
                const float x = w / scale;
                const uint32_t code = e4m3_code(fabsf(x)) | ((__float_as_uint(x) >> 24) & 0x80u);
                out[e >> 2] |= code << (8 * (e & 3));
            }
            codes[(size_t)j * nchunk + c] = make_uint2(out[0], out[1]);
        }
        if (lane == 0) {
            scales[j] = scale;
            d2t[j] = id;
        }
    }
}

// |x| -> E2M1 magnitude code (0, 0.5, 1, 1.5, 2, 3, 4, 6): nearest, ties to the even mantissa bit, saturating.
__device__ __forceinline__ uint32_t e2m1_code(float a)
{
    if (a < 2.0f)
        return (uint32_t)__builtin_rintf(a * 2.0f);        // 0 .. 4
    if (a < 4.0f)
        return (uint32_t)__builtin_rintf(a) + 2u;          // 2, 3, 4 -> codes 4, 5, 6
    const float q = fminf(__builtin_rintf(a * 0.5f), 3.0f);
    return (uint32_t)q + 4u;                               // 4, 6 -> codes 6, 7
}

// One wave per W_sub row, one lane per 32-weight block.
__global__ void __launch_bounds__(256) quant_mxfp4_kernel(const u32x4* __restrict__ W, int nblocks,
                                                          const int32_t* __restrict__ ids, int Vd,
                                                          u32x4* __restrict__ packed, uint8_t* __restrict__ ebytes,
                                                          int32_t* __restrict__ d2t)
{
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int nw = gridDim.x * (blockDim.x >> 6);
    for (int j = gw; j < Vd; j += nw) {
        const int id = ids[j];
        const u32x4* src = W + (size_t)id * nblocks * 4;
        for (int bk = lane; bk < nblocks; bk += kWave) {
            u32x4 v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                v[q] = src[bk * 4 + q];
            float amax = 0.0f;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                amax = fmaxf(amax, fabsf(bf16_lo(v[q >> 2][q & 3])));
                amax = fmaxf(amax, fabsf(bf16_hi(v[q >> 2][q & 3])));
            }
            // floor(log2(amax)) - 2 as a biased byte; fp32 subnormal maxima end at byte 0 like everything below 2^-125
            int eb = 127;
            if (amax > 0.0f) {
                eb = (int)(__float_as_uint(amax) >> 23) - 2;
                eb = eb < 0 ? 0 : (eb > 254 ? 254 : eb);
            }
            uint32_t out[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                const uint32_t word = v[e >> 3][(e >> 1) & 3];
                const float w = (e & 1) ? bf16_hi(word) : bf16_lo(word);
                const float x = __builtin_ldexpf(w, 127 - eb);  // exact
                const uint32_t code = e2m1_code(fabsf(x)) | ((__float_as_uint(x) >> 28) & 0x8u);
                out[e >> 3] |= code << (4 * (e & 7));
            }
            const u32x4 o = {out[0], out[1], out[2], out[3]};
            packed[(size_t)j * nblocks + bk] = o;
            ebytes[(size_t)j * nblocks + bk] = (uint8_t)eb;
        }
        if (lane == 0)
            d2t[j] = id;
    }
}

hipError_t launch_quant_gather(int fmt, const uint16_t* W, int H, const int32_t* ids, int Vd, uint8_t* codes,
                               void* scales, int32_t* d2t, hipStream_t s)
{
    int blocks = (Vd + 3) / 4;
    if (blocks > 8192)
        blocks = 8192;
    if (fmt == VT_Q_FP8_E4M3) {
        hipLaunchKernelGGL(quant_fp8_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<const u32x4*>(W), H / 8, ids,
                           Vd, reinterpret_cast<uint2*>(codes), static_cast<float*>(scales), d2t);
    } else if (fmt == VT_Q_MXFP4) {
        hipLaunchKernelGGL(quant_mxfp4_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<const u32x4*>(W), H / 32,
                           ids, Vd, reinterpret_cast<u32x4*>(codes), static_cast<uint8_t*>(scales), d2t);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace vt
