// Implementation of the MFMA-regime projection kernel; included by one translation unit per
// candidate-list length so that the instantiations compile in parallel.
#pragma once

#include <atomic>
#include <type_traits>

#include "vt_device.h"
#include "vt_internal.h"

namespace vt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

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

// ---- fused epilogue (shared by the projection kernels) ----
// EP_LDS: park each stream in LDS and walk it with run-time loops (needed when a wave holds 256
// accumulators: fully unrolled code over them does not fit the instruction cache); otherwise the
// accumulators are walked directly.  The caller guarantees that no wave still uses the operand
// tiles in LDS (the function starts with a workgroup barrier).
template <int WV, int WR, int SV, int SR, int KP, bool EP_LDS>
__device__ __forceinline__ void head_epilogue(f32x16 (&acc)[SV * SR], const GemmArgs& a, u32x4* smem, int v0, int r0,
                                              int vt_i, int wave, int lane)
{
    constexpr int BMV = WV * SV * 32;
    const int wv = wave / WR;
    const int wr = wave - wv * WR;
    const int frow = lane & 31;
    const int fhalf = lane >> 5;
    // Accumulator element e of sub-tile (sv, sr) is draft token
    //   v0 + wv*SV*32 + sv*32 + 8*(e/4) + 4*(lane/32) + e%4   of hidden-state row  r0 + wr*SR*32 + sr*32 + lane%32,
    // so for a fixed sr a lane holds NE = 16*SV logits of ONE row, in ascending token order.
    // That stream is parked in a lane-private LDS column (so that compact run-time loops can
    // walk it; fully unrolled code over 256 accumulators does not fit the instruction cache) and
    // reduced in two passes:
    //   pass 1  exact KP largest VALUES of the stream (one v_med3 per list slot and element);
    //   pass 2  sum of exp(z - max), and the (logit, token) pairs that make up those KP values:
    //           every element above the KP-th value, plus the earliest elements equal to it
    //           until KP are taken -- the lower-index-wins rule.
    // The KP survivors are stored as this stream's partial result (sorted best-first only when
    // KP > 16).
    __syncthreads();  // every wave is done with the operand tiles
    constexpr int NE = SV * 16;   // elements per stream
    constexpr int NG = NE / 4;    // 4-element groups
        constexpr int EP_WAVE_BYTES = (EP_LDS ? NE * 64 * 4 : 0) + KP * 64 * 8;
    char* ep = reinterpret_cast<char*>(smem) + wave * EP_WAVE_BYTES;
    f32x4* ep_val = reinterpret_cast<f32x4*>(ep);                                   // [NG][64 lanes]
    int2* ep_list = reinterpret_cast<int2*>(ep + (EP_LDS ? NE * 64 * 4 : 0));       // [KP][64 lanes]
    const int tok_base = v0 + wv * SV * 32 + 4 * fhalf;
    const int part = (vt_i * WV + wv) * 2 + fhalf;
    const bool full_v = (v0 + BMV) <= a.Vd;  // no vocabulary tail inside this tile

    static_for<SR>([&](auto Jc) {
        constexpr int sr = decltype(Jc)::value;
        const int row = r0 + wr * SR * 32 + sr * 32 + frow;
        const bool row_ok = row < a.rows;
        // tokens past the end of the vocabulary become -inf
        if (!full_v) {
            static_for<SV>([&](auto I) {
                constexpr int sv = decltype(I)::value;
                static_for<16>([&](auto E) {
                    constexpr int e = decltype(E)::value;
                    const int tok = tok_base + sv * 32 + 8 * (e >> 2) + (e & 3);
                    if (tok >= a.Vd)
                        acc[sv * SR + sr][e] = neg_inf();
                });
            });
        }
        if constexpr (EP_LDS) {
            static_for<SV>([&](auto I) {
                constexpr int sv = decltype(I)::value;
                static_for<4>([&](auto Q) {
                    constexpr int q = decltype(Q)::value;
                    const f32x4 v = {acc[sv * SR + sr][4 * q], acc[sv * SR + sr][4 * q + 1],
                                     acc[sv * SR + sr][4 * q + 2], acc[sv * SR + sr][4 * q + 3]};
                    ep_val[(sv * 4 + q) * 64 + lane] = v;
                });
            });
        }
        if (a.logits_out != nullptr && row_ok) {
            static_for<SV>([&](auto I) {
                constexpr int sv = decltype(I)::value;
                static_for<16>([&](auto E) {
                    constexpr int e = decltype(E)::value;
                    const int tok = tok_base + sv * 32 + 8 * (e >> 2) + (e & 3);
                    if (tok < a.Vd)
                        a.logits_out[(size_t)row * a.Vd + tok] = acc[sv * SR + sr][e];
                });
            });
        }
        // the stream's elements, in ascending token order, as (group g of 4, position c)
        auto for_each_group = [&](auto&& body) {
            if constexpr (EP_LDS) {
#pragma unroll 2
                for (int g = 0; g < NG; ++g)
                    body(ep_val[g * 64 + lane], tok_base + (g >> 2) * 32 + (g & 3) * 8);
            } else {
                static_for<NG>([&](auto G) {
                    constexpr int g = decltype(G)::value;
                    constexpr int sv = g >> 2, q = g & 3;
                    const f32x4 v = {acc[sv * SR + sr][4 * q], acc[sv * SR + sr][4 * q + 1],
                                     acc[sv * SR + sr][4 * q + 2], acc[sv * SR + sr][4 * q + 3]};
                    body(v, tok_base + sv * 32 + q * 8);
                });
            }
        };
        // pass 1: KP largest values, best first
        float top[KP];
        static_for<KP>([&](auto S) { top[decltype(S)::value] = neg_inf(); });
        for_each_group([&](const f32x4& v, int) {
            static_for<4>([&](auto C) {
                const float x = v[decltype(C)::value];
                static_for<KP - 1>([&](auto S) {
                    constexpr int sl = KP - 1 - decltype(S)::value;  // KP-1 .. 1, old neighbours still intact
                    top[sl] = __builtin_amdgcn_fmed3f(top[sl - 1], x, top[sl]);
                });
                top[0] = fmaxf(top[0], x);
            });
        });
        const float mx = top[0];
        const float thr = top[KP - 1];
        int quota = KP;  // how many elements equal to thr belong to the KP best
        static_for<KP>([&](auto S) { quota -= (top[decltype(S)::value] > thr) ? 1 : 0; });
        const float mref = mx > neg_inf() ? mx : 0.0f;  // an all-masked stream sums exp(-inf) = 0
        // pass 2, common case: every element >= thr is a survivor (at most KP of them unless the
        // KP-th value is tied beyond its quota, which the count n_ge reveals afterwards)
        constexpr float kLog2e = 1.4426950408889634f;
        const float mref_l2 = mref * kLog2e;
        float ssum = 0.0f;
        int cnt = 0, n_ge = 0;
        for_each_group([&](const f32x4& v, int t0) {
            static_for<4>([&](auto C) {
                constexpr int c = decltype(C)::value;
                const float z = v[c];
                ssum += __builtin_amdgcn_exp2f(__builtin_fmaf(z, kLog2e, -mref_l2));
                const bool take = z >= thr;
                n_ge += take ? 1 : 0;
                if (take && cnt < KP) {
                    const int tok = t0 + c;
                    ep_list[cnt * 64 + lane] = make_int2(__float_as_int(z), tok < a.Vd ? tok : kIdxNone);
                    ++cnt;
                }
            });
        });
        if (__builtin_amdgcn_ballot_w64(n_ge > KP) != 0ull) {
            // some lane has more elements equal to thr than belong to its KP best: take the
            // elements above thr and only the earliest `quota` equal ones (lower index wins)
            cnt = 0;
            for_each_group([&](const f32x4& v, int t0) {
                static_for<4>([&](auto C) {
                    constexpr int c = decltype(C)::value;
                    const float z = v[c];
                    const bool eq = (z == thr) && (quota > 0);
                    quota -= eq ? 1 : 0;
                    if (((z > thr) || eq) && cnt < KP) {
                        const int tok = t0 + c;
                        ep_list[cnt * 64 + lane] = make_int2(__float_as_int(z), tok < a.Vd ? tok : kIdxNone);
                        ++cnt;
                    }
                });
            });
        }
        // a stream shorter than KP leaves slots open: close them with the empty marker
        for (int sl = cnt; sl < KP; ++sl)
            ep_list[sl * 64 + lane] = make_int2(__float_as_int(neg_inf()), kIdxNone);
        // the survivors; short lists leave the ordering to the merge kernel, which sorts only the
        // few lists per row that can still contribute (their best logit is in the statistics)
        TopList<KP> L;
        static_for<KP>([&](auto S) {
            constexpr int sl = decltype(S)::value;
            const int2 e = ep_list[sl * 64 + lane];
            L.v[sl] = __int_as_float(e.x);
            L.i[sl] = e.y;
        });
        if constexpr (KP > 16)
            L.sort();
        if (row_ok) {
            const size_t slot = (size_t)row * a.P + part;
            if constexpr (KP >= 4) {
                static_for<KP / 4>([&](auto Q) {
                    constexpr int q = decltype(Q)::value;
                    const f32x4 vv = {L.v[4 * q], L.v[4 * q + 1], L.v[4 * q + 2], L.v[4 * q + 3]};
                    const i32x4 ii = {L.i[4 * q], L.i[4 * q + 1], L.i[4 * q + 2], L.i[4 * q + 3]};
                    reinterpret_cast<f32x4*>(a.part_val + slot * KP)[q] = vv;
                    reinterpret_cast<i32x4*>(a.part_idx + slot * KP)[q] = ii;
                });
            } else {
                static_for<KP>([&](auto Q) {
                    constexpr int q = decltype(Q)::value;
                    a.part_val[slot * KP + q] = L.v[q];
                    a.part_idx[slot * KP + q] = L.i[q];
                });
            }
            a.part_stat[slot] = make_float2(mx, ssum);
        }
    });
}

// Projection-only epilogue (the feature-fusion layer of Section 2.3): the tile of the product
// goes to memory as bf16 (round to nearest even), row-major [rows][Vd]; a lane stores runs of four
// consecutive outputs of its row.
template <int WV, int WR, int SV, int SR>
__device__ __forceinline__ void store_epilogue(f32x16 (&acc)[SV * SR], const GemmArgs& a, int v0, int r0, int wave, int lane)
{
    const int wv = wave / WR;
    const int wr = wave - wv * WR;
    const int frow = lane & 31;
    const int fhalf = lane >> 5;
    static_for<SR>([&](auto Jc) {
        constexpr int sr = decltype(Jc)::value;
        const int row = r0 + wr * SR * 32 + sr * 32 + frow;
        if (row < a.rows) {
            static_for<SV>([&](auto I) {
                constexpr int sv = decltype(I)::value;
                static_for<4>([&](auto Q) {
                    constexpr int q = decltype(Q)::value;
                    const int tok = v0 + wv * SV * 32 + sv * 32 + 8 * q + 4 * fhalf;
                    uint16_t* dst = a.store_out + (size_t)row * a.Vd + tok;
                    if (tok + 3 < a.Vd && (a.Vd & 3) == 0) {
                        const uint32_t lo = f32_to_bf16_bits(acc[sv * SR + sr][4 * q]) | (f32_to_bf16_bits(acc[sv * SR + sr][4 * q + 1]) << 16);
                        const uint32_t hi = f32_to_bf16_bits(acc[sv * SR + sr][4 * q + 2]) | (f32_to_bf16_bits(acc[sv * SR + sr][4 * q + 3]) << 16);
                        *reinterpret_cast<uint2*>(dst) = make_uint2(lo, hi);
                    } else {
                        static_for<4>([&](auto C) {
                            constexpr int c = decltype(C)::value;
                            if (tok + c < a.Vd)
                                dst[c] = (uint16_t)f32_to_bf16_bits(acc[sv * SR + sr][4 * q + c]);
                        });
                    }
                });
            });
        }
    });
}

// RS: K tiles in flight from memory, each in a set of staging registers of its own.  One suits a grid
// that fills the chip several times over (several workgroups per compute unit hide each other's
// latency); a grid of at most one workgroup per compute unit is bound by the latency of its own K
// loop (a K tile of the small tiles is a few hundred cycles of MFMA work, a load takes a thousand
// and more), and more tiles in flight shorten every one of its K tiles.
template <int WV, int WR, int SV, int SR, int KP, bool GUARD_K, bool STORE = false, int RS = 1>
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
    // Addresses are a uniform tile base (advanced by 128 B per K tile) plus a 32-bit per-lane
    // offset; rows past the end of the matrix are clamped to its last row (masked later).
    const int lrow = tid >> 3;
    const int lc = tid & 7;
    const size_t row_bytes = (size_t)nchunk * 16;
    const char* w_base = static_cast<const char*>(a.W) + (size_t)v0 * row_bytes;
    const char* h_base = static_cast<const char*>(a.h) + (size_t)r0 * row_bytes;
    uint32_t goff[NLD];
    static_for<NLD>([&](auto I) {
        constexpr int i = decltype(I)::value;
        const int rowid = lrow + i * RSTEP;
        if constexpr (i < NLD_W) {
            int v = v0 + rowid;
            v = (v < a.Vd ? v : a.Vd - 1) - v0;
            goff[i] = (uint32_t)v * (uint32_t)row_bytes + lc * 16;
        } else {
            int r = r0 + rowid - BMV;
            r = (r < a.rows ? r : a.rows - 1) - r0;
            goff[i] = (uint32_t)r * (uint32_t)row_bytes + lc * 16;
        }
    });
    const int st_off = lrow * 8 + (lc ^ ((lrow >> 1) & 7));

    u32x4 stage[RS][NLD];  // K tile t travels through register set t % RS
    auto load_one = [&](int kt, auto ST, auto I) {
        constexpr int i = decltype(I)::value;
        constexpr int st = decltype(ST)::value;
        const char* base = (i < NLD_W ? w_base : h_base) + (size_t)kt * 128;
        const u32x4* src = reinterpret_cast<const u32x4*>(base + goff[i]);
        if constexpr (GUARD_K) {
            const u32x4 zero = {0u, 0u, 0u, 0u};
            stage[st][i] = ((kt * 8 + lc) < nchunk) ? *src : zero;
        } else {
            stage[st][i] = *src;
        }
    };
    auto store_one = [&](u32x4* __restrict__ wr, auto ST, auto I) {
        constexpr int i = decltype(I)::value;
        wr[st_off + i * RSTEP * 8] = stage[decltype(ST)::value][i];
    };
    auto load_stage = [&](int kt, auto ST) { static_for<NLD>([&](auto I) { load_one(kt, ST, I); }); };
    auto store_stage = [&](u32x4* __restrict__ wr, auto ST) { static_for<NLD>([&](auto I) { store_one(wr, ST, I); }); };

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

    // Pipeline per K tile (4 K-steps of 16): tile kt is computed from LDS buffer kt%2.
    //   steps 0-2: tile kt+1 (in its staging registers since RS iterations ago) -> other buffer, and the
    //   same registers request tile kt+1+RS from memory
    //   one barrier between steps 2 and 3: by then every wave has issued its last read of this
    //   buffer and finished its writes of the other one, so step 3 can already fetch the next
    //   tile's first fragments, and the next iteration may overwrite this buffer.
    // Fragments are double-buffered in registers: the LDS reads for K-step ks+1 are issued
    // alongside the MFMAs of K-step ks (sched_group_barrier fixes the interleaving).
    const int KT = (nchunk + 7) >> 3;
    bf16x8 af[2][SV], bfr[2][SR];
    // fragment number f of a K-step: f < SV is the W_sub fragment of sub-tile f, else the h one
    auto read_one = [&](const u32x4* __restrict__ rd, auto KS, auto SET, auto F) {
        constexpr int ks = decltype(KS)::value;
        constexpr int set = decltype(SET)::value;
        constexpr int f = decltype(F)::value;
        const int pc = ((ks * 2 + fhalf) ^ fsw);
        if constexpr (f < SV)
            af[set][f] = __builtin_bit_cast(bf16x8, rd[a_base + f * 32 * 8 + pc]);
        else
            bfr[set][f - SV] = __builtin_bit_cast(bf16x8, rd[b_base + (f - SV) * 32 * 8 + pc]);
    };
    auto read_frags = [&](const u32x4* __restrict__ rd, auto KS, auto SET) {
        static_for<SV + SR>([&](auto F) { read_one(rd, KS, SET, F); });
    };
    auto mfma_one = [&](auto SET, auto M) {
        constexpr int set = decltype(SET)::value;
        constexpr int sv = decltype(M)::value / SR;
        constexpr int sr = decltype(M)::value % SR;
        acc[sv * SR + sr] =
            __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][sv], bfr[set][sr], acc[sv * SR + sr], 0, 0, 0);
    };
    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
    using C2 = std::integral_constant<int, 2>;
    using C3 = std::integral_constant<int, 3>;
    constexpr int NMF = SV * SR;   // MFMAs per K-step
    constexpr int NFR = SV + SR;   // fragment reads per K-step

    // One K-step: the MFMAs of fragment set SET, with the LDS reads of the next K-step's
    // fragments (from rd_next into the other set) issued one per MFMA.  In the two-stage pipeline
    // the staging registers are also turned over here, spread evenly over the K tile: piece i of
    // tile kt+1 is written to the other LDS buffer and the same register immediately requests
    // piece i of tile kt+2, so every load has a whole K tile of MFMAs to arrive and neither the
    // texture path nor the LDS sees a burst.  sched_barrier pins the order; the compiler still
    // places the s_waitcnt.
    constexpr int TSTEPS = 3;                           // K-steps that carry staging turnover
    constexpr int NPAIR = (NLD + TSTEPS - 1) / TSTEPS;  // staging pieces turned over per such K-step
    auto k_step = [&](auto SET, auto KS, auto KSN, const u32x4* __restrict__ rd_next, auto DO_READ,
                      u32x4* __restrict__ wr, auto DO_WRITE, int kt_load, auto DO_LOAD, auto ST) {
        constexpr int set = decltype(SET)::value;
        constexpr int ks = decltype(KS)::value;
        constexpr bool do_read = decltype(DO_READ)::value;
        constexpr bool do_write = decltype(DO_WRITE)::value;
        constexpr bool do_load = decltype(DO_LOAD)::value;
        constexpr int SPACING = NMF / NPAIR > 0 ? NMF / NPAIR : 1;
        constexpr int RPS = (NFR + NMF - 1) / NMF;    // fragment reads attached to one MFMA (1 unless the tile is small)
        constexpr int PPS = (NPAIR + NMF - 1) / NMF;  // staging pieces attached to one MFMA (likewise)
        static_for<NMF>([&](auto M) {
            constexpr int m = decltype(M)::value;
            mfma_one(SET, M);
            if constexpr (do_read) {
                static_for<RPS>([&](auto Q) {
                    constexpr int f = m + decltype(Q)::value * NMF;
                    if constexpr (f < NFR)
                        read_one(rd_next, KSN, std::integral_constant<int, set ^ 1>{}, std::integral_constant<int, f>{});
                });
            }
            if constexpr ((do_write || do_load) && (m % SPACING) == SPACING - 1) {
                static_for<PPS>([&](auto Q) {
                    constexpr int pr = m / SPACING + decltype(Q)::value * NMF;
                    constexpr int i = ks * NPAIR + pr;
                    if constexpr (pr < NPAIR && i < NLD) {
                        if constexpr (do_write)
                            store_one(wr, ST, std::integral_constant<int, i>{});
                        if constexpr (do_load)
                            load_one(kt_load, ST, std::integral_constant<int, i>{});
                    }
                });
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // Two LDS buffers per K tile (4 K-steps of 16): tile kt is computed from LDS buffer kt%2
    // while, during K-steps 0-2, tile kt+1 moves from its staging registers (set ST) into the other
    // buffer and tile kt+1+RS is requested into them.  One barrier between K-steps 2 and 3: by then
    // every wave has issued its last read of this buffer and finished its writes of the other one, so
    // K-step 3 can already fetch the next tile's first fragments and the next iteration may overwrite
    // this buffer.  HAS1: tile kt+1 exists; HAS2: tile kt+1+RS exists.
    auto k_tile = [&](int kt, auto ST, auto HAS1, auto HAS2) {
        // The two LDS buffers never overlap: say so, or the scheduler keeps every fragment
        // read behind the tile writes.
        const u32x4* __restrict__ rd = smem + (kt & 1) * STAGE;
        u32x4* __restrict__ wr = smem + ((kt & 1) ^ 1) * STAGE;
        k_step(C0{}, C0{}, C1{}, rd, std::true_type{}, wr, HAS1, kt + 1 + RS, HAS2, ST);
        k_step(C1{}, C1{}, C2{}, rd, std::true_type{}, wr, HAS1, kt + 1 + RS, HAS2, ST);
        k_step(C0{}, C2{}, C3{}, rd, std::true_type{}, wr, HAS1, kt + 1 + RS, HAS2, ST);
        __syncthreads();
        k_step(C1{}, C3{}, C0{}, smem + ((kt & 1) ^ 1) * STAGE, HAS1, wr, std::false_type{}, 0, std::false_type{}, ST);
    };
    // iteration kt with the register set (kt + 1) % RS picked at run time (the loop's first and last iterations)
    auto k_tile_any = [&](int kt) {
        static_for<RS>([&](auto ST) {
            if ((kt + 1) % RS == decltype(ST)::value) {
                if (kt + 1 + RS < KT)
                    k_tile(kt, ST, std::true_type{}, std::true_type{});
                else if (kt + 1 < KT)
                    k_tile(kt, ST, std::true_type{}, std::false_type{});
                else
                    k_tile(kt, ST, std::false_type{}, std::false_type{});
            }
        });
    };

    // tiles 0 .. RS-1 are requested together; tile 0 goes to LDS and its registers request tile RS
    static_for<RS>([&](auto ST) {
        if (decltype(ST)::value < KT)
            load_stage(decltype(ST)::value, ST);
    });
    store_stage(smem, C0{});
    if (RS < KT)
        load_stage(RS, C0{});
    __syncthreads();
    read_frags(smem, C0{}, C0{});
    {
        int kt = 0;
        if constexpr (RS == 1) {
            for (; kt + 2 < KT; ++kt)
                k_tile(kt, C0{}, std::true_type{}, std::true_type{});
            if (kt + 1 < KT) {
                k_tile(kt, C0{}, std::true_type{}, std::false_type{});
                ++kt;
            }
            k_tile(kt, C0{}, std::false_type{}, std::false_type{});
        } else {
            // groups of RS iterations whose register sets are known at compile time: iteration kt + j uses
            // set (j + 1) % RS (kt is a multiple of RS) and all of them have tiles left to move and to request
            for (; kt + 2 * RS < KT; kt += RS)
                static_for<RS>([&](auto J) {
                    k_tile(kt + decltype(J)::value, std::integral_constant<int, (decltype(J)::value + 1) % RS>{},
                           std::true_type{}, std::true_type{});
                });
            for (; kt < KT; ++kt)
                k_tile_any(kt);
        }
    }

    if constexpr (STORE)
        store_epilogue<WV, WR, SV, SR>(acc, a, v0, r0, wave, lane);
    else
        head_epilogue<WV, WR, SV, SR, KP, (SV * SR > 8)>(acc, a, smem, v0, r0, vt_i, wave, lane);
}

template <int WV, int WR, int SV, int SR, int KP, bool ALLOW_GUARD, bool STORE, int RS>
static hipError_t launch_tile_rs(const Plan& p, const GemmArgs& ga, hipStream_t s)
{
    constexpr int BMV = WV * SV * 32, BNR = WR * SR * 32, NT = WV * WR * 64;
    constexpr size_t lds_loop = (size_t)2 * (BMV + BNR) * 128;  // two operand stages
    constexpr size_t lds_epi =
        (size_t)(NT / 64) * ((SV * SR > 8 ? (size_t)SV * 16 * 64 * 4 : 0) + (size_t)KP * 64 * 8);  // epilogue columns
    constexpr size_t lds = lds_loop > lds_epi ? lds_loop : lds_epi;
    static_assert(lds <= 160 * 1024, "operand stages and epilogue staging must fit the LDS");
    const bool guard = (p.H % 64) != 0;
    void (*kern)(GemmArgs) = gemm_head_kernel<WV, WR, SV, SR, KP, false, STORE, RS>;
    if constexpr (ALLOW_GUARD) {
        if (guard)
            kern = gemm_head_kernel<WV, WR, SV, SR, KP, true, STORE, RS>;
    } else {
        if (guard)
            return hipErrorInvalidValue;
    }
    static std::atomic<bool> lds_raised[2] = {{false}, {false}};  // per instantiation and variant: raised once
    if (lds > 48 * 1024 && !lds_raised[guard].load()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return e;
        lds_raised[guard].store(true);
    }
    hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(NT), lds, s, ga);
    return hipGetLastError();
}

// The small tiles keep several K tiles in flight when the grid gives a compute unit at most one workgroup.
template <int WV, int WR, int SV, int SR, int KP, bool ALLOW_GUARD, bool STORE = false>
static hipError_t launch_tile(const Plan& p, const GemmArgs& ga, hipStream_t s)
{
    constexpr bool small = WV * SV * WR * SR < 32;  // not the 256 x 256 tile
    if constexpr (small) {
        if (p.n_vtiles * p.n_rtiles <= 256)
            return launch_tile_rs<WV, WR, SV, SR, KP, ALLOW_GUARD, STORE, (WV * SV * WR * SR >= 16 ? 3 : 4)>(p, ga, s);
    }
    return launch_tile_rs<WV, WR, SV, SR, KP, ALLOW_GUARD, STORE, 1>(p, ga, s);
}

template <int KP>
static hipError_t launch_gemm_kp(const Plan& p, const GemmArgs& ga, hipStream_t s)
{
    if (p.tile == 0)
        return launch_tile<2, 2, 2, 2, KP, true>(p, ga, s);
    if (p.tile == 2)
        return launch_tile<1, 4, 1, 1, KP, true>(p, ga, s);
    if constexpr (KP <= 16) {
        if (p.tile == 1)
            return launch_tile<2, 4, 4, 2, KP, false>(p, ga, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace vt
