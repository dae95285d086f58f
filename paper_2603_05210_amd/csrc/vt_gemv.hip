// Streaming regime of the draft head (1..16 hidden-state rows): the projection of Section
// 2.3 of the paper, z[r,j] = sum_i h[r,i] W_sub[j,i], is bound by reading W_sub once from
// HBM (2*H*V_draft bytes, the same number as the paper's 2dk FLOP count), so the kernels
// split W_sub by rows over the compute units and stream it exactly once.
//
// A workgroup of 16 waves owns a contiguous range of at most kGemvMaxRowsPerBlock W_sub rows.
// Two forms of the stream: gemv_head_kernel (dot products: a wave reads J consecutive rows at a
// time, one coalesced 128-bit load per lane per KiB, multiplies them against the hidden states
// held in LDS through v_dot2_f32_bf16 with fp32 accumulation and reduces across its 64 lanes by
// DPP / permlane swaps) and gemv_mfma_kernel (five rows or more: 16 W_sub rows at a time through
// v_mfma_f32_16x16x32_bf16, described there).  The logits of the range are parked in LDS, never
// in memory (except in the test hook).  When the range is done, wave r reduces hidden-state
// row r: softmax statistics and the k best logits of the range by k rounds of a wave-wide
// arg-max under the (logit, lower index) order.  One partial per (row, workgroup) goes to the
// merge kernel, or, for one or two rows, to the last workgroup of the same launch.
#include <atomic>
#include <type_traits>

#include "vt_gemv_common.h"

namespace vt {

// What every workgroup of the streaming kernels does once the logits of its range
// [j_lo, j_lo + n_local) are in LDS (zbuf[row][rpb]): per hidden-state row the softmax
// partial and the k best of the range, written as one partial result; then, when the call is
// fused, the last workgroup to arrive merges all partial results and emits the outputs.
template <bool STORE_LOGITS>
__device__ __forceinline__ void block_tail(const GemvArgs& a, u32x4* smem, const float* zbuf, int tid, int j_lo,
                                           int n_local)
{
    const int lane = tid & 63;
    const int wave = tid >> 6;
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
                v[i] = neg_inf();
                if (e < n_local) {
                    // zbuf[slice][row][rpb]: a logit is the sum of its slices' partial sums, in slice order
                    float z = zbuf[r * a.rpb + e];
                    for (int q = 1; q < a.ks; ++q)
                        z += zbuf[(q * a.rows + r) * a.rpb + e];
                    v[i] = z;
                    if (STORE_LOGITS && a.logits_out != nullptr)
                        a.logits_out[(size_t)r * a.Vd + j_lo + e] = z;
                }
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
            __hip_atomic_fetch_add(a.arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
        __hip_atomic_store(a.arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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

    block_tail<false>(a, smem, zbuf, tid, j_lo, n_local);
}

// Matrix-core variant for several hidden-state rows (2..16): the same row-split stream of
// W_sub, but a wave takes 16 consecutive W_sub rows at a time and feeds them to
// v_mfma_f32_16x16x32_bf16 as the A operand (lane l: row l%16, k-offset 8*(l/16) of the 32-wide
// step), the hidden states (LDS, 16-byte pieces XOR-swizzled by row so that the 16 rows of a
// step fall into distinct bank groups) as the B operand.  One MFMA, one 16-byte global load and
// a few LDS accesses per lane per KiB of W_sub whatever the row count, and no cross-lane
// reduction: lane l ends with the logits of hidden row l%16 for W_sub rows 4*(l/16)..+3 of
// the group.  Needs H % 256 == 0 (8 KiB per wave and loop iteration).  A narrow range (fewer
// 16-row groups than waves) is also cut along the hidden dimension: work items are (group,
// slice), every slice leaves partial logits in its own LDS plane, and the planes are added in
// slice order when the range is reduced, so the result does not depend on timing.
//
// STAGED: global loads stay line-sized (a load instruction takes 128 contiguous bytes of each
// of 8 rows; loading straight into the A layout touches 64 different lines per instruction and
// is bound by the L1 tag rate), and a 2 KiB wave-private LDS buffer turns 16 rows x 128 bytes
// into A fragments.  The direct form remains for shapes whose hidden states leave no LDS for
// the staging buffers.
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kMfmaGroup = 16;   // W_sub rows per wave and pass
constexpr int kMfmaUnroll = 8;   // KiB (load instructions) per wave and loop iteration
constexpr int kMfmaStage = 128;  // 16-byte pieces in a wave's staging buffer

template <bool STAGED>
__global__ void __launch_bounds__(kGemvThreads) gemv_mfma_kernel(GemvArgs a)
{
    extern __shared__ u32x4 smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nchunk = a.nchunk;
    float* zbuf = reinterpret_cast<float*>(smem + a.rows * nchunk);  // [ks][rows][rpb]
    u32x4* stage = reinterpret_cast<u32x4*>(zbuf + a.ks * a.rows * a.rpb) + wave * kMfmaStage;  // STAGED only

    const int j_lo = blockIdx.x * a.rpb;
    const int j_hi = (j_lo + a.rpb < a.Vd) ? j_lo + a.rpb : a.Vd;
    const int n_local = j_hi - j_lo;
    const int ngroups = (n_local + kMfmaGroup - 1) / kMfmaGroup;
    const int iters = nchunk / (4 * kMfmaUnroll) / a.ks;  // loop iterations per item (32 pieces each)
    // work item = (group of 16 W_sub rows, slice of the hidden dimension): a narrow range has
    // fewer groups than the workgroup has waves, so each group is cut into ks slices whose
    // partial logits are added up when the range is reduced
    const int nitems = ngroups * a.ks;

    const int lrow = lane & 15;
    const int kg = lane >> 4;
    const int hrow = lrow < a.rows ? lrow : a.rows - 1;  // columns beyond `rows` repeat the last row
    const u32x4* hbase = smem + hrow * nchunk;
    const int hsw = hrow & 15;
    // staged form: lane l loads piece (l%8) ^ f(row) of row l/8 (+8 for odd loads) of a 128-byte
    // column block and parks it at position l, so the A read of piece c of row i is at
    // i*8 + (c ^ f(i)) with f(i) = (i/2)%8: conflict-free on both sides
    const int ld_row = lane >> 3;
    const int ld_piece_a = (lane & 7) ^ ((ld_row >> 1) & 7);        // rows 0..7 of the group
    const int ld_piece_b = (lane & 7) ^ (((ld_row + 8) >> 1) & 7);  // rows 8..15
    const int a_sw = (lrow >> 1) & 7;

    // position = (item, iteration it); the loads of the next position are in flight while the
    // current one is multiplied, also across items
    auto load_pos = [&](int item, int it_in, u32x4(&buf)[kMfmaUnroll]) {
        const int gg = item / a.ks;
        const int it = (item - gg * a.ks) * iters + it_in;
        if constexpr (STAGED) {
            const int jr = j_lo + gg * kMfmaGroup + ld_row;
            const int ja = jr < j_hi ? jr : j_hi - 1;  // a short last group re-reads the range's last row
            const int jb = jr + 8 < j_hi ? jr + 8 : j_hi - 1;
            const u32x4* sa = a.W + (size_t)ja * nchunk + it * (4 * kMfmaUnroll) + ld_piece_a;
            const u32x4* sb = a.W + (size_t)jb * nchunk + it * (4 * kMfmaUnroll) + ld_piece_b;
#pragma unroll
            for (int q = 0; q < kMfmaUnroll / 2; ++q) {
                buf[2 * q] = __builtin_nontemporal_load(sa + 8 * q);
                buf[2 * q + 1] = __builtin_nontemporal_load(sb + 8 * q);
            }
        } else {
            int j = j_lo + gg * kMfmaGroup + lrow;
            j = j < j_hi ? j : j_hi - 1;
            const u32x4* src = a.W + (size_t)j * nchunk + it * (4 * kMfmaUnroll) + kg;
#pragma unroll
            for (int u = 0; u < kMfmaUnroll; ++u)
                buf[u] = src[4 * u];
        }
    };
    f32x4 acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
    int g = wave, it = 0;
    auto step = [&](u32x4(&cur)[kMfmaUnroll], u32x4(&nxt)[kMfmaUnroll]) {
        int itn = it + 1, gn = g;
        if (itn == iters) {
            itn = 0;
            gn = g + kGemvWaves;
        }
        if (gn < nitems)
            load_pos(gn, itn, nxt);
        const int grp = g / a.ks;
        const int slice = g - grp * a.ks;
#pragma unroll
        for (int q = 0; q < kMfmaUnroll / 2; ++q) {
            const int c0 = (slice * iters + it) * (4 * kMfmaUnroll) + 8 * q + kg;  // piece of the first 32-wide step
            u32x4 w0, w1;
            if constexpr (STAGED) {
                stage[lane] = cur[2 * q];
                stage[kWave + lane] = cur[2 * q + 1];
                __builtin_amdgcn_wave_barrier();  // keep the wave's LDS accesses in program order
                w0 = stage[lrow * 8 + (kg ^ a_sw)];
                w1 = stage[lrow * 8 + ((4 + kg) ^ a_sw)];
                __builtin_amdgcn_wave_barrier();
            } else {
                w0 = cur[2 * q];
                w1 = cur[2 * q + 1];
            }
            const u32x4 x0 = hbase[c0 ^ hsw];
            const u32x4 x1 = hbase[(c0 + 4) ^ hsw];
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w0),
                                                           __builtin_bit_cast(bf16x8, x0), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w1),
                                                           __builtin_bit_cast(bf16x8, x1), acc1, 0, 0, 0);
        }
        if (it == iters - 1) {
            const f32x4 z = acc0 + acc1;
            acc0 = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            acc1 = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            if (lrow < a.rows) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = grp * kMfmaGroup + 4 * kg + i;
                    if (e < n_local)
                        zbuf[(slice * a.rows + lrow) * a.rpb + e] = z[i];
                }
            }
        }
        it = itn;
        g = gn;
    };
    u32x4 bufA[kMfmaUnroll], bufB[kMfmaUnroll];
    if (g < nitems)
        load_pos(g, 0, bufA);  // in flight while the hidden states are staged

    for (int x = tid; x < a.rows * nchunk; x += kGemvThreads) {
        const int r = x / nchunk;
        const int c = x - r * nchunk;
        smem[r * nchunk + (c ^ (r & 15))] = a.h[x];
    }
    __syncthreads();
    while (g < nitems) {
        step(bufA, bufB);
        if (g >= nitems)
            break;
        step(bufB, bufA);
    }
    __syncthreads();
    block_tail<true>(a, smem, zbuf, tid, j_lo, n_local);
}

// LDS bytes of the matrix-core streaming kernel without / with the staging buffers
static size_t mfma_lds_bytes(int rows, int nchunk, int rpb, int ks, bool staged)
{
    size_t lds = (size_t)rows * nchunk * sizeof(u32x4) + (size_t)ks * rows * rpb * sizeof(float);
    if (staged)
        lds += (size_t)kGemvWaves * kMfmaStage * sizeof(u32x4);
    return lds;
}

static hipError_t launch_mfma(const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    if (ga.nchunk % (4 * kMfmaUnroll) != 0 || ga.rows > 16)
        return hipErrorInvalidValue;
    if (ga.ks < 1 || (ga.nchunk / (4 * kMfmaUnroll)) % ga.ks != 0)
        return hipErrorInvalidValue;
    const bool staged = mfma_lds_bytes(ga.rows, ga.nchunk, ga.rpb, ga.ks, true) <= (size_t)kGemvLdsLimit;
    size_t lds = mfma_lds_bytes(ga.rows, ga.nchunk, ga.rpb, ga.ks, staged);
    if (ga.fused) {
        if (ga.rows > kFusedMaxRows || ga.P > 256 || ga.KP > 16)
            return hipErrorInvalidValue;
        const size_t l1 = (size_t)ga.rows * 256 * ((size_t)ga.KP + 1) * 8 + kGemvWaves * sizeof(float2);
        lds = lds > l1 ? lds : l1;
    }
    if (lds > (size_t)kGemvLdsLimit)
        return hipErrorInvalidValue;
    auto kern = staged ? gemv_mfma_kernel<true> : gemv_mfma_kernel<false>;
    static std::atomic<size_t> lds_allowed[2] = {{48 * 1024}, {48 * 1024}};  // per variant: raised once, then remembered
    if (lds > lds_allowed[staged].load()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return e;
        lds_allowed[staged].store(lds);
    }
    hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(kGemvThreads), lds, s, ga);
    return hipGetLastError();
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
    static std::atomic<size_t> lds_allowed{48 * 1024};  // per instantiation: raised once, then remembered
    if (lds > lds_allowed.load()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return e;
        lds_allowed.store(lds);
    }
    hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(kGemvThreads), lds, s, ga);
    return hipGetLastError();
}

static void fill_gemv_args(const Plan& p, const HeadArgs& a, GemvArgs& ga);

hipError_t launch_gemv_q(int fmt, const Plan& p, const HeadArgs& a, hipStream_t s)
{
    GemvArgs ga;
    fill_gemv_args(p, a, ga);
    ga.nchunk = 0;  // the compressed kernels take the row length from the plan's hidden size
    if (p.few_rows)
        return launch_gemv_few_rows_q(fmt, p, ga, s);
    return launch_gemv_one_row_q(fmt, p, ga, s);
}

hipError_t launch_gemv(const Plan& p, const HeadArgs& a, hipStream_t s)
{
    GemvArgs ga;
    fill_gemv_args(p, a, ga);
    if (p.one_row)
        return launch_gemv_one_row(p, ga, s);
    if (p.few_rows)
        return launch_gemv_few_rows(p, ga, s);
    if (p.mfma)
        return launch_mfma(p, ga, s);
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

static void fill_gemv_args(const Plan& p, const HeadArgs& a, GemvArgs& ga)
{
    ga.h = reinterpret_cast<const u32x4*>(a.h);
    ga.W = reinterpret_cast<const u32x4*>(a.W);
    ga.scales = a.scales;
    ga.gamma = a.gamma;
    ga.eps = a.eps;
    ga.parent = a.parent;
    ga.h_out = a.h_out;
    ga.rows = p.rows;
    ga.nchunk = p.H / 8;
    ga.Vd = p.Vd;
    ga.P = p.P;
    ga.k = p.k;
    ga.KP = p.KP;
    ga.rpb = p.rpb;
    ga.ks = p.mfma ? p.ks : 1;
    ga.nsg = p.few_rows ? p.nsg : 1;
    ga.part_val = a.part_val;
    ga.part_idx = a.part_idx;
    ga.part_stat = a.part_stat;
    ga.logits_out = a.logits_out;
    ga.fused = p.fused;
    ga.arrive = a.arrive;
    ga.d2t = a.d2t;
    ga.out_ids = a.out_ids;
    ga.out_logp = a.out_logp;
    ga.lse_out = a.lse_out;
}

}  // namespace vt
