// The draft step for a few hidden states at once (2..16 rows: the nodes one tree-drafting step
// expands for one sequence, or a small batch): Section 2.3's projection, bound by reading W_sub
// once whatever the row count, with the log-softmax statistics, the k best per row and the d2t
// remap in the same launch.
//
//   - a workgroup owns a contiguous run of W_sub rows and walks it 16 rows (one MFMA block) at a
//     time; its 16 waves cut the hidden dimension between them: wave w multiplies columns
//     [w * H/16, (w+1) * H/16) of every block, so the hidden states it needs (B operands of
//     v_mfma_f32_16x16x32_bf16, columns beyond `rows` zero) stay in its registers for the whole
//     call and no hidden state passes through LDS;
//   - global loads stay line-sized (an instruction takes 128 contiguous bytes of each of 8 rows);
//     a wave-private LDS buffer turns them into A fragments (lane l: row l % 16, eight columns
//     number l / 16 of a 32-column step).  Eight 1 KiB loads per wave are in flight at all times:
//     the pieces of the next blocks are requested as the current ones are handed to LDS;
//   - after a block's multiplications every wave leaves its 16 x 16 partial sums in LDS, one bare
//     barrier (the loads in flight are not drained), and wave r < rows adds up, in a fixed order,
//     the 16 partials of hidden state r: lane c ends with the logit of block row c.  Wave r keeps
//     state r's softmax statistics (lane c over the block rows c) and its running list of the 16
//     best (lane q of a 16-lane row holds the q-th best); a block row enters the list only if it
//     beats the list's k-th entry -- rare once the list has warmed up -- by one shifted copy and
//     two compares.  Which wave and lane see which W_sub row is fixed by the row's number, so the
//     result does not depend on timing;
//   - a compressed W_sub (FP8 E4M3 with a scale per row, MXFP4 with an exponent per 32 weights: the
//     forms of vt_gemvq.hip) takes the same path: a staged 16-byte piece holds 16 or 32 codes, which
//     the hardware conversions widen to two or four bf16 fragments in registers (exact; an MXFP4
//     block's power of two goes in as the conversion's scale, an FP8 row's scale multiplies the
//     row's finished sum), and the hidden states' fragments are cut to match;
//   - lists travel as 64-bit order keys (logit key, then lower draft index) and are merged by the
//     bitonic network, one wave per hidden state: the lists of each group of 16 workgroups by the
//     last of the group to arrive, then the groups' lists by the last group to finish, which
//     emits ids (through d2t) and log-probabilities.
#include <atomic>

#include "vt_onerow.h"

namespace vt {

constexpr int kFewStageBytes = 2 * 2048;    // per wave: two staging areas of 16 rows x 128 bytes
// LDS map (bytes): staging areas, then two planes of partial sums for each of the NB blocks of an
// iteration (per wave 64 lanes x 16 bytes, one spare piece per 16 lanes); once the stream has ended
// the merge stages' candidates (k64[16 states][256]) overlay the staging areas.
constexpr int kFewLdsStage = 0;
constexpr int kFewLdsPart = kGemvWaves * kFewStageBytes;  // 64 KiB
constexpr int kFewPlaneBytes = 64 * 16 + 5 * 16;  // an odd number of 16-byte pieces: the four quarters of a read fall on two bank groups
constexpr int kFewLdsWl = 0;
constexpr int few_lds_bytes(int nb) { return kFewLdsPart + 2 * nb * kGemvWaves * kFewPlaneBytes; }

// How W_sub is stored (FMT 0: bf16; VT_Q_FP8_E4M3: one byte per weight and an fp32 scale per row;
// VT_Q_MXFP4: two weights per byte and an exponent byte per 32 weights) and what follows from it
// for a wave's share of a row -- H / 16 columns, whole 128-byte lines in every served case.
template <int FMT, int H>
struct FewGeom {
    static constexpr int kCols = H / 16;                                          // columns per wave
    static constexpr int kRowBytes = FMT == 0 ? H * 2 : FMT == VT_Q_FP8_E4M3 ? H : H / 2;
    static constexpr int kPieces = kRowBytes / 16;                                // 16-byte pieces per W_sub row
    static constexpr int kLines = kRowBytes / 16 / 128;                           // 128-byte lines per wave and row
    static constexpr int kSlots = 2 * kLines;                                     // load instructions per 16-row block
    static constexpr int D = kSlots >= 4 ? 8 : 4;                                 // 1 KiB load instructions in flight per wave
    static constexpr int NB = D / kSlots;                                         // 16-row blocks per loop iteration
    static constexpr int kMfmaPerLine = FMT == 0 ? 2 : FMT == VT_Q_FP8_E4M3 ? 4 : 8;  // a line holds 64 / 128 / 256 weights
    static constexpr int kHFrags = kCols / 32;                                    // B fragments (32 columns each)
    static constexpr int kHLines = kCols * 2 / 128;                               // 128-byte lines of a hidden state's share
    static constexpr int kHPieces = H / 8;                                        // 16-byte pieces per hidden state
    static_assert(kLines >= 1 && kRowBytes == kLines * 128 * 16, "a wave reads whole 128-byte lines of a row");
    static_assert(kHFrags == kLines * kMfmaPerLine && kHFrags == 2 * kHLines, "fragment counts agree");
    static_assert(NB >= 1 && NB <= 2, "partial-sum planes for at most two blocks");
};

// Two E4M3 words (eight codes) -> an A fragment of eight bf16 (exact).
__device__ __forceinline__ bf16x8 few_cvt_fp8(uint32_t lo, uint32_t hi)
{
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    const b2 p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false);
    const b2 p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true);
    const b2 p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false);
    const b2 p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true);
    return bf16x8{p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}
// One word of eight E2M1 codes (even element in the low nibble) times a power of two -> eight bf16 (exact).
__device__ __forceinline__ bf16x8 few_cvt_fp4(uint32_t w, float scale)
{
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    const b2 p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, scale, 0);
    const b2 p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, scale, 1);
    const b2 p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, scale, 2);
    const b2 p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, scale, 3);
    return bf16x8{p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}

// SHARED: several workgroups (one per group of 16 hidden states) stream the same W_sub rows side by
// side, so the loads leave the lines in the cache for the neighbours instead of marking them as used once.
template <int FMT, int H, bool SHARED>
__global__ void __launch_bounds__(kGemvThreads) gemv_few_rows_kernel(GemvArgs a)
{
    using G = FewGeom<FMT, H>;
    constexpr int D = G::D;
    constexpr int NB = G::NB;
    constexpr int KSL = G::kSlots;
    constexpr int NHF = G::kHFrags;
    extern __shared__ u32x4 smem[];
    __shared__ int s_flag;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m16 = lane & 15;  // MFMA: row of the A fragment / hidden state of the B fragment and of the result
    const int g4 = lane >> 4;   // MFMA: which eight columns of a 32-column step; the result's rows 4 * g4 ..+3
    char* lds = reinterpret_cast<char*>(smem);

    // More than 16 hidden states are served in groups of 16 by workgroups of their own: workgroup
    // (b, sg) walks run b of W_sub for states 16 sg .. 16 sg + 15.  The workgroups of one run sit next
    // to each other in launch order and on the same XCD (block number modulo 8), so all but the first
    // to ask find the run's lines in that XCD's L2.
    const int nsg = a.nsg;
    const int nb = gridDim.x / nsg;  // runs of W_sub rows
    int b, sg;
    if ((nb & 7) == 0) {
        const int y = blockIdx.x >> 3;
        sg = y % nsg;
        b = (y / nsg) * 8 + (blockIdx.x & 7);
    } else {
        sg = blockIdx.x % nsg;
        b = blockIdx.x / nsg;
    }
    const int s0 = sg * 16;                                     // first hidden state of this workgroup
    const int rows = a.rows - s0 < 16 ? a.rows - s0 : 16;       // and how many it serves
    // rows of this workgroup: an even split of V_draft over the runs, in order
    const int base = a.Vd / nb;
    const int rem = a.Vd - base * nb;
    const int n_wg = base + (b < rem ? 1 : 0);
    const int j0 = b * base + (b < rem ? b : rem);
    const int nblk = (n_wg + 15) >> 4;
    const int niter = (nblk + NB - 1) / NB;

    // Both operands are fetched line-sized: an instruction takes 128 contiguous bytes of each of 8 rows;
    // lane l takes piece (l % 8) ^ f(row) of row l / 8 (+8 for odd instructions) and parks it at
    // position l of a wave-private staging area, so that the fragment read of piece c of row i is at
    // i * 8 + (c ^ f(i)) with f(i) = (i / 2) % 8: no bank conflicts on either side.
    const int ld_row = lane >> 3;
    const int pc_a = (lane & 7) ^ ((ld_row >> 1) & 7);
    const int pc_b = (lane & 7) ^ (((ld_row + 8) >> 1) & 7);

    // B operands: the wave's columns of every hidden state, requested before anything else (hidden
    // states beyond `rows` repeat state 0 and are zeroed once they are fragments)
    u32x4 hreg[NHF];
#pragma unroll
    for (int d = 0; d < NHF; ++d) {
        const int r = ld_row + ((d & 1) ? 8 : 0);
        hreg[d] = a.h[(size_t)(s0 + (r < rows ? r : 0)) * G::kHPieces + wave * (G::kHLines * 8) + (d >> 1) * 8 +
                      ((d & 1) ? pc_b : pc_a)];
    }

    // A operands.  Slot d of an iteration: block d / KSL, 128-byte line (d % KSL) / 2 of the wave's
    // share of the row, rows 0..7 (even d) or 8..15 (odd d) of the block.  Rows past the workgroup's
    // run repeat its last row (their results are dropped).
    const u32x4* wbase = a.W + (size_t)j0 * G::kPieces + wave * (G::kLines * 8);
    u32x4 buf[D];
    auto issue = [&](int it, int d) {
        const int blk = it * NB + d / KSL;
        int r = blk * 16 + ld_row + ((d & 1) ? 8 : 0);
        r = r < n_wg ? r : n_wg - 1;
        const int piece = ((d % KSL) >> 1) * 8 + ((d & 1) ? pc_b : pc_a);
        if constexpr (SHARED)
            buf[d] = wbase[(size_t)r * G::kPieces + piece];
        else
            buf[d] = __builtin_nontemporal_load(wbase + (size_t)r * G::kPieces + piece);
    };
    // Scales.  FP8: the fp32 scale of block row c for lane c, fetched at the start of an iteration for
    // its blocks (used after the block's sums are complete).  MXFP4: the eight exponent bytes of the
    // wave's share of row l % 16 (one 8-byte load; byte g belongs to piece g, byte 4 + g to piece 4 + g),
    // fetched with the block's pieces, one iteration ahead.
    float rsc[NB];
    u32x2 ebuf[NB];
    auto issue_exp = [&](int it, int bi) {
        int r = (it * NB + bi) * 16 + m16;
        r = r < n_wg ? r : n_wg - 1;
        ebuf[bi] = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint8_t*>(a.scales) +
                                                  (size_t)(j0 + r) * (H / 32) + wave * (G::kCols / 32));
    };
#pragma unroll
    for (int d = 0; d < D; ++d) {
        if constexpr (FMT == VT_Q_MXFP4) {
            if (d % KSL == 0)
                issue_exp(0, d / KSL);
        }
        issue(0, d);
        __builtin_amdgcn_sched_barrier(0);  // in slot order, as every later iteration requests them
    }

    u32x4* stage = reinterpret_cast<u32x4*>(lds + kFewLdsStage + wave * kFewStageBytes);
    float* part = reinterpret_cast<float*>(lds + kFewLdsPart);
    const int a_sw = (m16 >> 1) & 7;
    // The hidden states become fragments while the first W_sub pieces are on their way.  Which eight
    // columns lane (state, g) needs for a fragment follows from where the format puts the weights of
    // the piece the lane will read: bf16 pieces g and 4 + g of a line hold columns 8 g.. and 32 + 8 g..
    // of its 64; an FP8 piece holds 16 columns, multiplied as two fragments, so hidden-state pieces
    // 2 g and 2 g + 1; an MXFP4 piece holds 32 columns, four fragments, so pieces 4 (g % 2) + j of
    // hidden-state line g / 2 (of the pair of lines staged together).
    if constexpr (FMT == VT_Q_MXFP4) {
#pragma unroll
        for (int t = 0; t < G::kHLines / 2; ++t) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                stage[e * 128 + lane] = hreg[4 * t + 2 * e];
                stage[e * 128 + kWave + lane] = hreg[4 * t + 2 * e + 1];
            }
            __builtin_amdgcn_wave_barrier();
            u32x4 x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                x[j] = stage[(g4 >> 1) * 128 + m16 * 8 + ((4 * (g4 & 1) + j) ^ a_sw)];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int j = 0; j < 4; ++j)
                hreg[4 * t + j] = m16 < rows ? x[j] : u32x4{0u, 0u, 0u, 0u};
        }
    } else {
#pragma unroll
        for (int c = 0; c < G::kHLines; ++c) {
            u32x4* st = stage + (c & 1) * 128;
            st[lane] = hreg[2 * c];
            st[kWave + lane] = hreg[2 * c + 1];
            __builtin_amdgcn_wave_barrier();
            const int p0 = FMT == 0 ? g4 : 2 * g4;
            const int p1 = FMT == 0 ? 4 + g4 : 2 * g4 + 1;
            const u32x4 x0 = st[m16 * 8 + (p0 ^ a_sw)];
            const u32x4 x1 = st[m16 * 8 + (p1 ^ a_sw)];
            __builtin_amdgcn_wave_barrier();
            hreg[2 * c] = m16 < rows ? x0 : u32x4{0u, 0u, 0u, 0u};
            hreg[2 * c + 1] = m16 < rows ? x1 : u32x4{0u, 0u, 0u, 0u};
        }
    }

    // wave r < rows keeps the results of hidden state s0 + r: the running list of its 16 best (lane q of every
    // 16-lane row holds the q-th best) and, in lane c, the running maximum and sum of exponentials
    // over the block rows c it has seen
    const bool mine = wave < rows;
    const int state = s0 + wave;
    const int kth = a.k - 1;
    int lkey = kKeyNone, lidx = kIdxNone;
    int thr = kKeyNone;  // key of the list's k-th entry: a logit that does not beat it cannot be among the k best
    float rm = neg_inf(), rs = 0.0f;
    f32x4 acc[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
        acc[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    // where the partial sums of (wave p, block bi) of a plane sit, and lane l's 16 bytes in them
    // (one spare piece per 16 lanes spreads the reads below over all banks)
    auto part_at = [&](int buf_i, int bi, int p, int l) {
        return part + ((buf_i * NB + bi) * kGemvWaves + p) * (kFewPlaneBytes / 4) + l * 4 + (l >> 4) * 4;
    };

    auto mfma = [&](const bf16x8& av, int hf, int bi) {
        acc[bi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, hreg[hf]), acc[bi], 0, 0, 0);
    };
    auto iteration = [&](int it, auto more_c) {
        constexpr bool MORE = decltype(more_c)::value;  // another iteration follows: its loads are unconditional
        if constexpr (FMT == VT_Q_FP8_E4M3) {
#pragma unroll
            for (int bi = 0; bi < NB; ++bi) {
                int r = (it * NB + bi) * 16 + m16;
                r = r < n_wg ? r : n_wg - 1;
                rsc[bi] = reinterpret_cast<const float*>(a.scales)[j0 + r];
            }
        }
#pragma unroll
        for (int c = 0; c < D / 2; ++c) {
            u32x4* st = stage + (c & 1) * 128;
            st[lane] = buf[2 * c];
            st[kWave + lane] = buf[2 * c + 1];
            const int bi = (2 * c) / KSL;          // block of the iteration
            const int ln = ((2 * c) % KSL) >> 1;   // line of the wave's share of its rows
            u32x2 eb = {0u, 0u};
            if constexpr (FMT == VT_Q_MXFP4)
                eb = ebuf[bi];
            if (MORE) {
                if constexpr (FMT == VT_Q_MXFP4)
                    issue_exp(it + 1, bi);
                issue(it + 1, 2 * c);
                issue(it + 1, 2 * c + 1);
            }
            __builtin_amdgcn_wave_barrier();  // the wave's LDS accesses stay in program order
            const u32x4 w0 = st[m16 * 8 + (g4 ^ a_sw)];
            const u32x4 w1 = st[m16 * 8 + ((4 + g4) ^ a_sw)];
            __builtin_amdgcn_wave_barrier();
            if constexpr (FMT == 0) {
                mfma(__builtin_bit_cast(bf16x8, w0), 2 * ln, bi);
                mfma(__builtin_bit_cast(bf16x8, w1), 2 * ln + 1, bi);
            } else if constexpr (FMT == VT_Q_FP8_E4M3) {
                mfma(few_cvt_fp8(w0[0], w0[1]), 4 * ln, bi);
                mfma(few_cvt_fp8(w0[2], w0[3]), 4 * ln + 1, bi);
                mfma(few_cvt_fp8(w1[0], w1[1]), 4 * ln + 2, bi);
                mfma(few_cvt_fp8(w1[2], w1[3]), 4 * ln + 3, bi);
            } else {
                // the piece's block exponent becomes the conversion's scale: 2^(byte - 127) as an fp32
                const float sc0 = __uint_as_float(((eb[0] >> (8 * g4)) & 0xffu) << 23);
                const float sc1 = __uint_as_float(((eb[1] >> (8 * g4)) & 0xffu) << 23);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    mfma(few_cvt_fp4(w0[j], sc0), j, bi);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    mfma(few_cvt_fp4(w1[j], sc1), 4 + j, bi);
            }
        }
        // the wave's partial sums of the iteration's blocks go to plane it % 2: lane (state m16, g4)
        // holds block rows 4 g4 .. 4 g4 + 3 of that state
#pragma unroll
        for (int bi = 0; bi < NB; ++bi) {
            *reinterpret_cast<f32x4*>(part_at(it & 1, bi, wave, lane)) = acc[bi];
            acc[bi] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0) only: the loads in flight stay in flight
        __builtin_amdgcn_s_barrier();
        if (!mine)
            return;
        // state `wave`: lane (c = m16, q = g4) adds the partials of waves 4 q .. 4 q + 3 for block row c,
        // two exchanges add the four quarters: every lane c ends with the logit of block row c
#pragma unroll
        for (int bi = 0; bi < NB; ++bi) {
            const int src = (m16 >> 2) * 16 + wave;  // the lane that held (state `wave`, block rows 4 (c / 4) ..)
            const float x0 = part_at(it & 1, bi, 4 * g4 + 0, src)[m16 & 3];
            const float x1 = part_at(it & 1, bi, 4 * g4 + 1, src)[m16 & 3];
            const float x2 = part_at(it & 1, bi, 4 * g4 + 2, src)[m16 & 3];
            const float x3 = part_at(it & 1, bi, 4 * g4 + 3, src)[m16 & 3];
            float z = (x0 + x1) + (x2 + x3);
            z += xchg_f<16>(z, lane);
            z += xchg_f<32>(z, lane);
            if constexpr (FMT == VT_Q_FP8_E4M3)
                z *= rsc[bi];  // the row's scale multiplies the row's sum
            const int jb = (it * NB + bi) * 16;  // the block's first row within the workgroup's run
            const bool valid = jb + m16 < n_wg;
            const int zk = valid ? f2key(z) : kKeyNone;
            if (valid) {
                // one exponential per logit: the smaller of (running maximum, logit) is rescaled
                const float d = z - rm;
                const float e = __expf(-fabsf(d));
                rs = d > 0.0f ? rs * e + 1.0f : rs + e;
                rm = fmaxf(rm, z);
                if (a.logits_out != nullptr && g4 == 0)
                    a.logits_out[(size_t)state * a.Vd + j0 + jb + m16] = z;
            }
            // block rows that beat the list's k-th entry enter the list one by one, in row order
            // (ties keep the earlier, lower index ahead)
            unsigned int todo = (unsigned int)__builtin_amdgcn_ballot_w64(zk > thr) & 0xffffu;
            while (todo != 0u) {
                const int c = __builtin_ctz(todo);
                todo &= todo - 1u;
                const int zs = __builtin_amdgcn_readlane(zk, c);
                if (zs > thr) {
                    const int sk = row_shr1(lkey, kKeyMax);
                    const int si = row_shr1(lidx, kIdxNone);
                    const bool c0 = zs > lkey;
                    const bool c1 = zs > sk;
                    lkey = c0 ? (c1 ? sk : zs) : lkey;
                    lidx = c0 ? (c1 ? si : j0 + jb + c) : lidx;
                    thr = __builtin_amdgcn_readlane(lkey, kth);
                }
            }
        }
    };
    // (a loop of the steady form alone, the last iteration on its own: the compiler then knows the
    // number of loads in flight at every wait)
    for (int it = 0; it + 1 < niter; ++it)
        iteration(it, std::true_type{});
    iteration(niter - 1, std::false_type{});
    __syncthreads();  // staging areas and partial planes are dead from here on

    // ---- the workgroup's result for state `wave` is the wave's own list and statistics ----
    k64* cand = reinterpret_cast<k64*>(lds + kFewLdsWl) + wave * 256;  // the wave's own 2 KiB (fetched lists)
    k64 best = k64_make(lkey, lidx);
    float mm = rm, ss = rs;
    if (mine)
        wave_stat_merge(mm, ss, lane < 16);
    // a result list goes to slot `slot` of the workspace: [slot][state] lists of 16 and one (max, sum) pair
    auto publish = [&](int slot) {
        if (mine) {
            const size_t at = (size_t)slot * a.rows + state;
            if (lane < 16) {
                st_dev(a.part_val + at * 16 + lane, key2f(k64_key(best)));
                st_dev(a.part_idx + at * 16 + lane, k64_idx(best));
            }
            if (lane == 0) {
                st_dev(reinterpret_cast<float*>(a.part_stat + at), mm);
                st_dev(reinterpret_cast<float*>(a.part_stat + at) + 1, ss);
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the coherent stores are acknowledged
        __syncthreads();
    };
    // the lists of slots first .. first + count - 1 (count <= 16), merged per hidden state
    auto merge_slots = [&](int first, int count) {
        if (!mine)
            return;
        f32x4 v = {neg_inf(), neg_inf(), neg_inf(), neg_inf()};
        i32x4 ix = {kIdxNone, kIdxNone, kIdxNone, kIdxNone};
        float2 st = make_float2(neg_inf(), 0.0f);
        const int li = lane >> 2;  // lane l: entries 4 * (l % 4) ..+3 of list l / 4
        if (li < count) {
            const size_t at = ((size_t)(first + li) * a.rows + state) * 16 + 4 * (lane & 3);
            coherent_load_issue(v, a.part_val + at);
            coherent_load_issue(ix, a.part_idx + at);
        }
        const bool act = lane < count;
        if (act)
            coherent_load_issue(st, a.part_stat + (size_t)(first + lane) * a.rows + state);
        coherent_load_wait(v, ix, st);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            cand[4 * lane + q] = k64_make(f2key(v[q]), ix[q]);
        __builtin_amdgcn_wave_barrier();
        best = k64_merge_16_lists(cand, lane);
        mm = st.x;
        ss = st.y;
        wave_stat_merge(mm, ss, act);
    };
    auto emit = [&]() {
        if (!mine)
            return;
        const float lse = mm + __logf(ss);
        if (lane < a.k) {
            const int oi = k64_idx(best);
            a.out_ids[(size_t)state * a.k + lane] = (oi != kIdxNone) ? a.d2t[oi] : -1;
            a.out_logp[(size_t)state * a.k + lane] =
                (key2f(k64_key(best)) - lse) + (a.parent != nullptr ? a.parent[state] : 0.0f);
        }
        if (lane == 0 && a.lse_out != nullptr)
            a.lse_out[state] = lse;
    };

    // The workgroups of one group of states arrive in two levels (groups of 16, then the groups).
    // Arrival counters in the workspace header: state group sg owns counters 1 + sg * (16 / nsg) ..
    // for its groups of workgroups, and counter 0 (sg = 0) or 16 + sg for the call.
    const int P = nb;
    const int grp = b >> 4;
    const int ngrp = (P + 15) >> 4;
    const int in_grp = (grp == ngrp - 1) ? P - grp * 16 : 16;
    unsigned int* call_ctr = a.arrive + (sg == 0 ? 0 : 16 + sg) * kArriveStrideWords;
    if (P == 1) {  // nothing to wait for
        emit();
        return;
    }
    publish(b);
    if (tid == 0) {
        unsigned int* ctr = a.arrive + (1 + sg * (16 / nsg) + grp) * kArriveStrideWords;
        const unsigned int t = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = ((int)t == in_grp - 1) ? 1 : 0;
        if (last)
            __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_flag = last;
    }
    __syncthreads();
    if (!s_flag)
        return;
    // ---- the last workgroup of its group of 16 merges the group's lists ----
    merge_slots(grp * 16, in_grp);
    if (ngrp == 1) {
        emit();
        return;
    }
    publish(P + grp);  // (every thread has read s_flag before this barrier)
    if (tid == 0) {
        const unsigned int t = __hip_atomic_fetch_add(call_ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = ((int)t == ngrp - 1) ? 1 : 0;
        if (last)
            __hip_atomic_store(call_ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_flag = last;
    }
    __syncthreads();
    if (!s_flag)
        return;
    // ---- the last group to finish merges the groups' lists and ends the call ----
    merge_slots(P, ngrp);
    emit();
}

// What the kernel assumes of a launch: 1..64 hidden states in nsg groups of 16, lists of 16, per group
// of states at most 256 / nsg workgroups (16 / nsg groups of 16, so that the arrival counters fit the
// workspace header), result slots for every workgroup and every group of workgroups.
static bool few_rows_launch_ok(const Plan& p, const GemvArgs& ga)
{
    const int nsg = ga.nsg;
    if (!(p.few_rows && ga.rows >= 1 && nsg >= 1 && nsg <= 4 && nsg == (ga.rows + 15) / 16))
        return false;
    const int nb = p.blocks / nsg;
    return p.blocks == nb * nsg && nb >= 1 && nb <= 16 * (16 / nsg) && ga.KP == 16 && ga.k <= 16 && ga.P == nb + 16 &&
           ga.fused && (p.H == 2048 || p.H == 4096);
}

template <int FMT, int H, bool SHARED>
static hipError_t launch_few_t(const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    constexpr int lds = few_lds_bytes(FewGeom<FMT, H>::NB);
    static_assert(lds <= kGemvLdsLimit, "fits a compute unit's LDS");
    static std::atomic<int> raised{0};  // the dynamic LDS limit of this instantiation is raised once
    if (!raised.load()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_few_rows_kernel<FMT, H, SHARED>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess)
            return e;
        raised.store(1);
    }
    hipLaunchKernelGGL((gemv_few_rows_kernel<FMT, H, SHARED>), dim3(p.blocks), dim3(kGemvThreads), lds, s, ga);
    return hipGetLastError();
}

template <int FMT, int H>
static hipError_t launch_few_fh(const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    return ga.nsg > 1 ? launch_few_t<FMT, H, true>(p, ga, s) : launch_few_t<FMT, H, false>(p, ga, s);
}

hipError_t launch_gemv_few_rows(const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    if (!few_rows_launch_ok(p, ga) || ga.nchunk != p.H / 8)
        return hipErrorInvalidValue;
    return p.H == 4096 ? launch_few_fh<0, 4096>(p, ga, s) : launch_few_fh<0, 2048>(p, ga, s);
}

// The same over a compressed W_sub: FP8 at H = 2048 / 4096, MXFP4 at H = 4096 (a wave's share of a row is
// then at least one 128-byte line).
hipError_t launch_gemv_few_rows_q(int fmt, const Plan& p, const GemvArgs& ga, hipStream_t s)
{
    if (!few_rows_launch_ok(p, ga) || ga.scales == nullptr)
        return hipErrorInvalidValue;
    if (fmt == VT_Q_FP8_E4M3)
        return p.H == 4096 ? launch_few_fh<VT_Q_FP8_E4M3, 4096>(p, ga, s) : launch_few_fh<VT_Q_FP8_E4M3, 2048>(p, ga, s);
    if (fmt == VT_Q_MXFP4 && p.H == 4096)
        return launch_few_fh<VT_Q_MXFP4, 4096>(p, ga, s);
    return hipErrorInvalidValue;
}

}  // namespace vt
