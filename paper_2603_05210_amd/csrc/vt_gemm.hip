// Tree-drafting regime of the draft head (hundreds to a thousand hidden-state rows): the
// projection of Section 2.3 of the paper, z[r,j] = sum_i h[r,i] W_sub[j,i], is now a dense
// contraction with ~500-1000 FLOP per byte and runs on the bf16 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// MFMA roles: the A operand is a W_sub tile (matrix rows = draft tokens), the B operand an h
// tile (matrix columns = hidden-state rows).  In the 32x32 accumulator layout a lane then owns
// ONE hidden-state row (column l%32) and 16 draft tokens per sub-tile, so the fused epilogue
// (softmax statistics and the k best candidates over the tile's vocabulary slice) runs
// lane-private on the accumulators with no shuffles and no LDS, in ascending token order.
// Each lane's partial goes to the workspace; the merge kernel finishes the row.  Logits are
// never written (except in the test hook).
//
// Data movement: both operands are K-contiguous, so a tile row is 64 bf16 = 128 B = eight
// 16-byte pieces.  Global loads are 128-bit, 8 adjacent lanes per row segment; LDS rows are
// 128 B with the piece index XOR-swizzled by (row/2)%8 so that the 16-byte fragment reads of
// 32 different rows spread over all banks.  Two LDS stages; the next stage's global loads
// are issued before the current stage's MFMAs.
#include "vt_device.h"
#include "vt_internal.h"

namespace vt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GemmArgs {
    const u32x4* h;
    const u32x4* W;
    int rows, nchunk, Vd, P;
    int n_vtiles, n_rtiles;
    float* part_val;
    int32_t* part_idx;
    float2* part_stat;
    float* logits_out;
};

template <int WV, int WR, int SV, int SR, int KP>
__global__ void __launch_bounds__(WV* WR * 64) gemm_head_kernel(GemmArgs a)
{
    constexpr int BMV = WV * SV * 32;    // draft tokens per workgroup tile
    constexpr int BNR = WR * SR * 32;    // hidden-state rows per workgroup tile
    constexpr int NT = WV * WR * 64;
    constexpr int TROWS = BMV + BNR;     // LDS rows per stage (W_sub rows, then h rows)
    constexpr int STAGE = TROWS * 8;     // 16-byte pieces per stage
    constexpr int NLD = STAGE / NT;      // 16-byte global loads per thread per stage
    constexpr int NLD_W = BMV * 8 / NT;  // the first NLD_W of them read W_sub
    static_assert(STAGE % NT == 0 && (BMV * 8) % NT == 0, "tile must split evenly over the threads");
    static_assert(NT % 8 == 0 && (NT / 8) % 16 == 0, "row stride per load must keep the swizzle per-thread constant");
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

    // ---- global -> register staging ----
    const int lrow = tid >> 3;  // + i * (NT/8)
    const int lc = tid & 7;
    const u32x4* gsrc[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int rowid = lrow + i * (NT / 8);
        if (i < NLD_W) {
            int v = v0 + rowid;
            v = v < a.Vd ? v : a.Vd - 1;
            gsrc[i] = a.W + (size_t)v * nchunk + lc;
        } else {
            int r = r0 + rowid - BMV;
            r = r < a.rows ? r : a.rows - 1;
            gsrc[i] = a.h + (size_t)r * nchunk + lc;
        }
    }
    const int st_off = lrow * 8 + (lc ^ ((lrow >> 1) & 7));  // + i * (NT/8) * 8

    u32x4 stage[NLD];
    auto load_stage = [&](int kt) {
        const bool ok = (kt * 8 + lc) < nchunk;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            u32x4 zero = {0u, 0u, 0u, 0u};
            stage[i] = ok ? gsrc[i][kt * 8] : zero;
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            smem[buf * STAGE + st_off + i * (NT / 8) * 8] = stage[i];
    };

    // ---- fragment addressing ----
    const int frow = lane & 31;
    const int fhalf = lane >> 5;
    const int fsw = (lane >> 1) & 7;
    const int a_base = (wv * SV * 32 + frow) * 8;
    const int b_base = (BMV + wr * SR * 32 + frow) * 8;

    f32x16 acc[SV][SR];
#pragma unroll
    for (int sv = 0; sv < SV; ++sv)
#pragma unroll
        for (int sr = 0; sr < SR; ++sr)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[sv][sr][e] = 0.0f;

    const int KT = (nchunk + 7) >> 3;
    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT)
            load_stage(kt + 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int pc = ((ks * 2 + fhalf) ^ fsw);
            bf16x8 af[SV], bfr[SR];
#pragma unroll
            for (int sv = 0; sv < SV; ++sv)
                af[sv] = __builtin_bit_cast(bf16x8, smem[buf * STAGE + a_base + sv * 32 * 8 + pc]);
#pragma unroll
            for (int sr = 0; sr < SR; ++sr)
                bfr[sr] = __builtin_bit_cast(bf16x8, smem[buf * STAGE + b_base + sr * 32 * 8 + pc]);
#pragma unroll
            for (int sv = 0; sv < SV; ++sv)
#pragma unroll
                for (int sr = 0; sr < SR; ++sr)
                    acc[sv][sr] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[sv], bfr[sr], acc[sv][sr], 0, 0, 0);
        }
        if (kt + 1 < KT)
            store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- fused epilogue, lane-private on the accumulators ----
    // accumulator element e of sub-tile (sv, sr): draft token v0 + wv*SV*32 + sv*32 + 8*(e/4) + 4*(lane/32) + e%4,
    // hidden-state row r0 + wr*SR*32 + sr*32 + lane%32.
    const int tok_base = v0 + wv * SV * 32 + 4 * fhalf;
    const int part = (vt_i * WV + wv) * 2 + fhalf;
#pragma unroll
    for (int sr = 0; sr < SR; ++sr) {
        const int row = r0 + wr * SR * 32 + sr * 32 + frow;
        const bool row_ok = row < a.rows;
        float mx = neg_inf();
#pragma unroll
        for (int sv = 0; sv < SV; ++sv)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int tok = tok_base + sv * 32 + 8 * (e >> 2) + (e & 3);
                if (tok >= a.Vd)
                    acc[sv][sr][e] = neg_inf();
                mx = fmaxf(mx, acc[sv][sr][e]);
            }
        TopList<KP> L;
        L.clear();
        float s = 0.0f;
#pragma unroll
        for (int sv = 0; sv < SV; ++sv)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int tok = tok_base + sv * 32 + 8 * (e >> 2) + (e & 3);
                const float z = acc[sv][sr][e];
                if (mx > neg_inf())
                    s += __expf(z - mx);
                L.insert_ordered(z, tok < a.Vd ? tok : kIdxNone);
                if (a.logits_out != nullptr && row_ok && tok < a.Vd)
                    a.logits_out[(size_t)row * a.Vd + tok] = z;
            }
        if (row_ok) {
            const size_t slot = (size_t)row * a.P + part;
#pragma unroll
            for (int q = 0; q < KP; ++q) {
                a.part_val[slot * KP + q] = L.v[q];
                a.part_idx[slot * KP + q] = L.i[q];
            }
            a.part_stat[slot] = make_float2(mx, s);
        }
    }
}

// ---- tile shapes ----
// tile 0: 128 tokens x 128 rows, 4 waves (2x2), 64x64 per wave.
// tile 1: 256 tokens x 256 rows, 4 waves (2x2), 128x128 per wave.
struct TileInfo {
    int BMV, BNR, parts_per_vtile;
};
static const TileInfo kTiles[] = {{128, 128, 4}, {256, 256, 4}};

void gemm_tile_dims(int tile, int& BMV, int& BNR, int& parts_per_vtile)
{
    BMV = kTiles[tile].BMV;
    BNR = kTiles[tile].BNR;
    parts_per_vtile = kTiles[tile].parts_per_vtile;
}

int gemm_pick_tile(int rows, int Vd, int KP)
{
    (void)Vd;
    if (KP > 16 || rows <= 128)
        return 0;
    return 1;
}

template <int WV, int WR, int SV, int SR, int KP>
static hipError_t launch_tile(const Plan& p, const GemmArgs& ga, hipStream_t s)
{
    constexpr int BMV = WV * SV * 32, BNR = WR * SR * 32, NT = WV * WR * 64;
    const size_t lds = (size_t)2 * (BMV + BNR) * 128;
    auto kern = gemm_head_kernel<WV, WR, SV, SR, KP>;
    static size_t lds_allowed = 48 * 1024;  // per instantiation: raised once, then remembered
    if (lds > lds_allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return e;
        lds_allowed = lds;
    }
    hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(NT), lds, s, ga);
    return hipGetLastError();
}

template <int KP>
static hipError_t launch_kp(const Plan& p, const GemmArgs& ga, hipStream_t s)
{
    if (p.tile == 0)
        return launch_tile<2, 2, 2, 2, KP>(p, ga, s);
    if constexpr (KP <= 16) {
        if (p.tile == 1)
            return launch_tile<2, 2, 4, 4, KP>(p, ga, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemm(const Plan& p, const HeadArgs& a, hipStream_t s)
{
    GemmArgs ga;
    ga.h = reinterpret_cast<const u32x4*>(a.h);
    ga.W = reinterpret_cast<const u32x4*>(a.W);
    ga.rows = p.rows;
    ga.nchunk = p.H / 8;
    ga.Vd = p.Vd;
    ga.P = p.P;
    ga.n_vtiles = p.n_vtiles;
    ga.n_rtiles = p.n_rtiles;
    ga.part_val = a.part_val;
    ga.part_idx = a.part_idx;
    ga.part_stat = a.part_stat;
    ga.logits_out = a.logits_out;
    switch (p.KP) {
    case 1: return launch_kp<1>(p, ga, s);
    case 2: return launch_kp<2>(p, ga, s);
    case 4: return launch_kp<4>(p, ga, s);
    case 8: return launch_kp<8>(p, ga, s);
    case 16: return launch_kp<16>(p, ga, s);
    case 32: return launch_kp<32>(p, ga, s);
    case 64: return launch_kp<64>(p, ga, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace vt
