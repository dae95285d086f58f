// Pure host part of the C ABI of include/vt.h: status strings, the argument checks that every
// entry point runs before it launches anything, and the per-call plan (which kernel family, how
// many partial results, where they live in the caller's workspace).  No HIP dependency, so the
// same file is also compiled with the host sanitizers by the test suite.
#include "vt.h"

#include <vector>

#include "vt_plan.h"

namespace vt {

static_assert(kWorkspaceHeader == VT_WORKSPACE_HEADER_BYTES, "header size is part of the C ABI");

static int next_pow2(int x)
{
    int p = 1;
    while (p < x)
        p <<= 1;
    return p;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- GEMM tile shapes ----
// tile 0: 128 tokens x 128 rows, 4 waves (2x2), 64x64 per wave: any k <= 64, any H % 8 == 0.
// tile 1: 256 tokens x 256 rows, 8 waves (2x4), 128x64 per wave (128 accumulators, two waves per
//         SIMD hide each other's LDS / barrier / epilogue stalls; operand traffic from L2 is that
//         of the largest tile): k <= 16, H % 64 == 0.
// tile 2: 32 tokens x 128 rows, 4 waves (1x4), 32x32 per wave: for at most 128 rows over a narrow
//         vocabulary, where 128-token tiles would leave most compute units without a workgroup
//         (the shape is bound by reading W_sub once, not by the matrix cores).
struct TileInfo {
    int BMV, BNR, parts_per_vtile;
};
static const TileInfo kTiles[] = {{128, 128, 4}, {256, 256, 4}, {32, 128, 2}};

void gemm_tile_dims(int tile, int& BMV, int& BNR, int& parts_per_vtile)
{
    BMV = kTiles[tile].BMV;
    BNR = kTiles[tile].BNR;
    parts_per_vtile = kTiles[tile].parts_per_vtile;
}

int gemm_pick_tile(int rows, int H, int Vd, int KP)
{
    // one row tile and fewer 128-token tiles than three quarters of the compute units: narrow tiles
    if (rows <= 128 && (Vd + 127) / 128 < 192)
        return 2;
    // the large tile has no K-tail variant and no room for long candidate lists
    if (KP > 16 || rows <= 128 || (H % 64) != 0)
        return 0;
    // a grid of large tiles that leaves a quarter of the compute units idle: the time of the step is the
    // time of one tile's whole K loop, which the 128 x 128 tile walks twice as fast (measured at H = 4096:
    // 512 rows x 13 264 tokens 114 -> 98 us, 256 x 13 264 109 -> 68, 1024 x 4380 119 -> 92; from 208 large
    // tiles on -- 1024 x 13 264 -- the large tile wins, 142 vs 178 us)
    const int large = ((Vd + 255) / 256) * ((rows + 255) / 256);
    if (large < 192)
        return 0;
    return 1;
}

bool make_plan(int64_t rows, int64_t H, int64_t Vd, int k, Plan& p)
{
    p = Plan{};
    p.rows = (int)rows;
    p.H = (int)H;
    p.Vd = (int)Vd;
    p.k = k;
    p.KP = next_pow2(k);
    bool streaming = rows <= kGemvMaxRows;
    if (streaming) {
        p.NR = next_pow2((int)rows);
        p.J = p.NR == 1 ? 1 : 2;
        int rpb = (int)((Vd + kGemvTargetBlocks - 1) / kGemvTargetBlocks);
        rpb = (rpb + 7) / 8 * 8;
        if (rpb > kGemvMaxRowsPerBlock)
            rpb = kGemvMaxRowsPerBlock;
        p.rpb = rpb;
        // hidden states and the range's logits live in LDS; very wide rows go to the other regime
        const size_t lds = (size_t)p.NR * (size_t)H * 2 + (size_t)p.NR * rpb * 4;
        if (lds > (size_t)kGemvLdsLimit)
            streaming = false;
    }
    const bool one_row = rows == 1 && p.KP <= 16 && (H == 512 || H == 1024 || H == 2048 || H == 4096) &&
                         Vd <= (int64_t)kGemvTargetBlocks * kGemvWaves * 64;
    if (one_row) {
        // one wave per run of W_sub rows, 16 waves per workgroup, at most one workgroup per compute unit
        p.regime = 0;
        p.one_row = 1;
        p.KP = 16;  // the one-row kernel always carries lists of 16
        p.NR = 1;
        p.J = 1;
        p.rpb = 0;
        int blocks = (int)((Vd + kGemvWaves - 1) / kGemvWaves);
        p.blocks = blocks > kGemvTargetBlocks ? kGemvTargetBlocks : blocks;  // measured: 128 or 64 workgroups are slower at every size
        p.P = p.blocks;
        p.fused = 1;
        p.ks = 1;
    } else if (rows >= 2 && rows <= kFewMaxRows && p.KP <= 16 && (H == 2048 || H == 4096) &&
               (rows <= 32 || Vd <= kFewWideMaxVd)) {
        // 16 waves share each block of 16 W_sub rows; every group of 16 rows has workgroups of its own
        // (at most one workgroup per compute unit in all, a multiple of 8 per group so that the
        // workgroups reading the same W_sub rows share an XCD); the workspace holds, per row, a result
        // slot per workgroup of its group and one per 16 of them
        static const int kRuns[4] = {256, 128, 80, 64};
        p.regime = 0;
        p.few_rows = 1;
        p.nsg = (int)((rows + 15) / 16);
        p.KP = 16;
        p.NR = 16;
        p.J = 1;
        p.rpb = 0;
        int runs = (int)((Vd + 15) / 16);
        runs = runs > kRuns[p.nsg - 1] ? kRuns[p.nsg - 1] : runs;
        p.blocks = runs * p.nsg;
        p.P = runs + 16;
        p.fused = 1;
        p.ks = 1;
    } else if (streaming) {
        p.regime = 0;
        p.blocks = (int)((Vd + p.rpb - 1) / p.rpb);
        p.P = p.blocks;
        // fusing pays while one workgroup can finish all rows in one pass
        p.fused = (rows <= 2 && p.P <= 256 && p.KP <= 16) ? 1 : 0;
        // five rows or more: matrix-core variant (measured: 93.6 vs 104 us at 8 rows, 96 vs 165 us at
        // 16; the dot-product form wins up to 4 rows).  A range with fewer 16-row groups than the
        // workgroup has waves is also cut along the hidden dimension (ks slices per group).
        p.mfma = (rows >= 5 && H % 256 == 0) ? 1 : 0;
        p.ks = 1;
        if (p.mfma) {
            const int groups = (p.rpb + 15) / 16;
            const int iters = (int)(H / 256);
            while (groups * p.ks < kGemvWaves && iters % (p.ks * 2) == 0)
                p.ks *= 2;
        }
    } else {
        p.regime = 1;
        p.tile = gemm_pick_tile((int)rows, (int)H, (int)Vd, p.KP);
        int BMV, BNR, ppv;
        gemm_tile_dims(p.tile, BMV, BNR, ppv);
        p.n_vtiles = (int)((Vd + BMV - 1) / BMV);
        p.n_rtiles = (int)((rows + BNR - 1) / BNR);
        const int total = p.n_vtiles * p.n_rtiles;
        p.blocks = ((total + 7) / 8) * 8;
        p.P = p.n_vtiles * ppv;
    }
    const size_t n = (size_t)p.rows * (size_t)p.P;
    p.off_val = kWorkspaceHeader;
    p.off_idx = align_up(p.off_val + n * p.KP * sizeof(float), 256);
    p.off_stat = align_up(p.off_idx + n * p.KP * sizeof(int32_t), 256);
    p.total_bytes = align_up(p.off_stat + n * 2 * sizeof(float), 256);  // (max, sum exp) pairs
    return true;
}

bool make_plan_q(int fmt, int64_t rows, int64_t H, int64_t Vd, int k, Plan& p)
{
    if (k < 1 || k > 16 || Vd < 1)
        return false;
    if (rows == 1 && fmt == VT_Q_MXFP4 && H == 4096 && Vd >= kFewOneRowMinVd) {
        // one MXFP4 row over a wide vocabulary: the kernel for a few rows with one state (its MFMA form
        // of the 4-bit conversion measured faster than the one-row kernel's dot products from V_draft
        // = 13 264 up: 15.4 vs 16.1 us there, 50.6 vs 53.7 us at 128 256; FP8 measured no faster)
        if (!make_plan(2, 4096, Vd, k, p) || !p.few_rows)
            return false;
        p.rows = 1;
    } else if (rows == 1) {
        const bool h_ok = (fmt == VT_Q_FP8_E4M3 && (H == 1024 || H == 2048 || H == 4096)) ||
                          (fmt == VT_Q_MXFP4 && (H == 2048 || H == 4096));
        if (!h_ok || Vd > (int64_t)kGemvTargetBlocks * kGemvWaves * 64)
            return false;
        // the one-row plan of the bf16 head with the same V_draft and k (the hidden size only selects the kernel)
        if (!make_plan(1, 4096, Vd, k, p) || !p.one_row)
            return false;
    } else {
        // a few rows: the plan of the bf16 kernel for a few rows (a wave's share of a compressed row must
        // still be whole 128-byte lines: FP8 from H = 2048, MXFP4 at H = 4096)
        const bool h_ok = (fmt == VT_Q_FP8_E4M3 && (H == 2048 || H == 4096)) || (fmt == VT_Q_MXFP4 && H == 4096);
        if (!h_ok || !make_plan(rows, 4096, Vd, k, p) || !p.few_rows)
            return false;
    }
    p.H = (int)H;
    return true;
}

static bool shape_ok(int64_t rows, int64_t H, int64_t Vd)
{
    const int64_t lim = (int64_t)1 << 31;
    if (rows < 1 || H < 8 || Vd < 1 || (H % 8) != 0)
        return false;
    if (rows >= lim || H >= lim || Vd >= lim)
        return false;
    if (rows * Vd >= ((int64_t)1 << 40) || Vd * (H / 8) >= lim)
        return false;
    return true;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace vt

using namespace vt;

extern "C" {

int vt_version(void) { return 100; }

const char* vt_status_str(vt_status s)
{
    switch (s) {
    case VT_OK: return "VT_OK";
    case VT_ERR_NULL: return "VT_ERR_NULL: a required pointer is NULL";
    case VT_ERR_SHAPE: return "VT_ERR_SHAPE: rows, H, V or V_draft out of range, or H not a multiple of 8";
    case VT_ERR_K: return "VT_ERR_K: k outside [1, min(V_draft, VT_MAX_K)]";
    case VT_ERR_ID_RANGE: return "VT_ERR_ID_RANGE: a token id is outside [0, V)";
    case VT_ERR_ID_DUP: return "VT_ERR_ID_DUP: a token id occurs twice";
    case VT_ERR_WORKSPACE: return "VT_ERR_WORKSPACE: workspace missing or too small";
    case VT_ERR_ALIGN: return "VT_ERR_ALIGN: a device pointer is not 16-byte aligned";
    case VT_ERR_DEVICE: return "VT_ERR_DEVICE: the HIP runtime reported an error";
    }
    return "unknown vt_status";
}

vt_status vt_validate_build_subset_args(const void* full_W, int64_t V, int64_t H, const void* token_ids,
                                        int64_t V_draft, const void* W_sub_out, const void* d2t_out)
{
    if (!full_W || !token_ids || !W_sub_out || !d2t_out)
        return VT_ERR_NULL;
    if (V < 1 || V >= ((int64_t)1 << 31) || V_draft > V || !shape_ok(1, H, V_draft) || V * (H / 8) >= ((int64_t)1 << 31))
        return VT_ERR_SHAPE;
    if (!aligned16(full_W) || !aligned16(W_sub_out) || (reinterpret_cast<uintptr_t>(token_ids) & 3u) ||
        (reinterpret_cast<uintptr_t>(d2t_out) & 3u))
        return VT_ERR_ALIGN;
    return VT_OK;
}

vt_status vt_check_token_ids_host(const int32_t* ids, int64_t V_draft, int64_t V)
{
    if (!ids)
        return VT_ERR_NULL;
    if (V < 1 || V_draft < 1 || V_draft > V || V >= ((int64_t)1 << 31))
        return VT_ERR_SHAPE;
    std::vector<bool> seen((size_t)V, false);
    for (int64_t j = 0; j < V_draft; ++j) {
        const int32_t id = ids[j];
        if (id < 0 || id >= V)
            return VT_ERR_ID_RANGE;
        if (seen[(size_t)id])
            return VT_ERR_ID_DUP;
        seen[(size_t)id] = true;
    }
    return VT_OK;
}

vt_status vt_validate_draft_head_args(const void* h, int64_t rows, int64_t H, const void* W_sub, const void* d2t,
                                      int64_t V_draft, int k, const void* out_target_ids, const void* out_logprobs,
                                      const void* workspace, size_t workspace_bytes)
{
    if (!h || !W_sub || !d2t || !out_target_ids || !out_logprobs)
        return VT_ERR_NULL;
    if (!shape_ok(rows, H, V_draft))
        return VT_ERR_SHAPE;
    if (k < 1 || k > VT_MAX_K || k > V_draft)
        return VT_ERR_K;
    if (!aligned16(h) || !aligned16(W_sub) || (reinterpret_cast<uintptr_t>(d2t) & 3u) ||
        (reinterpret_cast<uintptr_t>(out_target_ids) & 3u) || (reinterpret_cast<uintptr_t>(out_logprobs) & 3u))
        return VT_ERR_ALIGN;
    const size_t need = vt_draft_head_workspace_bytes(rows, H, V_draft, k);
    if (!workspace || workspace_bytes < need)
        return VT_ERR_WORKSPACE;
    if (!aligned16(workspace))
        return VT_ERR_ALIGN;
    return VT_OK;
}

size_t vt_draft_head_workspace_bytes(int64_t rows, int64_t H, int64_t V_draft, int k)
{
    if (!shape_ok(rows, H, V_draft) || k < 1 || k > VT_MAX_K || k > V_draft)
        return 0;
    Plan p;
    if (!make_plan(rows, H, V_draft, k, p))
        return 0;
    return p.total_bytes;
}

size_t vt_subset_q_code_bytes(int fmt, int64_t V_draft, int64_t H)
{
    if (V_draft < 1 || H < 32 || V_draft >= ((int64_t)1 << 31) || H >= ((int64_t)1 << 31))
        return 0;
    if (fmt == VT_Q_FP8_E4M3 && H % 16 == 0)
        return (size_t)V_draft * (size_t)H;
    if (fmt == VT_Q_MXFP4 && H % 32 == 0)
        return (size_t)V_draft * (size_t)H / 2;
    return 0;
}

size_t vt_subset_q_scale_bytes(int fmt, int64_t V_draft, int64_t H)
{
    if (vt_subset_q_code_bytes(fmt, V_draft, H) == 0)
        return 0;
    return fmt == VT_Q_FP8_E4M3 ? (size_t)V_draft * sizeof(float) : (size_t)V_draft * (size_t)(H / 32);
}

size_t vt_draft_head_q_workspace_bytes(int fmt, int64_t rows, int64_t H, int64_t V_draft, int k)
{
    Plan p;
    if (!make_plan_q(fmt, rows, H, V_draft, k, p))
        return 0;
    return p.total_bytes;
}

int vt_draft_head_regime(int64_t rows, int64_t H, int64_t V_draft, int k)
{
    if (!shape_ok(rows, H, V_draft) || k < 1 || k > VT_MAX_K || k > V_draft)
        return -1;
    Plan p;
    if (!make_plan(rows, H, V_draft, k, p))
        return -1;
    return p.regime;
}

}  // extern "C"
