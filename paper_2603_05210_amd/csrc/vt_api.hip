// The C ABI of include/vt.h: host-side argument checks, the per-call plan (which kernel
// family, how many partial results, where they live in the caller's workspace) and the launch
// sequences.  No computation of the method happens on the host.
#include "vt.h"

#include <hip/hip_runtime.h>

#include <mutex>
#include <vector>

#include "vt_internal.h"
#include "vt_select.h"
#include "vt_coverage.h"

namespace vt {

static int next_pow2(int x)
{
    int p = 1;
    while (p < x)
        p <<= 1;
    return p;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

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
    if (streaming) {
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
    p.off_val = 0;
    p.off_idx = align_up(p.off_val + n * p.KP * sizeof(float), 256);
    p.off_stat = align_up(p.off_idx + n * p.KP * sizeof(int32_t), 256);
    p.total_bytes = align_up(p.off_stat + n * sizeof(float2), 256);
    return true;
}

// ---- optional timing of the projection kernel ----
struct Timing {
    std::mutex mu;
    bool on = false;
    std::vector<hipEvent_t> ev;  // pairs
    int used = 0;                // events used
};
static Timing g_timing;

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

int vt_draft_head_regime(int64_t rows, int64_t H, int64_t V_draft, int k)
{
    if (!shape_ok(rows, H, V_draft) || k < 1 || k > VT_MAX_K || k > V_draft)
        return -1;
    Plan p;
    if (!make_plan(rows, H, V_draft, k, p))
        return -1;
    return p.regime;
}

vt_status vt_build_subset(const uint16_t* full_W, int64_t V, int64_t H, const int32_t* token_ids, int64_t V_draft,
                          uint16_t* W_sub_out, int32_t* d2t_out, void* stream)
{
    vt_status st = vt_validate_build_subset_args(full_W, V, H, token_ids, V_draft, W_sub_out, d2t_out);
    if (st != VT_OK)
        return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t words = (size_t)(V + 31) / 32;
    uint32_t* scratch = nullptr;  // bitmap words, then one int of error bits
    if (hipMalloc(reinterpret_cast<void**>(&scratch), (words + 1) * sizeof(uint32_t)) != hipSuccess)
        return VT_ERR_DEVICE;
    int err = 0;
    bool ok = hipMemsetAsync(scratch, 0, (words + 1) * sizeof(uint32_t), s) == hipSuccess;
    ok = ok && launch_check_ids(token_ids, (int)V_draft, (int)V, scratch, reinterpret_cast<int*>(scratch + words), s) ==
                   hipSuccess;
    ok = ok && hipMemcpyAsync(&err, scratch + words, sizeof(int), hipMemcpyDeviceToHost, s) == hipSuccess;
    ok = ok && hipStreamSynchronize(s) == hipSuccess;
    (void)hipFree(scratch);
    if (!ok)
        return VT_ERR_DEVICE;
    if (err & 1)
        return VT_ERR_ID_RANGE;
    if (err & 2)
        return VT_ERR_ID_DUP;
    if (launch_gather(full_W, (int)H, token_ids, (int)V_draft, W_sub_out, d2t_out, s) != hipSuccess)
        return VT_ERR_DEVICE;
    return VT_OK;
}

vt_status vt_draft_head_debug(const uint16_t* h, int64_t rows, int64_t H, const uint16_t* W_sub, const int32_t* d2t,
                              int64_t V_draft, int k, int32_t* out_target_ids, float* out_logprobs, void* workspace,
                              size_t workspace_bytes, void* stream, float* logits_out, float* lse_out)
{
    vt_status st = vt_validate_draft_head_args(h, rows, H, W_sub, d2t, V_draft, k, out_target_ids, out_logprobs,
                                               workspace, workspace_bytes);
    if (st != VT_OK)
        return st;
    Plan p;
    if (!make_plan(rows, H, V_draft, k, p))
        return VT_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    HeadArgs a;
    a.h = h;
    a.W = W_sub;
    a.d2t = d2t;
    a.out_ids = out_target_ids;
    a.out_logp = out_logprobs;
    a.part_val = reinterpret_cast<float*>(ws + p.off_val);
    a.part_idx = reinterpret_cast<int32_t*>(ws + p.off_idx);
    a.part_stat = reinterpret_cast<float2*>(ws + p.off_stat);
    a.logits_out = logits_out;
    a.lse_out = lse_out;

    hipEvent_t e0 = nullptr, e1 = nullptr;
    {
        std::lock_guard<std::mutex> g(g_timing.mu);
        if (g_timing.on && g_timing.used + 2 <= 2 * VT_TIMING_MAX_EVENTS) {
            while ((int)g_timing.ev.size() < g_timing.used + 2) {
                hipEvent_t e;
                if (hipEventCreate(&e) != hipSuccess)
                    return VT_ERR_DEVICE;
                g_timing.ev.push_back(e);
            }
            e0 = g_timing.ev[g_timing.used];
            e1 = g_timing.ev[g_timing.used + 1];
            g_timing.used += 2;
        }
    }
    if (e0 && hipEventRecord(e0, s) != hipSuccess)
        return VT_ERR_DEVICE;
    hipError_t e = (p.regime == 0) ? launch_gemv(p, a, s) : launch_gemm(p, a, s);
    if (e != hipSuccess)
        return VT_ERR_DEVICE;
    if (e1 && hipEventRecord(e1, s) != hipSuccess)
        return VT_ERR_DEVICE;
    if (!(p.regime == 0 && p.fused) && launch_merge(p, a, s) != hipSuccess)
        return VT_ERR_DEVICE;
    return VT_OK;
}

vt_status vt_draft_head(const uint16_t* h, int64_t rows, int64_t H, const uint16_t* W_sub, const int32_t* d2t,
                        int64_t V_draft, int k, int32_t* out_target_ids, float* out_logprobs, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    return vt_draft_head_debug(h, rows, H, W_sub, d2t, V_draft, k, out_target_ids, out_logprobs, workspace,
                               workspace_bytes, stream, nullptr, nullptr);
}

vt_status vt_kernel_timing_enable(int on)
{
    std::lock_guard<std::mutex> g(g_timing.mu);
    g_timing.on = on != 0;
    g_timing.used = 0;
    return VT_OK;
}

vt_status vt_kernel_timing_read(int* launches, double* total_ms)
{
    if (!launches || !total_ms)
        return VT_ERR_NULL;
    std::lock_guard<std::mutex> g(g_timing.mu);
    double total = 0.0;
    const int n = g_timing.used / 2;
    for (int i = 0; i < n; ++i) {
        float ms = 0.0f;
        if (hipEventSynchronize(g_timing.ev[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_timing.ev[2 * i], g_timing.ev[2 * i + 1]) != hipSuccess)
            return VT_ERR_DEVICE;
        total += ms;
    }
    *launches = n;
    *total_ms = total;
    g_timing.used = 0;
    return VT_OK;
}

size_t vt_select_vocab_workspace_bytes(int64_t V)
{
    if (V < 1 || V >= ((int64_t)1 << 27))
        return 0;
    return vt::select_layout(V).total;
}

vt_status vt_validate_select_vocab_args(const void* tokens, int64_t n_tokens, int64_t V, int64_t d, double F_fixed,
                                        double alpha, double c_min, int64_t k_min, int64_t k_max, const void* freq_out,
                                        const void* rank_ids_out, const void* token_ids_out, const void* result,
                                        const void* workspace, size_t workspace_bytes)
{
    if (!tokens || !freq_out || !rank_ids_out || !token_ids_out || !result)
        return VT_ERR_NULL;
    if (V < 1 || V >= ((int64_t)1 << 27) || n_tokens < 1 || n_tokens >= ((int64_t)1 << 32) || d < 1 ||
        !(F_fixed >= 0.0) || !(alpha >= 0.0 && alpha <= 1.0) || !(c_min >= 0.0 && c_min <= 1.0))
        return VT_ERR_SHAPE;
    if (k_min < 1 || k_min > k_max || k_max > V)
        return VT_ERR_K;
    if (!workspace || workspace_bytes < vt_select_vocab_workspace_bytes(V))
        return VT_ERR_WORKSPACE;
    if (!aligned16(tokens) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(freq_out) & 3u) ||
        (reinterpret_cast<uintptr_t>(rank_ids_out) & 3u) || (reinterpret_cast<uintptr_t>(token_ids_out) & 3u))
        return VT_ERR_ALIGN;
    return VT_OK;
}

vt_status vt_select_vocab(const int32_t* tokens, int64_t n_tokens, int64_t V, int64_t d, double F_fixed, double alpha,
                          double c_min, int64_t k_min, int64_t k_max, uint32_t* freq_out, int32_t* rank_ids_out,
                          int32_t* token_ids_out, vt_selection* result, void* workspace, size_t workspace_bytes,
                          void* stream)
{
    const vt_status st = vt_validate_select_vocab_args(tokens, n_tokens, V, d, F_fixed, alpha, c_min, k_min, k_max,
                                                       freq_out, rank_ids_out, token_ids_out, result, workspace,
                                                       workspace_bytes);
    if (st != VT_OK)
        return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const vt::SelectLayout L = vt::select_layout(V);
    vt::SelectParams prm;
    prm.d = d;
    prm.F_fixed = F_fixed;
    prm.alpha = alpha;
    prm.c_min = c_min;
    prm.k_min = k_min;
    prm.k_max = k_max;
    char* ws = static_cast<char*>(workspace);
    if (vt::launch_select(tokens, n_tokens, (int)V, prm, freq_out, rank_ids_out, token_ids_out, ws, L, s) != hipSuccess)
        return VT_ERR_DEVICE;
    int err = 0;
    vt_selection res;
    if (hipMemcpyAsync(&err, ws + L.off_err, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(&res, ws + L.off_result, sizeof(res), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return VT_ERR_DEVICE;
    if (err != 0)
        return VT_ERR_ID_RANGE;
    *result = res;
    return VT_OK;
}

size_t vt_coverage_workspace_bytes(int64_t V)
{
    if (V < 1 || V >= ((int64_t)1 << 31))
        return 0;
    return vt::coverage_layout(V).total;
}

vt_status vt_build_t2d(const int32_t* d2t, int64_t V_draft, int64_t V, int32_t* t2d_out, void* workspace,
                       size_t workspace_bytes, void* stream)
{
    if (!d2t || !t2d_out)
        return VT_ERR_NULL;
    if (V < 1 || V >= ((int64_t)1 << 31) || V_draft < 1 || V_draft > V)
        return VT_ERR_SHAPE;
    if (!workspace || workspace_bytes < vt_coverage_workspace_bytes(V))
        return VT_ERR_WORKSPACE;
    if (!aligned16(workspace) || (reinterpret_cast<uintptr_t>(d2t) & 3u) || (reinterpret_cast<uintptr_t>(t2d_out) & 3u))
        return VT_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const vt::CoverageLayout L = vt::coverage_layout(V);
    int* err_dev = reinterpret_cast<int*>(static_cast<char*>(workspace) + L.off_err);
    if (vt::launch_build_t2d(d2t, (int)V_draft, (int)V, t2d_out, err_dev, s) != hipSuccess)
        return VT_ERR_DEVICE;
    int err = 0;
    if (hipMemcpyAsync(&err, err_dev, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return VT_ERR_DEVICE;
    if (err & 1)
        return VT_ERR_ID_RANGE;
    if (err & 2)
        return VT_ERR_ID_DUP;
    return VT_OK;
}

vt_status vt_coverage(const int32_t* tokens, int64_t n_tokens, const int32_t* t2d, int64_t V, int32_t* draft_ids_out,
                      vt_coverage_result* result, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!tokens || !t2d || !result)
        return VT_ERR_NULL;
    if (V < 1 || V >= ((int64_t)1 << 31) || n_tokens < 1)
        return VT_ERR_SHAPE;
    if (!workspace || workspace_bytes < vt_coverage_workspace_bytes(V))
        return VT_ERR_WORKSPACE;
    if (!aligned16(workspace) || (reinterpret_cast<uintptr_t>(tokens) & 3u) || (reinterpret_cast<uintptr_t>(t2d) & 3u) ||
        (reinterpret_cast<uintptr_t>(draft_ids_out) & 3u))
        return VT_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const vt::CoverageLayout L = vt::coverage_layout(V);
    char* ws = static_cast<char*>(workspace);
    if (vt::launch_coverage(tokens, n_tokens, t2d, (int)V, draft_ids_out, ws, L, s) != hipSuccess)
        return VT_ERR_DEVICE;
    int err = 0;
    unsigned long long counters[3] = {0, 0, 0};
    if (hipMemcpyAsync(&err, ws + L.off_err, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(counters, ws + L.off_counters, sizeof(counters), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return VT_ERR_DEVICE;
    if (err != 0)
        return VT_ERR_ID_RANGE;
    result->n_tokens = (uint64_t)n_tokens;
    result->n_covered = counters[0];
    result->n_unique = counters[1];
    result->n_unique_covered = counters[2];
    result->freq_coverage = (double)counters[0] / (double)n_tokens;
    result->unique_coverage = (double)counters[2] / (double)counters[1];
    return VT_OK;
}

}  // extern "C"
