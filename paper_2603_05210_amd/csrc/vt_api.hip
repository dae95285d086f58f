// The device-facing part of the C ABI of include/vt.h: the launch sequences of the entry points
// (their pure host argument checks and the per-call plan are in vt_plan.cpp).  Every step of the
// method runs in the kernels; the host only reads back error flags and finished results.
#include "vt.h"

#include <hip/hip_runtime.h>
#include <string.h>

#include <atomic>

#include "vt_internal.h"
#include "vt_gemv_common.h"
#include "vt_select.h"
#include "vt_coverage.h"

namespace vt {

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The launch sequence of one draft step on validated arguments; `ws` is a workspace whose header
// has been initialised (arrival counter zero).
// What the variants of the step add to the plain call.
struct HeadExtras {
    int fmt = 0;                    // storage format of W_sub (0: bf16)
    const void* scales = nullptr;   // compressed forms only
    const uint16_t* gamma = nullptr;  // fused RMSNorm ahead of the head: weight [H], or NULL
    float eps = 0.0f;
    const float* parent = nullptr;  // per-row cumulative log-probability added to the outputs, or NULL
    uint16_t* h_out = nullptr;      // test hook: normalised hidden state
};

static vt_status run_head(const uint16_t* h, int64_t rows, int64_t H, const uint16_t* W_sub, const int32_t* d2t,
                          int64_t V_draft, int k, int32_t* out_target_ids, float* out_logprobs, char* ws,
                          hipStream_t s, float* logits_out, float* lse_out, const HeadExtras& ex = HeadExtras())
{
    const int fmt = ex.fmt;
    Plan p;
    if (!(fmt == 0 ? make_plan(rows, H, V_draft, k, p) : make_plan_q(fmt, rows, H, V_draft, k, p)))
        return VT_ERR_SHAPE;
    HeadArgs a;
    a.h = h;
    a.W = W_sub;
    a.scales = ex.scales;
    a.gamma = ex.gamma;
    a.eps = ex.eps;
    a.parent = ex.parent;
    a.h_out = ex.h_out;
    if (ex.gamma != nullptr && !p.one_row) {
        // only the one-row kernel normalises on the way in: the other shapes get a small kernel of
        // their own, which leaves the normalised state behind the partial results in the workspace
        uint16_t* hn = ex.h_out != nullptr ? ex.h_out : reinterpret_cast<uint16_t*>(ws + p.total_bytes);
        if (launch_rmsnorm(h, ex.gamma, ex.eps, (int)rows, (int)H, hn, s) != hipSuccess)
            return VT_ERR_DEVICE;
        a.h = hn;
        a.gamma = nullptr;
    }
    a.d2t = d2t;
    a.out_ids = out_target_ids;
    a.out_logp = out_logprobs;
    a.arrive = reinterpret_cast<unsigned int*>(ws);
    a.part_val = reinterpret_cast<float*>(ws + p.off_val);
    a.part_idx = reinterpret_cast<int32_t*>(ws + p.off_idx);
    a.part_stat = reinterpret_cast<float2*>(ws + p.off_stat);
    a.logits_out = logits_out;
    a.lse_out = lse_out;
    const hipError_t e = fmt != 0 ? launch_gemv_q(fmt, p, a, s) : (p.regime == 0) ? launch_gemv(p, a, s) : launch_gemm(p, a, s);
    if (e != hipSuccess)
        return VT_ERR_DEVICE;
    if (!(p.regime == 0 && p.fused) && launch_merge(p, a, s) != hipSuccess)
        return VT_ERR_DEVICE;
    return VT_OK;
}

// Range and distinctness of a draft vocabulary's ids, checked on the device; waits for the
// answer.  Allocates and frees a V-bit bitmap (set-up path).
static vt_status check_ids_on_device(const int32_t* token_ids, int64_t V_draft, int64_t V, hipStream_t s)
{
    const size_t words = (size_t)(V + 31) / 32;
    uint32_t* bits = nullptr;  // bitmap words, then one int of error bits
    if (hipMalloc(reinterpret_cast<void**>(&bits), (words + 1) * sizeof(uint32_t)) != hipSuccess)
        return VT_ERR_DEVICE;
    int err = 0;
    bool ok = hipMemsetAsync(bits, 0, (words + 1) * sizeof(uint32_t), s) == hipSuccess;
    ok = ok && launch_check_ids(token_ids, (int)V_draft, (int)V, bits, reinterpret_cast<int*>(bits + words), s) == hipSuccess;
    ok = ok && hipMemcpyAsync(&err, bits + words, sizeof(int), hipMemcpyDeviceToHost, s) == hipSuccess;
    ok = ok && hipStreamSynchronize(s) == hipSuccess;
    (void)hipFree(bits);
    if (!ok)
        return VT_ERR_DEVICE;
    if (err & 1)
        return VT_ERR_ID_RANGE;
    if (err & 2)
        return VT_ERR_ID_DUP;
    return VT_OK;
}

// ---- device-resident scratch for callers that cannot allocate ----
// One array per GPU (each device that loads the library holds its own copy at its own address,
// until the process ends).  In host code the array's name is only a handle for the symbol
// lookup; the device address obtained once per device is what every launch uses.  Its header
// (the arrival counter) is zero at load time and every call leaves it zero.
static __device__ __align__(256) unsigned char scratch[VT_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::atomic<char*> g_scratch_ptr[kMaxDevices];

// Device address of the current device's scratch array; on the first use on a device also
// enqueues a clear of its header on `s`.
static vt_status static_scratch(hipStream_t s, char** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return VT_ERR_DEVICE;
    char* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        void* addr = nullptr;
        if (hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)) != hipSuccess || addr == nullptr)
            return VT_ERR_DEVICE;
        p = static_cast<char*>(addr);
        if (launch_clear_words(reinterpret_cast<uint32_t*>(p), (int)(kWorkspaceHeader / sizeof(uint32_t)), s) != hipSuccess)
            return VT_ERR_DEVICE;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return VT_OK;
}

}  // namespace vt

using namespace vt;

extern "C" {

vt_status vt_build_subset(const uint16_t* full_W, int64_t V, int64_t H, const int32_t* token_ids, int64_t V_draft,
                          uint16_t* W_sub_out, int32_t* d2t_out, void* stream)
{
    vt_status st = vt_validate_build_subset_args(full_W, V, H, token_ids, V_draft, W_sub_out, d2t_out);
    if (st != VT_OK)
        return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = check_ids_on_device(token_ids, V_draft, V, s);
    if (st != VT_OK)
        return st;
    if (launch_gather(full_W, (int)H, token_ids, (int)V_draft, W_sub_out, d2t_out, s) != hipSuccess)
        return VT_ERR_DEVICE;
    return VT_OK;
}

vt_status vt_build_subset_q(const uint16_t* full_W, int64_t V, int64_t H, const int32_t* token_ids, int64_t V_draft,
                            int fmt, uint8_t* codes_out, void* scales_out, int32_t* d2t_out, void* stream)
{
    if (!codes_out || !scales_out)
        return VT_ERR_NULL;
    // the bf16 call's checks (pointers, ranges, alignment) with the code buffer in W_sub's place
    vt_status st = vt_validate_build_subset_args(full_W, V, H, token_ids, V_draft, codes_out, d2t_out);
    if (st != VT_OK)
        return st;
    if (vt_subset_q_code_bytes(fmt, V_draft, H) == 0)
        return VT_ERR_SHAPE;
    if (!aligned16(scales_out))
        return VT_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = check_ids_on_device(token_ids, V_draft, V, s);
    if (st != VT_OK)
        return st;
    if (launch_quant_gather(fmt, full_W, (int)H, token_ids, (int)V_draft, codes_out, scales_out, d2t_out, s) != hipSuccess)
        return VT_ERR_DEVICE;
    return VT_OK;
}

vt_status vt_draft_head_workspace_init(void* workspace, size_t workspace_bytes, void* stream)
{
    if (!workspace)
        return VT_ERR_NULL;
    if (workspace_bytes < kWorkspaceHeader)
        return VT_ERR_WORKSPACE;
    if (!aligned16(workspace))
        return VT_ERR_ALIGN;
    // a small fill kernel, not a memset node: the call may be recorded into a graph
    if (launch_clear_words(static_cast<uint32_t*>(workspace), (int)(kWorkspaceHeader / sizeof(uint32_t)),
                           static_cast<hipStream_t>(stream)) != hipSuccess)
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
    return run_head(h, rows, H, W_sub, d2t, V_draft, k, out_target_ids, out_logprobs, static_cast<char*>(workspace),
                    static_cast<hipStream_t>(stream), logits_out, lse_out);
}

vt_status vt_feature_fusion(const uint16_t* x, int64_t rows, int64_t d_in, const uint16_t* W_fc, int64_t d_out,
                            uint16_t* g_out, void* stream)
{
    if (!x || !W_fc || !g_out)
        return VT_ERR_NULL;
    const int64_t lim = (int64_t)1 << 31;
    if (rows < 1 || d_in < 8 || d_out < 1 || (d_in % 8) != 0 || rows >= lim || d_in >= lim || d_out >= lim ||
        d_out * (d_in / 8) >= lim || rows * (d_in / 8) >= lim)
        return VT_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(W_fc) || (reinterpret_cast<uintptr_t>(g_out) & 7u))
        return VT_ERR_ALIGN;
    if (launch_feature_fusion(x, (int)rows, (int)d_in, W_fc, (int)d_out, g_out, static_cast<hipStream_t>(stream)) != hipSuccess)
        return VT_ERR_DEVICE;
    return VT_OK;
}

size_t vt_draft_head_fused_workspace_bytes(int64_t rows, int64_t H, int64_t V_draft, int k)
{
    const size_t head = vt_draft_head_workspace_bytes(rows, H, V_draft, k);
    if (head == 0)
        return 0;
    return head + ((size_t)rows * (size_t)H * 2 + 255) / 256 * 256;  // room for the normalised state
}

vt_status vt_draft_head_fused_debug(const uint16_t* g, const uint16_t* gamma, float eps, const float* parent_scores,
                                    int64_t rows, int64_t H, const uint16_t* W_sub, const int32_t* d2t, int64_t V_draft,
                                    int k, int32_t* out_target_ids, float* out_scores, void* workspace,
                                    size_t workspace_bytes, void* stream, float* logits_out, float* lse_out,
                                    uint16_t* h_out)
{
    if (!gamma)
        return VT_ERR_NULL;
    if (!(eps >= 0.0f))
        return VT_ERR_SHAPE;
    vt_status st = vt_validate_draft_head_args(g, rows, H, W_sub, d2t, V_draft, k, out_target_ids, out_scores, workspace,
                                               workspace_bytes);
    if (st != VT_OK)
        return st;
    if (workspace_bytes < vt_draft_head_fused_workspace_bytes(rows, H, V_draft, k))
        return VT_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(gamma) & 7u) || (reinterpret_cast<uintptr_t>(parent_scores) & 3u) ||
        (reinterpret_cast<uintptr_t>(h_out) & 7u))
        return VT_ERR_ALIGN;
    HeadExtras ex;
    ex.gamma = gamma;
    ex.eps = eps;
    ex.parent = parent_scores;
    ex.h_out = h_out;
    return run_head(g, rows, H, W_sub, d2t, V_draft, k, out_target_ids, out_scores, static_cast<char*>(workspace),
                    static_cast<hipStream_t>(stream), logits_out, lse_out, ex);
}

vt_status vt_draft_head_fused(const uint16_t* g, const uint16_t* gamma, float eps, const float* parent_scores, int64_t rows,
                              int64_t H, const uint16_t* W_sub, const int32_t* d2t, int64_t V_draft, int k,
                              int32_t* out_target_ids, float* out_scores, void* workspace, size_t workspace_bytes,
                              void* stream)
{
    return vt_draft_head_fused_debug(g, gamma, eps, parent_scores, rows, H, W_sub, d2t, V_draft, k, out_target_ids, out_scores,
                                     workspace, workspace_bytes, stream, nullptr, nullptr, nullptr);
}

vt_status vt_draft_head_q_debug(const uint16_t* h, int64_t rows, int64_t H, const uint8_t* codes, const void* scales,
                                int fmt, const int32_t* d2t, int64_t V_draft, int k, int32_t* out_target_ids,
                                float* out_logprobs, void* workspace, size_t workspace_bytes, void* stream,
                                float* logits_out, float* lse_out)
{
    if (!h || !codes || !scales || !d2t || !out_target_ids || !out_logprobs)
        return VT_ERR_NULL;
    if (k < 1 || k > 16 || k > V_draft)
        return VT_ERR_K;
    const size_t need = vt_draft_head_q_workspace_bytes(fmt, rows, H, V_draft, k);
    if (need == 0)
        return VT_ERR_SHAPE;
    if (!workspace || workspace_bytes < need)
        return VT_ERR_WORKSPACE;
    if (!aligned16(h) || !aligned16(codes) || !aligned16(scales) || !aligned16(workspace) ||
        (reinterpret_cast<uintptr_t>(d2t) & 3u) || (reinterpret_cast<uintptr_t>(out_target_ids) & 3u) ||
        (reinterpret_cast<uintptr_t>(out_logprobs) & 3u))
        return VT_ERR_ALIGN;
    HeadExtras ex;
    ex.fmt = fmt;
    ex.scales = scales;
    return run_head(h, rows, H, reinterpret_cast<const uint16_t*>(codes), d2t, V_draft, k, out_target_ids, out_logprobs,
                    static_cast<char*>(workspace), static_cast<hipStream_t>(stream), logits_out, lse_out, ex);
}

vt_status vt_draft_head_q(const uint16_t* h, int64_t rows, int64_t H, const uint8_t* codes, const void* scales, int fmt,
                          const int32_t* d2t, int64_t V_draft, int k, int32_t* out_target_ids, float* out_logprobs,
                          void* workspace, size_t workspace_bytes, void* stream)
{
    return vt_draft_head_q_debug(h, rows, H, codes, scales, fmt, d2t, V_draft, k, out_target_ids, out_logprobs, workspace,
                                 workspace_bytes, stream, nullptr, nullptr);
}

vt_status vt_draft_head_static(const uint16_t* h, int64_t rows, int64_t H, const uint16_t* W_sub, const int32_t* d2t,
                               int64_t V_draft, int k, int32_t* out_target_ids, float* out_logprobs, void* stream)
{
    // the same argument checks, against the fixed capacity instead of a caller's buffer
    const size_t need = vt_draft_head_workspace_bytes(rows, H, V_draft, k);
    vt_status st = vt_validate_draft_head_args(h, rows, H, W_sub, d2t, V_draft, k, out_target_ids, out_logprobs,
                                               reinterpret_cast<const void*>(uintptr_t{256}), need);
    if (st != VT_OK)
        return st;
    if (need > (size_t)VT_STATIC_SCRATCH_BYTES)
        return VT_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = nullptr;
    st = static_scratch(s, &ws);
    if (st != VT_OK)
        return st;
    return run_head(h, rows, H, W_sub, d2t, V_draft, k, out_target_ids, out_logprobs, ws, s, nullptr, nullptr);
}

vt_status vt_draft_head(const uint16_t* h, int64_t rows, int64_t H, const uint16_t* W_sub, const int32_t* d2t,
                        int64_t V_draft, int k, int32_t* out_target_ids, float* out_logprobs, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    return vt_draft_head_debug(h, rows, H, W_sub, d2t, V_draft, k, out_target_ids, out_logprobs, workspace,
                               workspace_bytes, stream, nullptr, nullptr);
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
    unsigned long long counters[6] = {0, 0, 0, 0, 0, 0};  // three counts, a pad word, the two ratios (double bits)
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
    static_assert(sizeof(double) == sizeof(unsigned long long), "ratios travel as 64-bit words");
    memcpy(&result->freq_coverage, &counters[4], sizeof(double));
    memcpy(&result->unique_coverage, &counters[5], sizeof(double));
    return VT_OK;
}

}  // extern "C"
