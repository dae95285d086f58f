/*
 * vt.h -- C ABI of the trimmed-vocabulary draft LM head for AMD MI355X (gfx950).
 *
 * The paper (Section 2.1) replaces the draft model's vocabulary V (|V| = V tokens) by a
 * subset V_d of k = |V_d| tokens; only the language-modelling head depends on that size
 * (Section 2.3: a linear projection from hidden size d to k logits, 2*d*k FLOPs per row).
 * This library is that head:
 *
 *   vt_build_subset   once per draft vocabulary: gathers the rows of the full unembedding
 *                     matrix that belong to V_d into a compact W_sub[V_draft,H] and writes
 *                     the draft-to-target index buffer d2t (Section 1, EAGLE-3's buffers).
 *   vt_draft_head     once per draft step: logits = h . W_sub^T, softmax statistics over V_d,
 *                     the k best draft tokens per row, mapped through d2t to ids in V, with
 *                     their log-probabilities.
 *
 * Conventions
 *   - Every pointer documented "device" is a HIP device pointer on the current device;
 *     "host" pointers are ordinary memory.  The library never frees or keeps a caller's
 *     pointer.  Inputs are never modified; outputs are fully overwritten on success.
 *   - bf16 values travel as uint16_t bit patterns.  Matrices are row-major and contiguous.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Errors are return codes only.  Argument errors are detected on the host before any
 *     launch: on a non-VT_OK return nothing was launched and no output was touched
 *     (exception: VT_ERR_DEVICE may be returned after a partial launch sequence).
 *   - Preconditions: H % 8 == 0 (rows are moved in 128-bit pieces), 1 <= k <= min(V_draft,
 *     VT_MAX_K), rows >= 1, all sizes below 2^31, device pointers 16-byte aligned.
 *   - Non-finite inputs give undefined results.
 */
#ifndef VT_H_
#define VT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VT_MAX_K 64

typedef enum {
    VT_OK = 0,
    VT_ERR_NULL = 1,      /* a required pointer is NULL                                  */
    VT_ERR_SHAPE = 2,     /* rows, H, V or V_draft out of range, or H % 8 != 0            */
    VT_ERR_K = 3,         /* k < 1, k > V_draft or k > VT_MAX_K                           */
    VT_ERR_ID_RANGE = 4,  /* a token id is outside [0, V)                                 */
    VT_ERR_ID_DUP = 5,    /* a token id occurs twice (V_d is a set)                       */
    VT_ERR_WORKSPACE = 6, /* workspace missing or smaller than the size query's answer    */
    VT_ERR_ALIGN = 7,     /* a device pointer is not 16-byte aligned                      */
    VT_ERR_DEVICE = 8     /* the HIP runtime reported an error                            */
} vt_status;

/* Library version: major * 10000 + minor * 100 + patch. */
int vt_version(void);

/* Static, human-readable name of a status code. */
const char *vt_status_str(vt_status s);

/*
 * Section 2.1 / Section 1 (d2t buffer).  W_sub_out[j,:] = full_W[token_ids[j],:] bit for bit,
 * d2t_out[j] = token_ids[j], for j in [0, V_draft).  The order of token_ids defines the draft
 * indices (pass them ascending to make "lower draft index" mean "lower target id").
 *
 *   full_W     device, [V,H] bf16          token_ids  device, [V_draft] int32
 *   W_sub_out  device, [V_draft,H] bf16    d2t_out    device, [V_draft] int32
 *
 * The ids are checked on the device first (range and distinctness); the call waits for that
 * check, so VT_ERR_ID_RANGE / VT_ERR_ID_DUP are returned with the outputs untouched.  The
 * gather itself is then enqueued on `stream` and the call returns without waiting for it.
 * Allocates and frees a V-bit scratch bitmap internally (this is a set-up call, not a
 * per-step call).
 */
vt_status vt_build_subset(const uint16_t *full_W, int64_t V, int64_t H, const int32_t *token_ids,
                          int64_t V_draft, uint16_t *W_sub_out, int32_t *d2t_out, void *stream);

/* Host-side check of a host copy of the id list: VT_OK, VT_ERR_NULL, VT_ERR_SHAPE,
 * VT_ERR_ID_RANGE or VT_ERR_ID_DUP.  Touches no device. */
vt_status vt_check_token_ids_host(const int32_t *token_ids_host, int64_t V_draft, int64_t V);

/* Pure host argument checks, exactly the ones the two entry points run before launching. */
vt_status vt_validate_build_subset_args(const void *full_W, int64_t V, int64_t H, const void *token_ids,
                                        int64_t V_draft, const void *W_sub_out, const void *d2t_out);
vt_status vt_validate_draft_head_args(const void *h, int64_t rows, int64_t H, const void *W_sub,
                                      const void *d2t, int64_t V_draft, int k, const void *out_target_ids,
                                      const void *out_logprobs, const void *workspace, size_t workspace_bytes);

/* Bytes of device workspace vt_draft_head needs for this shape (0 on invalid arguments).
 * A pure function of its arguments: it does not depend on the device. */
size_t vt_draft_head_workspace_bytes(int64_t rows, int64_t H, int64_t V_draft, int k);

/*
 * One-time preparation of a workspace buffer for vt_draft_head: zeroes its header of
 * VT_WORKSPACE_HEADER_BYTES bytes, which holds the arrival counters of the single-launch merge of
 * the one- and two-row steps (Section 2.3's head is one kernel there; the last workgroup to
 * finish merges the partial results).  Every call leaves the counters at zero again, so one
 * initialisation serves any number of calls of any shapes; initialise again only if something
 * else has written to the buffer.  Enqueues one small kernel on `stream` (safe to record into a
 * graph); VT_ERR_NULL / VT_ERR_WORKSPACE (fewer than VT_WORKSPACE_HEADER_BYTES bytes) /
 * VT_ERR_ALIGN / VT_ERR_DEVICE.  Every size vt_draft_head_workspace_bytes returns includes the
 * header.
 */
#define VT_WORKSPACE_HEADER_BYTES 8192
vt_status vt_draft_head_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/* Which kernel family serves this shape: 0 = streaming kernels that read W_sub once per group
 * of 16 rows (memory bound: rows <= 16, and a few dozen rows at H = 2048 / 4096 and k <= 16),
 * 1 = bf16 MFMA thin GEMM; -1 on invalid arguments. */
int vt_draft_head_regime(int64_t rows, int64_t H, int64_t V_draft, int k);

/*
 * One draft step (Section 2.3's head over V_d, then the candidate proposal of Section 1):
 *   z[r,j]   = sum_i h[r,i] * W_sub[j,i]             bf16 inputs, fp32 accumulation
 *   lse[r]   = log sum_j exp(z[r,j])                  over the V_draft draft tokens only
 *   the k largest z[r,.] per row, best first, equal logits ordered by lower draft index j
 *   out_target_ids[r,p] = d2t[j_p],  out_logprobs[r,p] = z[r,j_p] - lse[r]
 *
 *   h               device, [rows,H] bf16        W_sub  device, [V_draft,H] bf16
 *   d2t             device, [V_draft] int32
 *   out_target_ids  device, [rows,k] int32       out_logprobs  device, [rows,k] fp32
 *   workspace       device, >= vt_draft_head_workspace_bytes(...) bytes, 16-byte aligned,
 *                   initialised once by vt_draft_head_workspace_init; contents are clobbered
 *
 * Asynchronous on `stream`: no allocation, no synchronisation, no host read.  Calls that may
 * overlap in time (different streams) must not share a workspace: it holds the call's partial
 * results and the arrival counter of its single-launch merge.  Calls on one stream run in order
 * and may share one.  The logits are never written to memory.  The first call of a kernel family
 * in a process may raise that kernel's dynamic shared-memory limit (a driver call, not a stream
 * operation): before capturing a call into a HIP graph, run it once outside the capture.
 */
vt_status vt_draft_head(const uint16_t *h, int64_t rows, int64_t H, const uint16_t *W_sub,
                        const int32_t *d2t, int64_t V_draft, int k, int32_t *out_target_ids,
                        float *out_logprobs, void *workspace, size_t workspace_bytes, void *stream);

/*
 * vt_draft_head for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments,
 * same kernels and same results as vt_draft_head, but the partial results and the arrival
 * counter live in a device-resident array of VT_STATIC_SCRATCH_BYTES bytes that is part of the
 * library image (every GPU the library runs on holds one copy until the process ends).  The call
 * allocates and frees nothing and never synchronises.
 *   - VT_ERR_WORKSPACE when vt_draft_head_workspace_bytes(rows, H, V_draft, k) exceeds
 *     VT_STATIC_SCRATCH_BYTES (nothing is launched); every other code as vt_draft_head.
 *   - All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU
 *     (different streams, different host threads) race and give undefined results; calls on one
 *     stream run in order and are safe.  The array keeps the previous call's partial results;
 *     every call overwrites what it reads and leaves the arrival counter at zero.
 */
#define VT_STATIC_SCRATCH_BYTES (40u << 20)
vt_status vt_draft_head_static(const uint16_t *h, int64_t rows, int64_t H, const uint16_t *W_sub,
                               const int32_t *d2t, int64_t V_draft, int k, int32_t *out_target_ids,
                               float *out_logprobs, void *stream);

/*
 * Test hook, same computation through the same kernels, which additionally store
 *   logits_out  device, [rows,V_draft] fp32 (may be NULL)
 *   lse_out     device, [rows] fp32         (may be NULL)
 */
vt_status vt_draft_head_debug(const uint16_t *h, int64_t rows, int64_t H, const uint16_t *W_sub,
                              const int32_t *d2t, int64_t V_draft, int k, int32_t *out_target_ids,
                              float *out_logprobs, void *workspace, size_t workspace_bytes, void *stream,
                              float *logits_out, float *lse_out);

/*
 * The feature-fusion layer of the draft model (Section 2.3, component 1; Table 1's "Feature fusion"
 * row, 2*3d*d FLOPs per row): g[r,j] = sum_i x[r,i] * W_fc[j,i], bf16 in, fp32 accumulation, one
 * rounding to bf16 (nearest even).
 *   x      device, [rows,d_in] bf16   (d_in = 3d: the three concatenated target features)
 *   W_fc   device, [d_out,d_in] bf16
 *   g_out  device, [rows,d_out] bf16, 8-byte aligned
 * d_in % 8 == 0.  Asynchronous on `stream`, allocates nothing.
 */
vt_status vt_feature_fusion(const uint16_t *x, int64_t rows, int64_t d_in, const uint16_t *W_fc, int64_t d_out,
                            uint16_t *g_out, void *stream);

/*
 * The draft step with its neighbours fused in: the hidden state arrives before the final
 * normalisation and leaves as path scores of a draft tree.
 *   h[r,i]      = bf16( g[r,i] * rsqrt(mean_i g[r,i]^2 + eps) * gamma[i] )   (root-mean-square norm; the
 *                 paper names no normalisation: this is the LLaMA family's, in fp32, one rounding)
 *   ids, logp   = vt_draft_head(h, ...)
 *   out_scores[r,p] = logp[r,p] + parent_scores[r]   (cumulative log-probability of the path that the
 *                 proposed token extends; parent_scores may be NULL: plain log-probabilities)
 * For one row the normalisation happens while the hidden state is staged inside the step's single
 * kernel (it never returns to memory); other row counts run a small kernel first.
 *   g              device, [rows,H] bf16      gamma  device, [H] bf16, 8-byte aligned
 *   parent_scores  device, [rows] fp32, or NULL
 *   workspace      device, >= vt_draft_head_fused_workspace_bytes(...), initialised once as for vt_draft_head
 * Everything else as vt_draft_head.  The _debug form also stores logits_out[rows,V_draft], lse_out[rows]
 * and the normalised state h_out[rows,H] (each may be NULL).
 */
size_t vt_draft_head_fused_workspace_bytes(int64_t rows, int64_t H, int64_t V_draft, int k);
vt_status vt_draft_head_fused(const uint16_t *g, const uint16_t *gamma, float eps, const float *parent_scores,
                              int64_t rows, int64_t H, const uint16_t *W_sub, const int32_t *d2t, int64_t V_draft,
                              int k, int32_t *out_target_ids, float *out_scores, void *workspace,
                              size_t workspace_bytes, void *stream);
vt_status vt_draft_head_fused_debug(const uint16_t *g, const uint16_t *gamma, float eps, const float *parent_scores,
                                    int64_t rows, int64_t H, const uint16_t *W_sub, const int32_t *d2t, int64_t V_draft,
                                    int k, int32_t *out_target_ids, float *out_scores, void *workspace,
                                    size_t workspace_bytes, void *stream, float *logits_out, float *lse_out,
                                    uint16_t *h_out);

/*
 * Compressed W_sub for the one-row draft step.  Sections 1 and 2.3: the head dominates the
 * draft's latency and costs 2*d*k per token; at one row that is the bytes of W_sub, which
 * trimming cuts through k and a narrower storage format cuts per weight.  Two formats:
 *   VT_Q_FP8_E4M3  one byte per weight: OCP E4M3 (bias 7, no infinities, largest value 448),
 *                  one fp32 scale per row: scale_j = max_i |W[j,i]| / 448 (1 for an all-zero row),
 *                  code = E4M3(W[j,i] / scale_j), nearest, ties to even, saturating.  H % 16 == 0.
 *   VT_Q_MXFP4     OCP microscaling: E2M1 codes (0, 0.5, 1, 1.5, 2, 3, 4, 6 and their negatives),
 *                  two per byte with the even element in the low nibble, and one exponent byte
 *                  (power of two, bias 127) per 32 consecutive weights of a row:
 *                  exponent = floor(log2(max |w| of the block)) - 2 (byte 127 for an all-zero
 *                  block), code = E2M1(w / 2^exponent).  H % 32 == 0.
 * vt_build_subset_q is vt_build_subset with the gathered rows stored in one of these formats:
 *   codes_out   device, vt_subset_q_code_bytes(...) bytes: [V_draft][H] (FP8) or [V_draft][H/2] (MXFP4)
 *   scales_out  device, vt_subset_q_scale_bytes(...) bytes: float[V_draft] (FP8) or
 *               uint8[V_draft][H/32] (MXFP4); both 16-byte aligned
 * Same id checks, waiting and error codes as vt_build_subset; VT_ERR_SHAPE for an unknown format.
 */
#define VT_Q_FP8_E4M3 1
#define VT_Q_MXFP4 2
size_t vt_subset_q_code_bytes(int fmt, int64_t V_draft, int64_t H);   /* 0 on invalid arguments */
size_t vt_subset_q_scale_bytes(int fmt, int64_t V_draft, int64_t H);
vt_status vt_build_subset_q(const uint16_t *full_W, int64_t V, int64_t H, const int32_t *token_ids,
                            int64_t V_draft, int fmt, uint8_t *codes_out, void *scales_out, int32_t *d2t_out,
                            void *stream);

/*
 * One draft step over a compressed W_sub: vt_draft_head's computation with every weight taken
 * as its code's value times its scale (bf16 hidden state, exact products, fp32 accumulation; the
 * scale multiplies the fp32 sum of its row or 32-weight block).  Served shapes (the memory-bound
 * regime the compression is for), k <= 16 throughout: rows == 1 with V_draft <= 262144 and H in
 * {1024, 2048, 4096} (FP8) or {2048, 4096} (MXFP4); 2 <= rows <= 32 (up to 64 when V_draft <= 16384)
 * with H in {2048, 4096} (FP8) or H == 4096 (MXFP4); anything else is VT_ERR_SHAPE (VT_ERR_K for k).  Pointers,
 * workspace rules (vt_draft_head_workspace_init once), asynchrony and outputs as vt_draft_head;
 * the _debug form also stores logits_out[rows][V_draft] and lse_out[rows] (either may be NULL).
 */
size_t vt_draft_head_q_workspace_bytes(int fmt, int64_t rows, int64_t H, int64_t V_draft, int k);
vt_status vt_draft_head_q(const uint16_t *h, int64_t rows, int64_t H, const uint8_t *codes, const void *scales,
                          int fmt, const int32_t *d2t, int64_t V_draft, int k, int32_t *out_target_ids,
                          float *out_logprobs, void *workspace, size_t workspace_bytes, void *stream);
vt_status vt_draft_head_q_debug(const uint16_t *h, int64_t rows, int64_t H, const uint8_t *codes, const void *scales,
                                int fmt, const int32_t *d2t, int64_t V_draft, int k, int32_t *out_target_ids,
                                float *out_logprobs, void *workspace, size_t workspace_bytes, void *stream,
                                float *logits_out, float *lse_out);

/*
 * Draft-vocabulary size selection (Section 2, Eq. 1-5).  From a stream of token ids (the
 * assistant-span tokens of a training corpus, Section 2.2) the call computes, on the device:
 *   f(v)   the frequency of every token id (freq_out),
 *   the frequency ranking, most frequent first, equal frequencies by lower id (rank_ids_out:
 *          its first k entries are the paper's top-k, Section 2.1),
 *   C(k)   = sum of the k largest frequencies / n_tokens                              (Eq. 2)
 *   R(k)   = 1 - (F_fixed + 2 d k) / (F_fixed + 2 d V)                                (Eq. 3)
 *   U(k)   = alpha C(k) + (1 - alpha) R(k)                                            (Eq. 4)
 *   U~(k)  = U(k) if C(k) >= c_min, else -1                                           (Eq. 5)
 *   k*     = the k in [k_min, k_max] with the largest U~(k), the smallest such k      (Eq. 1)
 * and writes the k* selected ids in ascending order to token_ids_out[0..k*), the form
 * vt_build_subset takes.  The paper searches k with 100 TPE samples (Section 2.5); this call
 * evaluates every k of the range, which is the maximum that search approximates.  All
 * floating-point work is IEEE double with one rounding per operation in the order written
 * above (C = prefix/n; R = 1 - (F + (2d)k) / (F + (2d)V); U = alpha*C + (1-alpha)*R).
 *
 *   tokens          device, int32[n_tokens], 16-byte aligned, ids in [0, V)
 *   n_tokens        1 <= n_tokens < 2^32
 *   V               1 <= V < 2^27
 *   d, F_fixed      d >= 1, F_fixed >= 0 (Table 1's fixed components)
 *   alpha, c_min    0 <= alpha <= 1, 0 <= c_min <= 1
 *   k_min, k_max    1 <= k_min <= k_max <= V
 *   freq_out        device, uint32[V]
 *   rank_ids_out    device, int32[V]
 *   token_ids_out   device, int32[V] (capacity; the first k* entries are written)
 *   result          host; filled on VT_OK
 *   workspace       device, >= vt_select_vocab_workspace_bytes(V) bytes, 16-byte aligned
 * The call enqueues its kernels on `stream`, waits for them once and then fills *result.
 * VT_ERR_ID_RANGE: some token id lies outside [0, V) (outputs are then unspecified).
 * If no k of the range meets the coverage constraint, result->feasible is 0 and k* = k_min.
 */
typedef struct {
    int64_t k_star;
    int32_t feasible;
    double C, R, U;      /* Eq. 2, 3, 4 at k* (U is the unpenalised utility) */
    uint64_t n_tokens;   /* sum of all frequencies */
} vt_selection;

size_t vt_select_vocab_workspace_bytes(int64_t V);

vt_status vt_validate_select_vocab_args(const void *tokens, int64_t n_tokens, int64_t V, int64_t d, double F_fixed,
                                        double alpha, double c_min, int64_t k_min, int64_t k_max,
                                        const void *freq_out, const void *rank_ids_out, const void *token_ids_out,
                                        const void *result, const void *workspace, size_t workspace_bytes);

vt_status vt_select_vocab(const int32_t *tokens, int64_t n_tokens, int64_t V, int64_t d, double F_fixed,
                          double alpha, double c_min, int64_t k_min, int64_t k_max, uint32_t *freq_out,
                          int32_t *rank_ids_out, int32_t *token_ids_out, vt_selection *result, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * Target-to-draft index buffer (Section 1: the t2d / d2t buffers of a draft with a reduced
 * vocabulary).  t2d_out[v] = j where d2t[j] = v, and -1 for every target id outside V_d.
 *
 *   d2t        device, int32[V_draft], distinct ids in [0, V)  (vt_build_subset's d2t_out)
 *   t2d_out    device, int32[V]
 *   workspace  device, >= vt_coverage_workspace_bytes(V) bytes, 16-byte aligned
 * The call waits for its kernels once so that VT_ERR_ID_RANGE / VT_ERR_ID_DUP can be
 * returned (t2d_out is then unspecified).
 */
vt_status vt_build_t2d(const int32_t *d2t, int64_t V_draft, int64_t V, int32_t *t2d_out, void *workspace,
                       size_t workspace_bytes, void *stream);

/*
 * Coverage of a draft vocabulary on a stream of token ids (Section 2.2, Eq. 2 evaluated on the
 * stream; Section 5.1, Table 4): the share of token occurrences whose token has a draft index
 * (the table's frequency-weighted column) and the share of distinct tokens of the stream that
 * have one (its unique-token column).
 * Counts of several streams add up (Table 4's combined row).  Optionally writes the stream
 * mapped through t2d (-1 where the target token has no draft index), the remapping that masks
 * out-of-vocabulary targets.
 *
 *   tokens          device, int32[n_tokens], ids in [0, V); 1 <= n_tokens
 *   t2d             device, int32[V]  (vt_build_t2d)
 *   draft_ids_out   device, int32[n_tokens], or NULL
 *   result          host; filled on VT_OK
 *   workspace       device, >= vt_coverage_workspace_bytes(V) bytes, 16-byte aligned
 * The call waits for its kernels once.  VT_ERR_ID_RANGE: a token id outside [0, V).
 */
typedef struct {
    uint64_t n_tokens;          /* occurrences                                   */
    uint64_t n_covered;         /* occurrences whose token is in V_d             */
    uint64_t n_unique;          /* distinct tokens in the stream                 */
    uint64_t n_unique_covered;  /* distinct tokens in the stream that are in V_d */
    double freq_coverage;       /* n_covered / n_tokens                          */
    double unique_coverage;     /* n_unique_covered / n_unique                   */
} vt_coverage_result;

size_t vt_coverage_workspace_bytes(int64_t V);

vt_status vt_coverage(const int32_t *tokens, int64_t n_tokens, const int32_t *t2d, int64_t V,
                      int32_t *draft_ids_out, vt_coverage_result *result, void *workspace,
                      size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* VT_H_ */
