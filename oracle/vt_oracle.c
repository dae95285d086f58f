/*
 * TEST INFRASTRUCTURE -- not part of the product.
 *
 * Plain, slow, obviously-correct CPU statement of what the trimmed-vocabulary draft LM head
 * computes.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may call
 * it; the product path never does.  It shares no code, header or constant with the HIP
 * library.
 *
 * What is computed (citations are to the paper's sections / equations / tables):
 *
 *   - Section 2.1: the draft vocabulary V_d is a subset of the target vocabulary V with
 *     |V_d| = k tokens, given as a list of token ids.  The trimmed head is the full head's
 *     projection restricted to those tokens' rows, so W_sub[j,:] = W[ids[j],:].
 *   - Section 1 (the draft-to-target index buffer of EAGLE-3 style drafts): d2t[j] = ids[j],
 *     the id in V of draft token j.
 *   - Section 2.3: the LM head is a linear projection from hidden size d to vocabulary size
 *     k and costs 2*d*k FLOPs per hidden-state row: z[r,j] = sum_i h[r,i] * W_sub[j,i]
 *     (no bias term appears in that cost).  Table 1's "LM head (V=128K)" row is this count
 *     at d = 4096, k = 128 256.
 *   - Drafting proposes candidate tokens (Section 1): the k best draft tokens by logit,
 *     ordered best first, equal logits ordered by lower draft index, together with their
 *     log-probabilities under the softmax taken over V_d only; ids are reported in V.
 *
 * Precision: inputs are bf16 (carried as uint16_t bit patterns); each logit is a sequential
 * fp32 accumulation in ascending i with a separate multiply and add (build with
 * -ffp-contract=off; the product of two bf16 numbers is exact in fp32); the softmax
 * normaliser is summed in double.  A double-accumulated logit is offered only for error
 * reporting.
 *
 * Every function here is pinned by tests/test_oracle_pins.py to facts outside itself
 * (restriction and identity invariants, normalisation, brute force, exact integer
 * arithmetic, the printed Table 1 count, library routines).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static inline float widen_bf16(uint16_t u)
{
    uint32_t w = (uint32_t)u << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return f;
}

int vto_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Section 2.1 + the d2t buffer.  Returns 0, or -1 if an id is outside [0,V), or -2 if an id
 * repeats (V_d is a set).  On error the outputs are left untouched. */
int vto_build_subset(const uint16_t *W, int64_t V, int64_t H, const int32_t *ids, int64_t Vd,
                     uint16_t *W_sub, int32_t *d2t)
{
    unsigned char *seen = (unsigned char *)calloc((size_t)V, 1);
    if (!seen)
        return -3;
    for (int64_t j = 0; j < Vd; ++j) {
        if (ids[j] < 0 || ids[j] >= V) {
            free(seen);
            return -1;
        }
        if (seen[ids[j]]) {
            free(seen);
            return -2;
        }
        seen[ids[j]] = 1;
    }
    free(seen);
    for (int64_t j = 0; j < Vd; ++j) {
        memcpy(W_sub + j * H, W + (int64_t)ids[j] * H, (size_t)H * sizeof(uint16_t));
        d2t[j] = ids[j];
    }
    return 0;
}

/* Section 2.3 projection, fp32 sequential accumulation.  z is [R,Vd] row-major.
 * *flops (if given) receives the number of multiplies plus adds executed. */
void vto_logits(const uint16_t *h, int64_t R, int64_t H, const uint16_t *W_sub, int64_t Vd,
                float *z, int64_t *flops)
{
    int64_t count = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(+ : count)
    for (int64_t r = 0; r < R; ++r) {
        for (int64_t j = 0; j < Vd; ++j) {
            const uint16_t *hr = h + r * H;
            const uint16_t *wj = W_sub + j * H;
            float acc = 0.0f;
            for (int64_t i = 0; i < H; ++i) {
                float prod = widen_bf16(hr[i]) * widen_bf16(wj[i]);
                acc = acc + prod;
                count += 2;
            }
            z[r * Vd + j] = acc;
        }
    }
    if (flops)
        *flops = count;
}

/* Same projection accumulated in double: error reporting and near-tie classification only. */
void vto_logits_f64(const uint16_t *h, int64_t R, int64_t H, const uint16_t *W_sub, int64_t Vd,
                    double *z)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t r = 0; r < R; ++r) {
        for (int64_t j = 0; j < Vd; ++j) {
            const uint16_t *hr = h + r * H;
            const uint16_t *wj = W_sub + j * H;
            double acc = 0.0;
            for (int64_t i = 0; i < H; ++i)
                acc += (double)widen_bf16(hr[i]) * (double)widen_bf16(wj[i]);
            z[r * Vd + j] = acc;
        }
    }
}

/* log-sum-exp of one row over the draft vocabulary: max + log(sum exp(z - max)), sum in double. */
float vto_lse_row(const float *z, int64_t Vd)
{
    float m = z[0];
    for (int64_t j = 1; j < Vd; ++j)
        if (z[j] > m)
            m = z[j];
    double s = 0.0;
    for (int64_t j = 0; j < Vd; ++j)
        s += exp((double)(z[j] - m));
    return m + (float)log(s);
}

typedef struct {
    float z;
    int32_t j;
} entry_t;

static int by_logit_then_index(const void *a, const void *b)
{
    const entry_t *x = (const entry_t *)a, *y = (const entry_t *)b;
    if (x->z > y->z)
        return -1;
    if (x->z < y->z)
        return 1;
    return (x->j > y->j) - (x->j < y->j);
}

/* The k best draft indices of one row: full sort by (logit descending, index ascending). */
void vto_topk_row(const float *z, int64_t Vd, int k, int32_t *idx_out)
{
    entry_t *e = (entry_t *)malloc((size_t)Vd * sizeof(entry_t));
    for (int64_t j = 0; j < Vd; ++j) {
        e[j].z = z[j];
        e[j].j = (int32_t)j;
    }
    qsort(e, (size_t)Vd, sizeof(entry_t), by_logit_then_index);
    for (int p = 0; p < k; ++p)
        idx_out[p] = e[p].j;
    free(e);
}

/* Rows of logits -> outputs: softmax normaliser over V_d, k best, d2t remap (shared by the
 * bf16 head and the head over dequantised weights; z is [R,Vd]). */
static void emit_rows(const float *z, int64_t R, int64_t Vd, const int32_t *d2t, int k, int32_t *out_ids,
                      float *out_logp, int32_t *out_draft_idx, float *lse_out)
{
#pragma omp parallel for schedule(dynamic)
    for (int64_t r = 0; r < R; ++r) {
        const float *zr = z + r * Vd;
        float lse = vto_lse_row(zr, Vd);
        int32_t *best = (int32_t *)malloc((size_t)k * sizeof(int32_t));
        vto_topk_row(zr, Vd, k, best);
        for (int p = 0; p < k; ++p) {
            out_ids[r * k + p] = d2t[best[p]];
            out_logp[r * k + p] = zr[best[p]] - lse;
            if (out_draft_idx)
                out_draft_idx[r * k + p] = best[p];
        }
        if (lse_out)
            lse_out[r] = lse;
        free(best);
    }
}

/*
 * The whole per-step head: logits, softmax normaliser over V_d, k best, d2t remap.
 *   out_ids[R,k]   ids in the target vocabulary, best first
 *   out_logp[R,k]  log-softmax over V_d of those tokens
 * Optional (may be NULL): out_draft_idx[R,k] positions inside V_d, z_out[R,Vd], lse_out[R],
 * flops.  Returns 0, or -1 when k is outside [1,Vd].
 */
int vto_draft_head(const uint16_t *h, int64_t R, int64_t H, const uint16_t *W_sub,
                   const int32_t *d2t, int64_t Vd, int k, int32_t *out_ids, float *out_logp,
                   int32_t *out_draft_idx, float *z_out, float *lse_out, int64_t *flops)
{
    if (k < 1 || k > Vd)
        return -1;
    float *z = z_out ? z_out : (float *)malloc((size_t)R * (size_t)Vd * sizeof(float));
    vto_logits(h, R, H, W_sub, Vd, z, flops);
    emit_rows(z, R, Vd, d2t, k, out_ids, out_logp, out_draft_idx, lse_out);
    if (!z_out)
        free(z);
    return 0;
}

/*
 * The same head over a weight matrix given in fp32 (a compressed W_sub after dequantisation:
 * the stored code times its scale, rounded once to fp32): bf16 hidden states, fp32 weights,
 * sequential fp32 accumulation in ascending i with a separate multiply and add.
 */
void vto_logits_w32(const uint16_t *h, int64_t R, int64_t H, const float *W32, int64_t Vd, float *z)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t r = 0; r < R; ++r) {
        for (int64_t j = 0; j < Vd; ++j) {
            const uint16_t *hr = h + r * H;
            const float *wj = W32 + j * H;
            float acc = 0.0f;
            for (int64_t i = 0; i < H; ++i) {
                float prod = widen_bf16(hr[i]) * wj[i];
                acc = acc + prod;
            }
            z[r * Vd + j] = acc;
        }
    }
}

int vto_draft_head_w32(const uint16_t *h, int64_t R, int64_t H, const float *W32, const int32_t *d2t,
                       int64_t Vd, int k, int32_t *out_ids, float *out_logp, int32_t *out_draft_idx,
                       float *z_out, float *lse_out)
{
    if (k < 1 || k > Vd)
        return -1;
    float *z = z_out ? z_out : (float *)malloc((size_t)R * (size_t)Vd * sizeof(float));
    vto_logits_w32(h, R, H, W32, Vd, z);
    emit_rows(z, R, Vd, d2t, k, out_ids, out_logp, out_draft_idx, lse_out);
    if (!z_out)
        free(z);
    return 0;
}
