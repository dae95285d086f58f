/* Driver for the host-sanitizer build of the CPU oracle (address + undefined-behaviour
 * sanitizers): runs every oracle function on small inputs, including the error returns, and
 * prints a checksum.  Any out-of-bounds access, leak or undefined operation aborts the run. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int vto_num_threads(void);
int vto_build_subset(const uint16_t *W, int64_t V, int64_t H, const int32_t *ids, int64_t Vd, uint16_t *W_sub,
                     int32_t *d2t);
void vto_logits(const uint16_t *h, int64_t R, int64_t H, const uint16_t *W_sub, int64_t Vd, float *z, int64_t *flops);
void vto_logits_f64(const uint16_t *h, int64_t R, int64_t H, const uint16_t *W_sub, int64_t Vd, double *z);
float vto_lse_row(const float *z, int64_t Vd);
void vto_topk_row(const float *z, int64_t Vd, int k, int32_t *idx_out);
int vto_draft_head(const uint16_t *h, int64_t R, int64_t H, const uint16_t *W_sub, const int32_t *d2t, int64_t Vd,
                   int k, int32_t *out_ids, float *out_logp, int32_t *out_draft_idx, float *z_out, float *lse_out,
                   int64_t *flops);

static uint32_t lcg(uint32_t *s)
{
    *s = *s * 1664525u + 1013904223u;
    return *s >> 8;
}

int main(void)
{
    enum { V = 97, H = 40, VD = 31, R = 3, K = 7 };
    uint32_t seed = 12345u;
    uint16_t *W = malloc(sizeof(uint16_t) * V * H), *h = malloc(sizeof(uint16_t) * R * H);
    uint16_t *W_sub = malloc(sizeof(uint16_t) * VD * H);
    int32_t *ids = malloc(sizeof(int32_t) * VD), *d2t = malloc(sizeof(int32_t) * VD);
    for (int i = 0; i < V * H; ++i) /* small finite bf16 patterns: sign, exponent 120..127, 7 mantissa bits */
        W[i] = (uint16_t)(((lcg(&seed) & 1u) << 15) | ((120u + lcg(&seed) % 8u) << 7) | (lcg(&seed) & 0x7fu));
    for (int i = 0; i < R * H; ++i)
        h[i] = (uint16_t)(((lcg(&seed) & 1u) << 15) | ((124u + lcg(&seed) % 4u) << 7) | (lcg(&seed) & 0x7fu));
    for (int j = 0; j < VD; ++j)
        ids[j] = (j * 3 + 1) % V;
    if (vto_build_subset(W, V, H, ids, VD, W_sub, d2t) != 0)
        return 2;
    ids[5] = V; /* out of range */
    if (vto_build_subset(W, V, H, ids, VD, W_sub, d2t) != -1)
        return 3;
    ids[5] = ids[4]; /* duplicate */
    if (vto_build_subset(W, V, H, ids, VD, W_sub, d2t) != -2)
        return 4;
    float *z = malloc(sizeof(float) * R * VD), *lse = malloc(sizeof(float) * R), *logp = malloc(sizeof(float) * R * K);
    double *z64 = malloc(sizeof(double) * R * VD);
    int32_t *out = malloc(sizeof(int32_t) * R * K), *didx = malloc(sizeof(int32_t) * R * K), top[VD];
    int64_t flops = 0;
    vto_logits(h, R, H, W_sub, VD, z, &flops);
    vto_logits_f64(h, R, H, W_sub, VD, z64);
    if (flops != 2LL * R * H * VD)
        return 5;
    double sum = vto_lse_row(z, VD);
    vto_topk_row(z, VD, VD, top); /* k == V_draft */
    vto_topk_row(z, VD, 1, top);
    if (vto_draft_head(h, R, H, W_sub, d2t, VD, K, out, logp, didx, z, lse, &flops) != 0)
        return 6;
    if (vto_draft_head(h, R, H, W_sub, d2t, VD, K, out, logp, NULL, NULL, NULL, NULL) != 0)
        return 7;
    if (vto_draft_head(h, R, H, W_sub, d2t, VD, VD + 1, out, logp, NULL, NULL, NULL, NULL) != -1)
        return 8;
    for (int i = 0; i < R * K; ++i)
        sum += logp[i] + out[i];
    printf("san_oracle ok threads=%d checksum=%.6f\n", vto_num_threads(), sum + z64[0]);
    free(W); free(h); free(W_sub); free(ids); free(d2t); free(z); free(z64); free(lse); free(logp); free(out); free(didx);
    return 0;
}
