/*
 * Sanitizer leg of the CPU oracle: compiled together with oracle/moe_oracle.c
 * under -fsanitize=address,undefined and run by tests/test_sanitizers.py.
 * Walks every exported function of the oracle over small layers that include
 * the edge cases (an expert without tokens, no local assignment at all, a
 * single token, group-limited routing, block scales, column shards, staged
 * combine) and checks a few invariants; any out-of-bounds access, use of an
 * uninitialised index or undefined arithmetic aborts the run.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_route(int T, int H, int E, int k, int score_fn, int renormalize, double routed_scale,
                  int n_groups, int topk_groups, int group_score_n, const float *x,
                  const float *gate_w, const float *logit_bias, const float *select_bias,
                  const float *logits_in, int32_t *ids, float *w, double *margin, double *logits_out);
void oracle_dispatch(int T, int k, int H, int e_lo, int e_hi, const int32_t *ids, const float *x,
                     int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv, float *xs);
void oracle_expert_ffn(int n_experts, const int32_t *offsets, int H, int I, const float *xs,
                       const float *w_gate, const float *w_up, const float *w_down,
                       const float *s_gate, const float *s_up, const float *s_down, double *ys);
void oracle_quant_act_1x128(int rows, int K, const float *x, uint8_t *codes, float *scales);
void oracle_expert_ffn_fp8act(int n_experts, const int32_t *offsets, int H, int I, const float *xs,
                              const float *w_gate, const float *w_up, const float *w_down,
                              const float *s_gate, const float *s_up, const float *s_down, double *ys);
void oracle_combine(int T, int k, int H, const double *ys, const int32_t *inv, const float *w,
                    const double *shared_ys, float *out);
void oracle_dispatch_shard(int T, int k, int H, int e_lo, int e_hi, int tp_rank, int tp_size,
                           const int32_t *ids, const float *x, int32_t *counts, int32_t *offsets,
                           int32_t *perm, int32_t *inv, float *xs_shard);
void oracle_combine_stage(int T, int k, int Hb, const double *ys_block, const int32_t *inv,
                          const float *w, int accumulate, float *out_block);
void oracle_decode_e4m3(const uint8_t *codes, size_t n, float *out);
void oracle_decode_bf16(const uint16_t *bits, size_t n, float *out);
int oracle_num_threads(void);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static float rnd(void)            /* uniform in [-1, 1) */
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
static float *vec(size_t n, float scale)
{
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = rnd() * scale;
    return p;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); exit(3); } } while (0)

static void layer(int T, int H, int E, int k, int I, int score_fn, int G, int Kg, int gn,
                  int e_lo, int e_hi, int fp8, int shared)
{
    float *x = vec((size_t)T * H, 1.0f), *gw = vec((size_t)E * H, 0.1f);
    float *lb = vec(E, 0.5f), *sb = vec(E, 0.05f);
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * T * k);
    float *w = (float *)malloc(sizeof(float) * T * k);
    double *margin = (double *)malloc(sizeof(double) * T);
    double *logits = (double *)malloc(sizeof(double) * T * E);
    oracle_route(T, H, E, k, score_fn, 1, 2.5, G, Kg, gn, x, gw, score_fn ? NULL : lb,
                 score_fn ? sb : NULL, NULL, ids, w, margin, logits);
    for (int t = 0; t < T; ++t) {
        double sum = 0.0;
        for (int j = 0; j < k; ++j) {
            CHECK(ids[t * k + j] >= 0 && ids[t * k + j] < E);
            for (int i = 0; i < j; ++i) CHECK(ids[t * k + i] != ids[t * k + j]);
            sum += w[t * k + j];
        }
        CHECK(fabs(sum - 2.5) < 1e-4);
        CHECK(margin[t] >= 0.0);
    }
    /* the same selection from given logits */
    float *lin = (float *)malloc(sizeof(float) * T * E);
    for (int i = 0; i < T * E; ++i) lin[i] = (float)logits[i];
    int32_t *ids2 = (int32_t *)malloc(sizeof(int32_t) * T * k);
    oracle_route(T, H, E, k, score_fn, 0, 1.0, G, Kg, gn, NULL, gw, NULL, score_fn ? sb : NULL, lin,
                 ids2, w, margin, NULL);

    int El = e_hi - e_lo, A = T * k;
    int32_t *counts = (int32_t *)malloc(sizeof(int32_t) * El), *offsets = (int32_t *)malloc(sizeof(int32_t) * (El + 1));
    int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * A), *inv = (int32_t *)malloc(sizeof(int32_t) * A);
    float *xs = (float *)calloc((size_t)A * H, sizeof(float));
    oracle_dispatch(T, k, H, e_lo, e_hi, ids, x, counts, offsets, perm, inv, xs);
    int n = offsets[El];
    CHECK(offsets[0] == 0 && n <= A);
    for (int p = 0; p < n; ++p) CHECK(inv[perm[p]] == p);

    int bH = (H + 127) / 128, bI = (I + 127) / 128;
    float *wg = vec((size_t)El * I * H, 0.05f), *wu = vec((size_t)El * I * H, 0.05f), *wd = vec((size_t)El * H * I, 0.05f);
    float *sg = vec((size_t)El * bI * bH, 1.0f), *su = vec((size_t)El * bI * bH, 1.0f), *sd = vec((size_t)El * bH * bI, 1.0f);
    double *ys = (double *)calloc((size_t)A * H, sizeof(double));
    if (fp8 == 2)
        oracle_expert_ffn_fp8act(El, offsets, H, I, xs, wg, wu, wd, sg, su, sd, ys);
    else
        oracle_expert_ffn(El, offsets, H, I, xs, wg, wu, wd, fp8 ? sg : NULL, fp8 ? su : NULL, fp8 ? sd : NULL, ys);
    double *ysh = NULL;
    if (shared) {
        int32_t so[2] = {0, T};
        ysh = (double *)calloc((size_t)T * H, sizeof(double));
        oracle_expert_ffn(1, so, H, I, x, wg, wu, wd, NULL, NULL, NULL, ysh);
    }
    float *out = (float *)malloc(sizeof(float) * T * H);
    oracle_combine(T, k, H, ys, inv, w, ysh, out);
    for (int i = 0; i < T * H; ++i) CHECK(isfinite(out[i]));

    /* column shards and staged combine over two ranks */
    if (H % 2 == 0) {
        int Hs = H / 2;
        float *xsh = (float *)calloc((size_t)A * Hs, sizeof(float));
        oracle_dispatch_shard(T, k, H, e_lo, e_hi, 1, 2, ids, x, counts, offsets, perm, inv, xsh);
        for (int p = 0; p < n; ++p) CHECK(xsh[(size_t)p * Hs] == xs[(size_t)p * H + Hs]);
        double *yb = (double *)calloc((size_t)(A ? A : 1) * Hs, sizeof(double));
        float *ob = (float *)malloc(sizeof(float) * T * Hs);
        oracle_combine_stage(T, k, Hs, yb, inv, w, 0, ob);
        oracle_combine_stage(T, k, Hs, yb, inv, w, 1, ob);
        free(xsh); free(yb); free(ob);
    }
    free(x); free(gw); free(lb); free(sb); free(ids); free(ids2); free(w); free(margin); free(logits); free(lin);
    free(counts); free(offsets); free(perm); free(inv); free(xs); free(wg); free(wu); free(wd);
    free(sg); free(su); free(sd); free(ys); free(ysh); free(out);
}

int main(void)
{
    CHECK(oracle_num_threads() >= 1);
    /* softmax top-2 of 8, all local; one token; an EP range; nobody local */
    layer(17, 64, 8, 2, 32, 0, 1, 1, 0, 0, 8, 0, 0);
    layer(1, 64, 8, 3, 32, 0, 1, 1, 0, 0, 8, 0, 1);
    layer(33, 64, 16, 4, 32, 0, 1, 1, 0, 5, 9, 0, 0);
    layer(3, 64, 16, 1, 32, 0, 1, 1, 0, 15, 16, 0, 0);
    /* sigmoid, group-limited: 4 groups of 4, keep 2, group score of 2 keys */
    layer(29, 64, 16, 4, 32, 1, 4, 2, 2, 0, 8, 0, 1);
    /* block-scaled weights (128-multiples) and 8-bit activations */
    layer(9, 256, 8, 2, 128, 1, 2, 1, 1, 2, 6, 1, 0);
    layer(9, 256, 8, 2, 128, 0, 1, 1, 0, 0, 8, 2, 0);
    /* storage decoders over every code / a spread of patterns */
    uint8_t c8[256]; float f8[256];
    for (int i = 0; i < 256; ++i) c8[i] = (uint8_t)i;
    oracle_decode_e4m3(c8, 256, f8);
    CHECK(f8[0x7E] == 448.0f && f8[0xFE] == -448.0f);
    uint16_t b16[4] = {0x3F80, 0xBF80, 0x0000, 0x4000}; float f16[4];
    oracle_decode_bf16(b16, 4, f16);
    CHECK(f16[0] == 1.0f && f16[1] == -1.0f && f16[2] == 0.0f && f16[3] == 2.0f);
    /* the quantiser on an all-zero block and an outlier */
    float row[256] = {0}; uint8_t codes[256]; float scales[2];
    row[130] = 1000.0f;
    oracle_quant_act_1x128(1, 256, row, codes, scales);
    CHECK(scales[0] == 1.0f && codes[130] == 0x7E);
    puts("oracle sanitizer leg: ok");
    return 0;
}
