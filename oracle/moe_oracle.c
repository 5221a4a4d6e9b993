/*
 * CPU oracle for one GPU's share of a Mixture-of-Experts layer.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct loops that state
 * what the layer share computes; nothing here is tuned and nothing here is
 * shared with the HIP library (no common header, helper, table or constant).
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.
 *
 * The layer share, as the paper states it (Sec. II background on TP / EP,
 * Sec. III-B-2 "A2A", Alg. 1 and Alg. 2):
 *   route    each token is assigned to its top-k activated experts; the
 *            expert map is computed from the local hidden states (Alg. 2,
 *            the `route` step)
 *   dispatch each token is sent to the device hosting the expert: here, the
 *            expert-contiguous buffer that exchange would carry
 *   MLP      every expert is an independent MLP; under TP its weights are
 *            sliced and the partial results are summed afterwards
 *   combine  results return along the original route, weighted by the top-k
 *            weights (the accumulation step of Alg. 1); the result is
 *            the partial sum the intra-node all-reduce would finish
 * The paper fixes no numerical detail (score function, MLP form, precision);
 * those follow the benchmark configurations: softmax or sigmoid scores,
 * optional group-limited selection, renormalised weights times a scale,
 * SwiGLU experts without biases.
 *
 * Arithmetic: inputs are fp32 arrays (bf16 / e4m3 storage is decoded exactly
 * by the Python wrapper); every sum, score and activation is fp64; the final
 * output is stored fp32.  Ties go to the lowest index.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define SCORE_SOFTMAX 0
#define SCORE_SIGMOID 1

/* ---- route: gate scores + top-k (Sec. III-B-2; Alg. 2 `route`) ---------- */
/*
 * x [T,H], gate_w [E,H]; logit_bias / select_bias [E] or NULL; logits_in [T,E]
 * or NULL (when given the dot products are skipped and these values are the
 * logits).  Outputs: ids [T,k] in pick order (descending key), w [T,k],
 * margin [T] = smallest gap between two keys (or two group scores) that the
 * selection had to tell apart, logits_out [T,E] or NULL.
 */
void oracle_route(int T, int H, int E, int k, int score_fn, int renormalize,
                  double routed_scale, int n_groups, int topk_groups, int group_score_n,
                  const float *x, const float *gate_w, const float *logit_bias,
                  const float *select_bias, const float *logits_in,
                  int32_t *ids, float *w, double *margin, double *logits_out)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double *z = (double *)malloc(sizeof(double) * E);      /* logits            */
        double *s = (double *)malloc(sizeof(double) * E);      /* scores            */
        double *key = (double *)malloc(sizeof(double) * E);    /* selection keys    */
        char *eligible = (char *)malloc(E);
        char *taken = (char *)malloc(E);
        double mgn = INFINITY;

        for (int e = 0; e < E; ++e) {
            double acc;
            if (logits_in) {
                acc = (double)logits_in[(size_t)t * E + e];
            } else {
                acc = 0.0;
                for (int h = 0; h < H; ++h)
                    acc += (double)x[(size_t)t * H + h] * (double)gate_w[(size_t)e * H + h];
            }
            if (logit_bias) acc += (double)logit_bias[e];
            z[e] = acc;
            if (logits_out) logits_out[(size_t)t * E + e] = acc;
        }

        /* scores and selection keys */
        if (score_fn == SCORE_SOFTMAX) {
            double zmax = z[0];
            for (int e = 1; e < E; ++e) if (z[e] > zmax) zmax = z[e];
            double den = 0.0;
            for (int e = 0; e < E; ++e) { s[e] = exp(z[e] - zmax); den += s[e]; }
            for (int e = 0; e < E; ++e) s[e] /= den;
            /* softmax is increasing in the logit: select on the logit itself */
            for (int e = 0; e < E; ++e) key[e] = z[e];
        } else {
            for (int e = 0; e < E; ++e) {
                s[e] = 1.0 / (1.0 + exp(-z[e]));
                key[e] = s[e] + (select_bias ? (double)select_bias[e] : 0.0);
            }
        }

        /* group-limited eligibility */
        for (int e = 0; e < E; ++e) eligible[e] = 1;
        if (n_groups > 1) {
            int gs = E / n_groups;
            double *gscore = (double *)malloc(sizeof(double) * n_groups);
            char *gkept = (char *)calloc(n_groups, 1);
            for (int g = 0; g < n_groups; ++g) {
                /* sum of the group_score_n largest keys of the group */
                memset(taken, 0, E);
                double sum = 0.0;
                for (int r = 0; r < group_score_n && r < gs; ++r) {
                    int best = -1;
                    for (int e = g * gs; e < (g + 1) * gs; ++e)
                        if (!taken[e] && (best < 0 || key[e] > key[best])) best = e;
                    taken[best] = 1;
                    sum += key[best];
                }
                gscore[g] = sum;
            }
            double last_kept = 0.0;
            for (int r = 0; r < topk_groups; ++r) {
                int best = -1;
                for (int g = 0; g < n_groups; ++g)
                    if (!gkept[g] && (best < 0 || gscore[g] > gscore[best])) best = g;
                gkept[best] = 1;
                last_kept = gscore[best];
            }
            for (int g = 0; g < n_groups; ++g) {
                if (!gkept[g]) {
                    if (last_kept - gscore[g] < mgn) mgn = last_kept - gscore[g];
                    for (int e = g * gs; e < (g + 1) * gs; ++e) eligible[e] = 0;
                }
            }
            free(gscore);
            free(gkept);
        }

        /* top-k: k times the largest remaining eligible key, ties -> lowest id */
        memset(taken, 0, E);
        double prev = 0.0;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (eligible[e] && !taken[e] && (best < 0 || key[e] > key[best])) best = e;
            taken[best] = 1;
            ids[(size_t)t * k + j] = best;
            if (j > 0 && prev - key[best] < mgn) mgn = prev - key[best];
            prev = key[best];
        }
        for (int e = 0; e < E; ++e)
            if (eligible[e] && !taken[e] && prev - key[e] < mgn) mgn = prev - key[e];
        margin[t] = mgn;

        /* weights: un-biased scores of the picked experts */
        double den = 1.0;
        if (renormalize) {
            den = 0.0;
            for (int j = 0; j < k; ++j) den += s[ids[(size_t)t * k + j]];
        }
        for (int j = 0; j < k; ++j)
            w[(size_t)t * k + j] = (float)(s[ids[(size_t)t * k + j]] / den * routed_scale);

        free(z); free(s); free(key); free(eligible); free(taken);
    }
}

/* ---- dispatch: expert-contiguous send buffer (Sec. II EP; Alg. 2) -------- */
/*
 * ids [T,k] global expert ids; local range [e_lo,e_hi).  Flat assignment
 * a = t*k+j.  counts [E_loc], offsets [E_loc+1] (exclusive scan), perm
 * [T*k] (first offsets[E_loc] entries valid: position -> a), inv [T*k]
 * (a -> position, -1 when the expert is not local), xs [T*k,H] (first
 * offsets[E_loc] rows valid; row copies of x).  Stable: inside an expert the
 * assignments keep ascending a.
 */
void oracle_dispatch(int T, int k, int H, int e_lo, int e_hi,
                     const int32_t *ids, const float *x,
                     int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv,
                     float *xs)
{
    int E_loc = e_hi - e_lo;
    int A = T * k;
    for (int e = 0; e < E_loc; ++e) counts[e] = 0;
    for (int a = 0; a < A; ++a)
        if (ids[a] >= e_lo && ids[a] < e_hi) counts[ids[a] - e_lo]++;
    offsets[0] = 0;
    for (int e = 0; e < E_loc; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t *fill = (int32_t *)calloc(E_loc > 0 ? E_loc : 1, sizeof(int32_t));
    for (int a = 0; a < A; ++a) {
        int e = ids[a] - e_lo;
        if (e >= 0 && e < E_loc) {
            int pos = offsets[e] + fill[e]++;
            perm[pos] = a;
            inv[a] = pos;
            if (xs) memcpy(xs + (size_t)pos * H, x + (size_t)(a / k) * H, sizeof(float) * H);
        } else {
            inv[a] = -1;
        }
    }
    free(fill);
}

/* ---- expert MLP: SwiGLU on a TP slice (Sec. II TP / EP; Sec. III-B-1) ---- */
/*
 * For expert e the rows offsets[e]..offsets[e+1] of xs [rows,H]:
 *   g = Wgate_e xs_r, u = Wup_e xs_r, hmid = g*sigmoid(g)*u, ys_r = Wdown_e hmid
 * Wgate,Wup [n,I,H]; Wdown [n,H,I].  Optional block scales (fp8 storage):
 * s_gate,s_up [n,ceil(I/128),ceil(H/128)], s_down [n,ceil(H/128),ceil(I/128)];
 * the weight is stored_value * scale[row/128][col/128], formed in fp64.
 * ys [rows,H] fp64.  No intermediate is rounded.
 */
void oracle_expert_ffn(int n_experts, const int32_t *offsets, int H, int I,
                       const float *xs, const float *w_gate, const float *w_up,
                       const float *w_down, const float *s_gate, const float *s_up,
                       const float *s_down, double *ys)
{
    int bH = (H + 127) / 128, bI = (I + 127) / 128;
    for (int e = 0; e < n_experts; ++e) {
        const float *Wg = w_gate + (size_t)e * I * H;
        const float *Wu = w_up + (size_t)e * I * H;
        const float *Wd = w_down + (size_t)e * H * I;
#pragma omp parallel for schedule(dynamic, 1)
        for (int r = offsets[e]; r < offsets[e + 1]; ++r) {
            const float *xr = xs + (size_t)r * H;
            double *hmid = (double *)malloc(sizeof(double) * I);
            for (int i = 0; i < I; ++i) {
                double g = 0.0, u = 0.0;
                for (int h = 0; h < H; ++h) {
                    double wg = (double)Wg[(size_t)i * H + h];
                    double wu = (double)Wu[(size_t)i * H + h];
                    if (s_gate) wg *= (double)s_gate[((size_t)e * bI + i / 128) * bH + h / 128];
                    if (s_up) wu *= (double)s_up[((size_t)e * bI + i / 128) * bH + h / 128];
                    g += wg * (double)xr[h];
                    u += wu * (double)xr[h];
                }
                hmid[i] = g / (1.0 + exp(-g)) * u;
            }
            for (int h = 0; h < H; ++h) {
                double acc = 0.0;
                for (int i = 0; i < I; ++i) {
                    double wd = (double)Wd[(size_t)h * I + i];
                    if (s_down) wd *= (double)s_down[((size_t)e * bH + h / 128) * bI + i / 128];
                    acc += wd * hmid[i];
                }
                ys[(size_t)r * H + h] = acc;
            }
            free(hmid);
        }
    }
}

/* ---- expert MLP with 8-bit activations (scope extension, not in the paper) -- */
/*
 * Activations are quantised on the fly, one fp32 scale per row and block of
 * 128 columns: amax = max|x| over the block, scale = amax / 448 (1 when the
 * block is all zero), code = e4m3(x / scale) with round-to-nearest-even after
 * clamping to +-448.  amax, the two divisions and the clamp are fp32 operations
 * (the decision which code a value gets is taken in fp32 on both sides); the
 * value a code stands for, decode(code) * scale, and every sum are fp64.
 */
static double e4m3_value(int c)
{
    int ex = (c >> 3) & 15, m = c & 7;
    double v = ex == 0 ? ldexp((double)m / 8.0, -6) : ldexp(1.0 + (double)m / 8.0, ex - 7);
    return (c & 0x80) ? -v : v;
}

/* nearest finite e4m3 value, ties to the even code: a search over all codes */
static uint8_t e4m3_nearest(float q)
{
    int best = 0;
    double bd = fabs((double)q);
    for (int c = 1; c < 0x7F; ++c) {
        double d = fabs(fabs((double)q) - e4m3_value(c));
        if (d < bd || (d == bd && (c & 1) == 0 && (best & 1) == 1)) { bd = d; best = c; }
    }
    return (uint8_t)(best | (signbit(q) ? 0x80 : 0));
}

/* x [rows,K] fp32, K a multiple of 128 -> codes [rows,K], scales [rows,K/128] */
void oracle_quant_act_1x128(int rows, int K, const float *x, uint8_t *codes, float *scales)
{
    int nb = K / 128;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r)
        for (int b = 0; b < nb; ++b) {
            const float *xb = x + (size_t)r * K + (size_t)b * 128;
            float amax = 0.0f;
            for (int j = 0; j < 128; ++j) amax = fmaxf(amax, fabsf(xb[j]));
            float scale = amax > 0.0f ? amax / 448.0f : 1.0f;
            scales[(size_t)r * nb + b] = scale;
            for (int j = 0; j < 128; ++j) {
                float q = xb[j] / scale;
                q = fminf(fmaxf(q, -448.0f), 448.0f);
                codes[(size_t)r * K + (size_t)b * 128 + j] = e4m3_nearest(q);
            }
        }
}

/*
 * The grouped SwiGLU MLP of oracle_expert_ffn with quantised activations:
 *   xq = quant(xs row);  g = Wgate_e xq, u = Wup_e xq;  hmid = g*sigmoid(g)*u
 *   (fp64, no intermediate storage format), handed to the same quantiser as
 *   its fp32 value;  ys_r = Wdown_e hq.
 * Weights are e4m3 values (already decoded to fp32) with 128x128 block scales.
 * H and I are multiples of 128.  ys [rows,H] fp64.
 */
void oracle_expert_ffn_fp8act(int n_experts, const int32_t *offsets, int H, int I,
                              const float *xs, const float *w_gate, const float *w_up,
                              const float *w_down, const float *s_gate, const float *s_up,
                              const float *s_down, double *ys)
{
    int bH = H / 128, bI = I / 128;
    for (int e = 0; e < n_experts; ++e) {
        const float *Wg = w_gate + (size_t)e * I * H;
        const float *Wu = w_up + (size_t)e * I * H;
        const float *Wd = w_down + (size_t)e * H * I;
#pragma omp parallel for schedule(dynamic, 1)
        for (int r = offsets[e]; r < offsets[e + 1]; ++r) {
            uint8_t *cx = (uint8_t *)malloc((size_t)H), *ch = (uint8_t *)malloc((size_t)I);
            float *sx = (float *)malloc(sizeof(float) * bH), *sh = (float *)malloc(sizeof(float) * bI);
            float *hb = (float *)malloc(sizeof(float) * I);
            double *xq = (double *)malloc(sizeof(double) * H), *hq = (double *)malloc(sizeof(double) * I);
            oracle_quant_act_1x128(1, H, xs + (size_t)r * H, cx, sx);
            for (int h = 0; h < H; ++h) xq[h] = e4m3_value(cx[h]) * (double)sx[h / 128];
            for (int i = 0; i < I; ++i) {
                double g = 0.0, u = 0.0;
                for (int h = 0; h < H; ++h) {
                    double wg = (double)Wg[(size_t)i * H + h] * (double)s_gate[((size_t)e * bI + i / 128) * bH + h / 128];
                    double wu = (double)Wu[(size_t)i * H + h] * (double)s_up[((size_t)e * bI + i / 128) * bH + h / 128];
                    g += wg * xq[h];
                    u += wu * xq[h];
                }
                hb[i] = (float)(g / (1.0 + exp(-g)) * u);
            }
            oracle_quant_act_1x128(1, I, hb, ch, sh);
            for (int i = 0; i < I; ++i) hq[i] = e4m3_value(ch[i]) * (double)sh[i / 128];
            for (int h = 0; h < H; ++h) {
                double acc = 0.0;
                for (int i = 0; i < I; ++i)
                    acc += (double)Wd[(size_t)h * I + i] * (double)s_down[((size_t)e * bH + h / 128) * bI + i / 128] * hq[i];
                ys[(size_t)r * H + h] = acc;
            }
            free(cx); free(ch); free(sx); free(sh); free(hb); free(xq); free(hq);
        }
    }
}

/* ---- combine: weighted return along the route (Alg. 1; Sec. III-B-2 AR) -- */
/*
 * out[t,:] = sum over j ascending with inv[t*k+j] >= 0 of
 *            w[t,j] * ys[inv[t*k+j],:]   (+ shared_ys[t,:] when given)
 * fp64 accumulation, stored fp32: the partial sum awaiting the all-reduce.
 */
void oracle_combine(int T, int k, int H, const double *ys, const int32_t *inv,
                    const float *w, const double *shared_ys, float *out)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j) {
                int pos = inv[(size_t)t * k + j];
                if (pos >= 0) acc += (double)w[(size_t)t * k + j] * ys[(size_t)pos * H + h];
            }
            if (shared_ys) acc += shared_ys[(size_t)t * H + h];
            out[(size_t)t * H + h] = (float)acc;
        }
    }
}

/* ---- collective-ready layouts of the fused schedules (Sec. III-C, Alg. 1, 2) ---- */
/*
 * Fused AG-Dispatch (Alg. 2): hidden states are replicated in the TP group, so
 * TP rank r of m computes the expert map on its own and sends only its hidden-
 * column shard X_r of every routed row.  Index outputs as oracle_dispatch;
 *   xs_shard [A_loc, H/m]:  xs_shard[pos][c] = x[perm[pos]/k][r*H/m + c].
 */
void oracle_dispatch_shard(int T, int k, int H, int e_lo, int e_hi, int tp_rank, int tp_size,
                           const int32_t *ids, const float *x,
                           int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv,
                           float *xs_shard)
{
    int E_loc = e_hi - e_lo;
    int A = T * k;
    int Hs = H / tp_size;
    for (int e = 0; e < E_loc; ++e) counts[e] = 0;
    for (int a = 0; a < A; ++a)
        if (ids[a] >= e_lo && ids[a] < e_hi) counts[ids[a] - e_lo]++;
    offsets[0] = 0;
    for (int e = 0; e < E_loc; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t *fill = (int32_t *)calloc(E_loc > 0 ? E_loc : 1, sizeof(int32_t));
    for (int a = 0; a < A; ++a) {
        int e = ids[a] - e_lo;
        if (e >= 0 && e < E_loc) {
            int pos = offsets[e] + fill[e]++;
            perm[pos] = a;
            inv[a] = pos;
            for (int c = 0; c < Hs; ++c)
                xs_shard[(size_t)pos * Hs + c] = x[(size_t)(a / k) * H + (size_t)tp_rank * Hs + c];
        } else {
            inv[a] = -1;
        }
    }
    free(fill);
}

/*
 * One stage of the fused RS-Combine (Alg. 1): the rows S_i of stage i, scaled by
 * their top-k weights, are added to the running block Y_i,
 * on one hidden-column block of width Hb = H/m.
 *   s[t][c] = sum_{j: inv[t*k+j] >= 0} w[t][j] * ys_block[inv[t*k+j]][c]   (fp64)
 *   out_block[t][c] = (accumulate ? out_block[t][c] : 0) + s[t][c], stored fp32.
 */
void oracle_combine_stage(int T, int k, int Hb, const double *ys_block, const int32_t *inv,
                          const float *w, int accumulate, float *out_block)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int c = 0; c < Hb; ++c) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j) {
                int pos = inv[(size_t)t * k + j];
                if (pos >= 0) acc += (double)w[(size_t)t * k + j] * ys_block[(size_t)pos * Hb + c];
            }
            if (accumulate) acc += (double)out_block[(size_t)t * Hb + c];
            out_block[(size_t)t * Hb + c] = (float)acc;
        }
    }
}

/* ---- storage decoders (exact) ------------------------------------------- */
/* OCP e4m3: 1 sign, 4 exponent (bias 7), 3 mantissa bits; exponent field 0 is
 * subnormal (m/8 * 2^-6); 0x7F / 0xFF are NaN; there are no infinities. */
void oracle_decode_e4m3(const uint8_t *codes, size_t n, float *out)
{
    for (size_t i = 0; i < n; ++i) {
        int c = codes[i];
        int sgn = c >> 7, ex = (c >> 3) & 15, m = c & 7;
        double v;
        if (ex == 15 && m == 7) v = NAN;
        else if (ex == 0) v = ldexp((double)m / 8.0, -6);
        else v = ldexp(1.0 + (double)m / 8.0, ex - 7);
        out[i] = (float)(sgn ? -v : v);
    }
}

/* bf16 is the upper half of an fp32 pattern. */
void oracle_decode_bf16(const uint16_t *bits, size_t n, float *out)
{
    for (size_t i = 0; i < n; ++i) {
        uint32_t u = (uint32_t)bits[i] << 16;
        memcpy(out + i, &u, 4);
    }
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
