/*
 * CPU oracle for the routed-expert forward of a sub-expert MoE layer with a
 * per-token routing budget.  TEST INFRASTRUCTURE ONLY: it exists to check the
 * HIP library and to be timed beside it; nothing in the product path may call
 * it.  It shares no code with the HIP path.
 *
 * Everything here is the plain definition, one output at a time, with no
 * blocking, fusion or reordering:
 *   - SwiGLU expert and its neuron-wise decomposition: Sec. 3.2.1, Eq. 1-3.
 *   - Expanded linear gate over all E = N*S sub-experts with a layer-wide
 *     top-k: Sec. 3.2.2 ("Low-Cost Fine-Tuning" paragraph).
 *   - The budget k belongs to the request and every token inherits it:
 *     Sec. 3.3.1.
 *   - Gate-weighted sum of the selected sub-expert outputs: Sec. 3.2.2 (the
 *     routed-output expression of the proxy-gating paragraph; the linear gate
 *     uses the same sum with one weight per sub-expert).
 *   - Training-free proxy gate (original router, gate-neuron scores, per-expert
 *     top-kappa): Sec. 3.2.2 ("Training-Free Proxy Gating"); at the end of this file.
 *
 * Precision.  Router logits decide integers (which sub-experts are chosen), so
 * they are computed in the precision the device uses for that decision: one
 * IEEE-754 binary32 fused multiply-add chain per logit, hidden index ascending,
 * then one binary32 add of the bias.  All value arithmetic after the decision
 * (softmax weights, FFN, combine) is binary64.
 *
 * Parity pins (tests/test_oracle_pins.py): every function below is pinned to
 * something other than itself; none is "parity unpinned".
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC (see oracle/build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_API __attribute__((visibility("default")))

static int clamp_k(int k, int k_max) { return k < 0 ? 0 : (k > k_max ? k_max : k); }

/* Router logits, Sec. 3.2.2: a standard linear layer scoring every sub-expert.
 * l[t,g] = fl32( chain_j fma(x[t,j], w_r[g,j], acc) ) (+ bias[g], one fl32 add). */
ORACLE_API int oracle_logits(int T, int d, int E, const float *x, const float *w_r,
                             const float *bias, float *logits)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int g = 0; g < E; ++g) {
            float acc = 0.0f;
            for (int j = 0; j < d; ++j)
                acc = fmaf(x[(size_t)t * d + j], w_r[(size_t)g * d + j], acc);
            if (bias) acc = acc + bias[g];
            logits[(size_t)t * E + g] = acc;
        }
    }
    return 0;
}

/* Layer-wide top-k_t on the logits, Sec. 3.2.2.  The j-th pick is the largest
 * logit not yet picked; equal logits go to the smaller sub-expert id.  Unused
 * entries are -1. */
ORACLE_API int oracle_select(int T, int E, int k_max, const float *logits,
                             const int32_t *k_tok, int32_t *ids)
{
    if (k_max > E) return -1;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *l = logits + (size_t)t * E;
        int32_t *o = ids + (size_t)t * k_max;
        int kt = clamp_k(k_tok[t], k_max);
        char *taken = (char *)calloc((size_t)E, 1);
        for (int j = 0; j < k_max; ++j) o[j] = -1;
        for (int j = 0; j < kt; ++j) {
            int best = -1;
            for (int g = 0; g < E; ++g) {
                if (taken[g]) continue;
                if (best < 0 || l[g] > l[best]) best = g;
            }
            taken[best] = 1;
            o[j] = best;
        }
        free(taken);
    }
    return 0;
}

/* Routing weights, Sec. 3.2.2: softmax of the logits, either over all E
 * sub-experts (renormalize = 0) or over the k_t chosen ones (renormalize = 1),
 * times the routed scale.  Unused entries are 0. */
ORACLE_API int oracle_weights(int T, int E, int k_max, const float *logits,
                              const int32_t *ids, const int32_t *k_tok, int renormalize,
                              double routed_scale, double *w)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *l = logits + (size_t)t * E;
        const int32_t *id = ids + (size_t)t * k_max;
        double *o = w + (size_t)t * k_max;
        int kt = clamp_k(k_tok[t], k_max);
        double m = (double)l[0];
        for (int g = 1; g < E; ++g) if ((double)l[g] > m) m = (double)l[g];
        double denom = 0.0;
        if (renormalize) {
            for (int j = 0; j < kt; ++j) denom += exp((double)l[id[j]] - m);
        } else {
            for (int g = 0; g < E; ++g) denom += exp((double)l[g] - m);
        }
        for (int j = 0; j < k_max; ++j)
            o[j] = j < kt ? routed_scale * exp((double)l[id[j]] - m) / denom : 0.0;
    }
    return 0;
}

/* Dispatch: the token-sub-expert assignments (Sec. 2.1) grouped by sub-expert.
 * A pair is named t*k_max + j.  Pairs are visited token-ascending, pick-ascending
 * and appended to their sub-expert's group; since a token picks a sub-expert at
 * most once, every group lists its tokens in ascending order.  cnt[E], off[E+1]
 * (exclusive prefix, off[E] = number of pairs), sorted_pair[T*k_max] (slot ->
 * pair), slot_of_pair[T*k_max] (pair -> slot); unused entries are -1. */
ORACLE_API int oracle_dispatch(int T, int E, int k_max, const int32_t *ids, int32_t *cnt,
                               int32_t *off, int32_t *sorted_pair, int32_t *slot_of_pair)
{
    size_t n = (size_t)T * k_max;
    for (int g = 0; g < E; ++g) cnt[g] = 0;
    for (size_t p = 0; p < n; ++p) {
        if (ids[p] >= E) return -1;
        if (ids[p] >= 0) cnt[ids[p]]++;
    }
    off[0] = 0;
    for (int g = 0; g < E; ++g) off[g + 1] = off[g] + cnt[g];
    int32_t *fill = (int32_t *)calloc((size_t)E, sizeof(int32_t));
    for (size_t p = 0; p < n; ++p) { sorted_pair[p] = -1; slot_of_pair[p] = -1; }
    for (size_t p = 0; p < n; ++p) {
        int g = ids[p];
        if (g < 0) continue;
        int32_t slot = off[g] + fill[g]++;
        sorted_pair[slot] = (int32_t)p;
        slot_of_pair[p] = slot;
    }
    free(fill);
    return 0;
}

/* One sub-expert applied to one token, Eq. 1-2 restricted to the sub-expert's
 * neurons (Eq. 3):  a_c = x . Wg[c,:],  u_c = x . Wu[c,:],
 * h_c = SiLU(a_c) * u_c,  y[q] = sum_c h_c * Wd[q,c].
 * w_gu is [2*Is, d] (gate rows first, then up rows); w_dn is [d, Is]. */
static void ffn_one(int d, int Is, const float *x, const float *w_gu, const float *w_dn,
                    double *h, double *y)
{
    for (int c = 0; c < Is; ++c) {
        const float *wg = w_gu + (size_t)c * d;
        const float *wu = w_gu + (size_t)(Is + c) * d;
        double a = 0.0, u = 0.0;
        for (int j = 0; j < d; ++j) {
            a += (double)x[j] * (double)wg[j];
            u += (double)x[j] * (double)wu[j];
        }
        h[c] = a / (1.0 + exp(-a)) * u;
    }
    for (int q = 0; q < d; ++q) {
        const float *wd = w_dn + (size_t)q * Is;
        double s = 0.0;
        for (int c = 0; c < Is; ++c) s += h[c] * (double)wd[c];
        y[q] = s;
    }
}

ORACLE_API int oracle_ffn_one(int d, int Is, const float *x, const float *w_gu,
                              const float *w_dn, double *y)
{
    double *h = (double *)malloc(sizeof(double) * (size_t)Is);
    ffn_one(d, Is, x, w_gu, w_dn, h, y);
    free(h);
    return 0;
}

/* Grouped FFN: row p of y (p < off[E]) is the sub-expert of slot p's group
 * applied to slot p's token.  Rows >= off[E] are left untouched. */
ORACLE_API int oracle_grouped_ffn(int T, int d, int E, int Is, int k_max, const float *x,
                                  const float *w_gu, const float *w_dn, const int32_t *off,
                                  const int32_t *sorted_pair, double *y)
{
    (void)T;
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)Is);
#pragma omp for schedule(dynamic, 4)
        for (int p = 0; p < off[E]; ++p) {
            int g = 0;
            while (off[g + 1] <= p) ++g;
            int t = sorted_pair[p] / k_max;
            ffn_one(d, Is, x + (size_t)t * d, w_gu + (size_t)g * 2 * Is * d,
                    w_dn + (size_t)g * d * Is, h, y + (size_t)p * d);
        }
        free(h);
    }
    return 0;
}

/* Combine, Sec. 3.2.2: out[t,:] = sum_{j<k_t} w[t,j] * y[slot(t,j),:], j ascending. */
ORACLE_API int oracle_combine(int T, int d, int k_max, const double *y,
                              const int32_t *slot_of_pair, const double *w,
                              const int32_t *k_tok, double *out)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        int kt = clamp_k(k_tok[t], k_max);
        double *o = out + (size_t)t * d;
        for (int q = 0; q < d; ++q) o[q] = 0.0;
        for (int j = 0; j < kt; ++j) {
            const double *yr = y + (size_t)slot_of_pair[(size_t)t * k_max + j] * d;
            double wj = w[(size_t)t * k_max + j];
            for (int q = 0; q < d; ++q) o[q] += wj * yr[q];
        }
    }
    return 0;
}

/* The layer for a chosen set of tokens: the same steps, token by token, without
 * building the dispatch tables (a token's output does not depend on any other
 * token).  out is [n_sel, d]; ids_out / w_out ([n_sel, k_max]) may be NULL. */
ORACLE_API int oracle_layer_tokens(int n_sel, const int32_t *tokens, int d, int E, int Is,
                                   int k_max, int renormalize, double routed_scale,
                                   const float *x, const float *w_r, const float *bias,
                                   const int32_t *k_tok, const float *w_gu, const float *w_dn,
                                   double *out, int32_t *ids_out, double *w_out)
{
    if (k_max > E) return -1;
    int rc = 0;
#pragma omp parallel
    {
        float *l = (float *)malloc(sizeof(float) * (size_t)E);
        int32_t *id = (int32_t *)malloc(sizeof(int32_t) * (size_t)k_max);
        double *w = (double *)malloc(sizeof(double) * (size_t)k_max);
        double *h = (double *)malloc(sizeof(double) * (size_t)Is);
        double *y = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n_sel; ++i) {
            int t = tokens[i];
            const float *xr = x + (size_t)t * d;
            oracle_logits(1, d, E, xr, w_r, bias, l);
            if (oracle_select(1, E, k_max, l, k_tok + t, id)) rc = -1;
            oracle_weights(1, E, k_max, l, id, k_tok + t, renormalize, routed_scale, w);
            int kt = clamp_k(k_tok[t], k_max);
            double *o = out + (size_t)i * d;
            for (int q = 0; q < d; ++q) o[q] = 0.0;
            for (int j = 0; j < kt; ++j) {
                int g = id[j];
                ffn_one(d, Is, xr, w_gu + (size_t)g * 2 * Is * d, w_dn + (size_t)g * d * Is,
                        h, y);
                for (int q = 0; q < d; ++q) o[q] += w[j] * y[q];
            }
            if (ids_out) memcpy(ids_out + (size_t)i * k_max, id, sizeof(int32_t) * (size_t)k_max);
            if (w_out) memcpy(w_out + (size_t)i * k_max, w, sizeof(double) * (size_t)k_max);
        }
        free(l); free(id); free(w); free(h); free(y);
    }
    return rc;
}

/* ------------------------------------------------------------------------
 * Training-free proxy gating ("complex gate"), Sec. 3.2.2.
 *
 * The pre-existing router scores the N original experts and takes its native
 * top m (oracle_logits / oracle_select / oracle_weights with E = N, k = m).
 * For a token routed to original expert e, sub-expert n of e is scored by the
 * mean absolute activation of its r gate neurons,
 *     s_n(x) = (1/r) sum_{c in G_n} | SiLU(x . Wg[c,:]) * (x . Wu[c,:]) |,
 * and among the S sub-experts of the expert ranked j the top kappa_j by s are
 * executed, where (kappa_1..kappa_m) is the configured split of the token's
 * budget k.  Every selected sub-expert inherits the weight of its expert.
 *
 * w_proxy holds, per original expert, the gate rows of its S*r gate neurons
 * (sub-expert-major: neuron c of sub-expert n at row n*r + c) followed by
 * their up rows: [N][2*S*r][d].  Scores are binary64.
 * ------------------------------------------------------------------------ */
ORACLE_API int oracle_proxy_scores(int T, int d, int S, int r, int m, const float *x,
                                   const float *w_proxy, const int32_t *ids0, double *scores)
{
    const int R = S * r;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *xr = x + (size_t)t * d;
        for (int j = 0; j < m; ++j) {
            int e = ids0[(size_t)t * m + j];
            double *s = scores + ((size_t)t * m + j) * S;
            for (int n = 0; n < S; ++n) s[n] = 0.0;
            if (e < 0) continue;
            const float *wg = w_proxy + (size_t)e * 2 * R * d;
            const float *wu = wg + (size_t)R * d;
            for (int n = 0; n < S; ++n) {
                double sum = 0.0;
                for (int c = 0; c < r; ++c) {
                    const float *g = wg + (size_t)(n * r + c) * d;
                    const float *u = wu + (size_t)(n * r + c) * d;
                    double a = 0.0, b = 0.0;
                    for (int i = 0; i < d; ++i) {
                        a += (double)xr[i] * (double)g[i];
                        b += (double)xr[i] * (double)u[i];
                    }
                    sum += fabs(a / (1.0 + exp(-a)) * b);
                }
                s[n] = sum / (double)r;
            }
        }
    }
    return 0;
}

/* Per expert rank j: the kappa[k_t][j] best-scored sub-experts of expert
 * ids0[t,j] (score descending, equal scores to the smaller index), appended in
 * rank order; flat sub-expert id e*S + n; weight w0[t,j].  kappa is
 * [(k_cap+1)][m]; budgets are clamped to [0, min(k_max, k_cap)]. */
ORACLE_API int oracle_proxy_select(int T, int S, int m, int k_max, int k_cap,
                                   const double *scores, const int32_t *ids0, const double *w0,
                                   const int32_t *k_tok, const int32_t *kappa, int32_t *ids,
                                   double *w)
{
    int rc = 0;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        int kt = clamp_k(k_tok[t], k_max < k_cap ? k_max : k_cap);
        int32_t *o = ids + (size_t)t * k_max;
        double *ow = w + (size_t)t * k_max;
        for (int i = 0; i < k_max; ++i) { o[i] = -1; ow[i] = 0.0; }
        int pos = 0;
        for (int j = 0; j < m; ++j) {
            int kap = kappa[(size_t)kt * m + j];
            int e = ids0[(size_t)t * m + j];
            if (kap < 0 || kap > S) { rc = -1; continue; }
            if (e < 0) continue;
            const double *s = scores + ((size_t)t * m + j) * S;
            char taken[64] = {0};
            for (int i = 0; i < kap && pos < k_max; ++i) {
                int best = -1;
                for (int n = 0; n < S && n < 64; ++n) {
                    if (taken[n]) continue;
                    if (best < 0 || s[n] > s[best]) best = n;
                }
                taken[best] = 1;
                o[pos] = e * S + best;
                ow[pos] = w0[(size_t)t * m + j];
                ++pos;
            }
        }
    }
    return rc;
}
