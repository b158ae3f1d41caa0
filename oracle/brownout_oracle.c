/*
 * brownout_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step CPU statement of what one BrownoutMoE layer
 * computes, written from the paper (BrownoutServe, arXiv 2507.17133).  It
 * exists to check the GPU library and to be timed as a CPU baseline.  It shares
 * no code with the GPU path and nothing in the product may call it.
 *
 * Precision: all inputs are float arrays (callers that test a bf16 GPU path
 * round the values to bf16 first and widen them, so both sides start from the
 * same numbers).  Every sum is accumulated in double.  Gate logits are rounded
 * to float once and the top-K decision is taken on those floats (the GPU takes
 * it on its own fp32 logits); the double logits are kept to measure how close
 * each decision was.
 *
 * Layouts (row-major everywhere):
 *   x        [T][d]
 *   gate_w   [m][d]      row i is the centroid e_i of expert i
 *   w1, w3   [n][F][d]   "gate" and "up" projections of n experts
 *   w2       [n][d][F]   "down" projection
 *
 * No blocking, fusion or reordering beyond what each definition states.
 * OpenMP only parallelises the outermost independent loop (tokens / rows).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- */
/* Affinity s_{i,t} = x_t^T e_i  (Architecture of BrownoutMoE, last equation), */
/* plus an optional per-expert bias used only by the synthetic skewed-load     */
/* workloads.  s64 keeps the double value, s32 the float the decision uses.    */
/* ------------------------------------------------------------------------- */
void oracle_gate_logits(const float *x, int T, int d, const float *gate_w,
                        const float *gate_bias, int m, double *s64, float *s32)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int i = 0; i < m; ++i) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c)
                acc += (double)x[(size_t)t * d + c] * (double)gate_w[(size_t)i * d + c];
            if (gate_bias) acc += (double)gate_bias[i];
            s64[(size_t)t * m + i] = acc;
            s32[(size_t)t * m + i] = (float)acc;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* TopK(.,K) and g_{i,t} (Architecture of BrownoutMoE, the g equation): the K  */
/* highest affinities of a token, listed by descending score (equal scores:    */
/* lower expert index first), and their weights:                               */
/*   score_fn 0: exp(s_i) / sum_{j in TopK} exp(s_j)                           */
/*   score_fn 1: sigmoid(s_i) / sum_{j in TopK} sigmoid(s_j)  (selection is on */
/*               s itself, sigmoid being monotone)                             */
/* margin[t] = the smallest gap, measured on the double logits, between        */
/* neighbours in the list "K winners followed by the best loser".  A small or  */
/* negative margin marks a decision that fp32 summation order could flip.      */
/* ------------------------------------------------------------------------- */
void oracle_topk(const double *s64, const float *s32, int T, int m, int K, int score_fn,
                 int32_t *topk_idx, float *topk_w, double *margin)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *s = s32 + (size_t)t * m;
        const double *sd = s64 + (size_t)t * m;
        int32_t *idx = topk_idx + (size_t)t * K;
        char *taken = (char *)calloc((size_t)m, 1);
        for (int j = 0; j < K; ++j) {
            int best = -1;
            for (int i = 0; i < m; ++i) {
                if (taken[i]) continue;
                if (best < 0 || s[i] > s[best]) best = i; /* strict: ties keep the lower index */
            }
            taken[best] = 1;
            idx[j] = best;
        }
        /* the best expert that was not selected, if any */
        int loser = -1;
        for (int i = 0; i < m; ++i) {
            if (taken[i]) continue;
            if (loser < 0 || s[i] > s[loser]) loser = i;
        }
        double mg = INFINITY;
        for (int j = 0; j + 1 < K; ++j) {
            double g = sd[idx[j]] - sd[idx[j + 1]];
            if (g < mg) mg = g;
        }
        if (loser >= 0) {
            double g = sd[idx[K - 1]] - sd[loser];
            if (g < mg) mg = g;
        }
        if (margin) margin[t] = mg;

        double num[64];
        double *nump = (K <= 64) ? num : (double *)malloc(sizeof(double) * (size_t)K);
        double den = 0.0;
        if (score_fn == 0) {
            double mx = (double)s[idx[0]];
            for (int j = 0; j < K; ++j) { nump[j] = exp((double)s[idx[j]] - mx); den += nump[j]; }
        } else {
            for (int j = 0; j < K; ++j) { nump[j] = 1.0 / (1.0 + exp(-(double)s[idx[j]])); den += nump[j]; }
        }
        for (int j = 0; j < K; ++j) topk_w[(size_t)t * K + j] = (float)(nump[j] / den);
        if (nump != num) free(nump);
        free(taken);
    }
}

/* cnt_i = number of tokens that list expert i in their TopK (input of Algorithm 1). */
void oracle_expert_counts(const int32_t *topk_idx, int T, int K, int m, int32_t *cnt)
{
    for (int i = 0; i < m; ++i) cnt[i] = 0;
    for (size_t r = 0; r < (size_t)T * K; ++r) cnt[topk_idx[r]] += 1;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 (BrownoutMoE), the split into S1 / S2 and the grouping of S2,   */
/* read so that it reproduces the worked examples of the Brownout Approach     */
/* section (the printed test on sum_partial cannot: it would send the most     */
/* loaded expert to S2):                                                       */
/*   - experts sorted by cnt descending, equal counts by ascending id;         */
/*   - Tthr = S * threshold with S = sum cnt (threshold is a double, so that   */
/*     20 * 0.6 is exactly 12 as in the worked example);                       */
/*   - walking the sorted list with P = tokens already covered, an expert      */
/*     joins S1 while P < Tthr; the rest form S2 (partial) or are dropped      */
/*     (full brownout);                                                        */
/*   - S2 is grouped by floor(id / way); a group whose S2 members that hold    */
/*     tokens number exactly one is served by that expert itself (special      */
/*     case), a group with two or more goes to united expert g.                */
/* Outputs: in_s1[i] in {0,1}; unit[i] = i (served by itself), m+g (united     */
/* expert g) or -1 (dropped).  Experts without tokens keep unit[i] = i.        */
/* ------------------------------------------------------------------------- */
void oracle_brownout_decide(const int32_t *cnt, int m, int way, double threshold,
                            int use_full_brownout, int32_t *unit, uint8_t *in_s1)
{
    int *order = (int *)malloc(sizeof(int) * (size_t)m);
    for (int i = 0; i < m; ++i) order[i] = i;
    /* stable insertion sort, descending count */
    for (int a = 1; a < m; ++a) {
        int e = order[a], b = a - 1;
        while (b >= 0 && cnt[order[b]] < cnt[e]) { order[b + 1] = order[b]; --b; }
        order[b + 1] = e;
    }
    long long S = 0;
    for (int i = 0; i < m; ++i) S += cnt[i];
    const double Tthr = (double)S * threshold; /* one double product, as a Python float would give */

    long long sum_partial = 0;
    for (int a = 0; a < m; ++a) {
        int e = order[a];
        in_s1[e] = ((double)sum_partial < Tthr) ? 1 : 0;
        sum_partial += cnt[e];
    }
    const int G = (m + way - 1) / way;
    for (int i = 0; i < m; ++i) unit[i] = i;
    for (int g = 0; g < G; ++g) {
        int lo = g * way, hi = lo + way < m ? lo + way : m;
        int members = 0;
        for (int i = lo; i < hi; ++i)
            if (!in_s1[i] && cnt[i] > 0) ++members;
        for (int i = lo; i < hi; ++i) {
            if (in_s1[i] || cnt[i] == 0) continue;
            if (use_full_brownout) unit[i] = -1;
            else if (members >= 2) unit[i] = m + g;
            /* members == 1: the expert serves its own tokens */
        }
    }
    free(order);
}

/* ------------------------------------------------------------------------- */
/* concat_tokens / process_tokens bookkeeping of Algorithm 1: the list of rows */
/* each execution unit receives.  Units are numbered 0..m-1 (original experts),*/
/* m..m+G-1 (united experts), m+G.. (shared experts, which take every token    */
/* with weight 1).  Within a unit rows are in ascending token order.  A token  */
/* whose TopK holds several experts delegated to the same united expert gives  */
/* that unit ONE row whose weight is the sum of those g (the layer equation    */
/* sums q_{i,t} over i on the same FFN output).                                */
/* token_rows[t][j], j < K: row of TopK entry j, or -1 if dropped or merged    */
/* into an earlier entry's row; j >= K: rows in the shared units.              */
/* Returns the number of rows R'.  Buffers sized for T*(K+n_shared) rows.      */
/* ------------------------------------------------------------------------- */
int32_t oracle_build_rows(const int32_t *topk_idx, const float *topk_w, int T, int K, int m, int way,
                          int n_shared, const int32_t *unit, int32_t *unit_cnt, int32_t *unit_off,
                          int32_t *row_token, float *row_weight, int32_t *token_rows)
{
    const int G = (m + way - 1) / way;
    const int U = m + G + n_shared;
    const int slots = K + n_shared;
    for (int u = 0; u < U; ++u) unit_cnt[u] = 0;
    /* pass 1: rows per unit */
    for (int t = 0; t < T; ++t) {
        for (int j = 0; j < K; ++j) {
            int u = unit[topk_idx[(size_t)t * K + j]];
            if (u < 0) continue;
            int dup = 0;
            for (int q = 0; q < j; ++q)
                if (unit[topk_idx[(size_t)t * K + q]] == u) dup = 1;
            if (!dup) unit_cnt[u] += 1;
        }
        for (int s = 0; s < n_shared; ++s) unit_cnt[m + G + s] += 1;
    }
    unit_off[0] = 0;
    for (int u = 0; u < U; ++u) unit_off[u + 1] = unit_off[u] + unit_cnt[u];
    /* pass 2: fill, ascending token inside each unit */
    int32_t *fill = (int32_t *)calloc((size_t)(U > 0 ? U : 1), sizeof(int32_t));
    for (int t = 0; t < T; ++t) {
        for (int j = 0; j < K; ++j) {
            token_rows[(size_t)t * slots + j] = -1;
            int u = unit[topk_idx[(size_t)t * K + j]];
            if (u < 0) continue;
            int first = -1;
            for (int q = 0; q < j; ++q)
                if (unit[topk_idx[(size_t)t * K + q]] == u) { first = q; break; }
            if (first >= 0) {
                int32_t r = token_rows[(size_t)t * slots + first];
                row_weight[r] = row_weight[r] + topk_w[(size_t)t * K + j]; /* float add, in j order */
            } else {
                int32_t r = unit_off[u] + fill[u]++;
                row_token[r] = t;
                row_weight[r] = topk_w[(size_t)t * K + j];
                token_rows[(size_t)t * slots + j] = r;
            }
        }
        for (int s = 0; s < n_shared; ++s) {
            int u = m + G + s;
            int32_t r = unit_off[u] + fill[u]++;
            row_token[r] = t;
            row_weight[r] = 1.0f;
            token_rows[(size_t)t * slots + K + s] = r;
        }
    }
    free(fill);
    return unit_off[U];
}

/* ------------------------------------------------------------------------- */
/* One expert FFN on n rows: FFN(x) = W2 ( silu(W1 x) * (W3 x) ),              */
/* silu(z) = z / (1 + exp(-z)).  (The paper writes FFN_i(x) without its        */
/* inside; SwiGLU is what the evaluated model families use.)                   */
/* w1, w3: [F][d], w2: [d][F] for this one expert.  y: [n][d] double.          */
/* ------------------------------------------------------------------------- */
static void ffn_row(const float *xr, int d, int F, const float *w1, const float *w3, const float *w2,
                    double *h, double *y)
{
    for (int f = 0; f < F; ++f) {
        double a = 0.0, b = 0.0;
        for (int c = 0; c < d; ++c) {
            a += (double)xr[c] * (double)w1[(size_t)f * d + c];
            b += (double)xr[c] * (double)w3[(size_t)f * d + c];
        }
        h[f] = (a / (1.0 + exp(-a))) * b;
    }
    for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int f = 0; f < F; ++f) acc += h[f] * (double)w2[(size_t)c * F + f];
        y[c] = acc;
    }
}

void oracle_ffn(const float *x, int n, int d, int F, const float *w1, const float *w3, const float *w2,
                double *y)
{
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)F);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n; ++r)
            ffn_row(x + (size_t)r * d, d, F, w1, w3, w2, h, y + (size_t)r * d);
        free(h);
    }
}

/* ------------------------------------------------------------------------- */
/* The layer equation (Architecture of BrownoutMoE, first equation):           */
/*   h_t = [x_t] + sum_s FFN^(s)_s(x_t) + sum_i p_{i,t} FFN^(r)_i(x_t)         */
/*                 + sum_i q_{i,t} FFN^(u)_{f(i)}(x_t),   f(i) = floor(i/way), */
/* p = g on experts served by themselves, q = g on experts delegated to their  */
/* united expert, both 0 for dropped experts (no renormalisation).  unit[] is  */
/* Algorithm 1's decision.  Evaluated token by token straight from the         */
/* equation (no permutation, no merging of rows).  tok_list (n_tok entries,    */
/* or NULL for all T tokens) selects which tokens to evaluate; out is          */
/* [n_tok][d] float.  Any weight pointer may be NULL if no token needs it.     */
/* ------------------------------------------------------------------------- */
void oracle_forward_tokens(const float *x, int T, int d, int F, int m, int K, int way,
                           const int32_t *topk_idx, const float *topk_w, const int32_t *unit,
                           const float *ew1, const float *ew3, const float *ew2,
                           const float *uw1, const float *uw3, const float *uw2,
                           int n_shared, int F_s, const float *sw1, const float *sw3, const float *sw2,
                           int add_residual, const int32_t *tok_list, int n_tok, float *out)
{
    (void)way;
    if (!tok_list) n_tok = T;
    const int Fmax = F > F_s ? F : F_s;
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)Fmax);
        double *y = (double *)malloc(sizeof(double) * (size_t)d);
        double *acc = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 1)
        for (int q = 0; q < n_tok; ++q) {
            const int t = tok_list ? tok_list[q] : q;
            const float *xr = x + (size_t)t * d;
            for (int c = 0; c < d; ++c) acc[c] = add_residual ? (double)xr[c] : 0.0;
            for (int s = 0; s < n_shared; ++s) {
                ffn_row(xr, d, F_s, sw1 + (size_t)s * F_s * d, sw3 + (size_t)s * F_s * d,
                        sw2 + (size_t)s * d * F_s, h, y);
                for (int c = 0; c < d; ++c) acc[c] += y[c];
            }
            for (int j = 0; j < K; ++j) {
                const int i = topk_idx[(size_t)t * K + j];
                const int u = unit[i];
                if (u < 0) continue;
                const double g = (double)topk_w[(size_t)t * K + j];
                if (u < m) {
                    ffn_row(xr, d, F, ew1 + (size_t)u * F * d, ew3 + (size_t)u * F * d,
                            ew2 + (size_t)u * d * F, h, y);
                } else {
                    const int gi = u - m;
                    ffn_row(xr, d, F, uw1 + (size_t)gi * F * d, uw3 + (size_t)gi * F * d,
                            uw2 + (size_t)gi * d * F, h, y);
                }
                for (int c = 0; c < d; ++c) acc[c] += g * y[c];
            }
            for (int c = 0; c < d; ++c) out[(size_t)q * d + c] = (float)acc[c];
        }
        free(h); free(y); free(acc);
    }
}

/* ------------------------------------------------------------------------- */
/* United experts (United Expert Model).  The paper trains one student per     */
/* group of `way` consecutive experts by distillation but gives no recipe;     */
/* this build's moe_build_united produces the student's starting point: the    */
/* element-wise mean of the group's parameters (last group: its actual         */
/* members).  n_elem = elements of one expert's tensor.  Sum in member order   */
/* in double, one division, result as double (the caller rounds).              */
/* ------------------------------------------------------------------------- */
void oracle_united_mean(const float *w, int m, int way, size_t n_elem, double *u)
{
    const int G = (m + way - 1) / way;
    for (int g = 0; g < G; ++g) {
        int lo = g * way, hi = lo + way < m ? lo + way : m;
#pragma omp parallel for schedule(static)
        for (size_t e = 0; e < n_elem; ++e) {
            double s = 0.0;
            for (int i = lo; i < hi; ++i) s += (double)w[(size_t)i * n_elem + e];
            u[(size_t)g * n_elem + e] = s / (double)(hi - lo);
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Distillation loss of group j (United Expert Model, the MSE equation):       */
/*   L^j = (1/k_j) sum_i || H_u^j - H_o^{j*way+i} ||^2                         */
/* with H = FFN outputs on n_calib calibration tokens, ||.||^2 summed over     */
/* features and averaged over the tokens, k_j = members of group j.            */
/* ------------------------------------------------------------------------- */
void oracle_united_loss(const float *calib_x, int n_calib, int d, int F, int m, int way,
                        const float *ew1, const float *ew3, const float *ew2,
                        const float *uw1, const float *uw3, const float *uw2, double *loss)
{
    const int G = (m + way - 1) / way;
    double *hu = (double *)malloc(sizeof(double) * (size_t)n_calib * d);
    double *ho = (double *)malloc(sizeof(double) * (size_t)n_calib * d);
    for (int g = 0; g < G; ++g) {
        int lo = g * way, hi = lo + way < m ? lo + way : m;
        oracle_ffn(calib_x, n_calib, d, F, uw1 + (size_t)g * F * d, uw3 + (size_t)g * F * d,
                   uw2 + (size_t)g * d * F, hu);
        double tot = 0.0;
        for (int i = lo; i < hi; ++i) {
            oracle_ffn(calib_x, n_calib, d, F, ew1 + (size_t)i * F * d, ew3 + (size_t)i * F * d,
                       ew2 + (size_t)i * d * F, ho);
            double s = 0.0;
            for (size_t e = 0; e < (size_t)n_calib * d; ++e) {
                double df = hu[e] - ho[e];
                s += df * df;
            }
            tot += s;
        }
        loss[g] = tot / (double)(hi - lo) / (double)n_calib;
    }
    free(hu); free(ho);
}
