/*
 * CPU oracle for the routed-expert mixture-of-experts FFN block.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against; nothing in the product path may call it.
 * It shares no code, header, table or helper with the GPU library.
 *
 * What it defines.  The paper trains a Qwen3-30B-A3B-class mixture-of-experts
 * policy (Section 4.1, "Training Details"); it names the model and says
 * nothing else about the layer, so the definition written out here is the
 * standard dropless top-K MoE with SwiGLU experts, with every free choice
 * fixed as follows (T tokens, H hidden, E experts, K experts per token,
 * I expert intermediate size; assignment id a = t*K + k):
 *
 *  logits    l[t,e] = fl32( sum_h x[t,h]*Wr[e,h] + b[e] ), the sum and the bias
 *            add carried in double, one rounding to float at the end.
 *  selection experts ordered by (logit descending, index ascending); the first
 *            K are the token's experts, slot 0 being the arg-max.
 *  weights   p_k = exp(l_k - l_0); renormalised: w_k = p_k / sum_{j<K} p_j
 *            (equal to the full softmax renormalised over the selected K);
 *            otherwise w_k = p_k / sum_{e<E} exp(l_e - l_0).  Evaluated in
 *            double, stored as float.
 *  permute   stable counting sort of the assignments by expert:
 *            off[e+1] = off[e] + #{a : idx[a] = e};  row(a) = off[idx[a]] +
 *            #{a' < a : idx[a'] = idx[a]}.
 *  expert    g_i = sum_h v_h*Wg[e,i,h];  u_i = sum_h v_h*Wu[e,i,h];
 *            a_i = g_i / (1 + exp(-g_i)) * u_i;  y_j = sum_i a_i*Wd[e,j,i].
 *            No biases, no shared expert, no capacity limit.
 *  combine   out[t,:] = sum_{k=0..K-1} w[t,k] * y[row(t*K+k),:], in k order.
 *
 * Arithmetic: inputs are float (bf16 inputs are widened exactly by the
 * caller); every sum, the SiLU and the combine are carried in double and no
 * intermediate is rounded to a narrower type.  y and out are returned as
 * double.  Loops over independent tokens / rows may run under OpenMP; no
 * arithmetic is blocked, fused or reordered.
 *
 * Parity pins (tests, CPU only): weights sum to one; permutation round trip
 * and stability; E=1,K=1 equals a dense SwiGLU MLP from library matmuls; K=E
 * equals the full softmax mixture; an independent dense brute force written in
 * another language; a hand-worked 2-expert example; all-equal logits tie-break;
 * zero input; power-of-two scaling.  The last ulp of the float weights is
 * parity unpinned (bounded by tolerance only).
 *
 * All functions return 0 on success, a negative number on bad arguments.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* logits[t,e] as defined above; logits is [T,E] float. */
int oracle_router_logits(int T, int H, int E, const float *x, const float *w_router,
                         const float *bias, float *logits)
{
    if (T < 0 || H < 1 || E < 1 || !x || !w_router || !logits) return -1;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            double s = 0.0;
            for (int h = 0; h < H; ++h)
                s += (double)x[(size_t)t * H + h] * (double)w_router[(size_t)e * H + h];
            if (bias) s += (double)bias[e];
            logits[(size_t)t * E + e] = (float)s;
        }
    }
    return 0;
}

/* Selection and weights from given logits. idx [T,K] int32, w [T,K] float. */
int oracle_topk_from_logits(int T, int E, int K, int renormalize, const float *logits,
                            int32_t *idx, float *w)
{
    if (T < 0 || E < 1 || K < 1 || K > E || !logits || !idx || !w) return -1;
    int rc = 0;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *l = logits + (size_t)t * E;
        unsigned char *taken = (unsigned char *)calloc((size_t)E, 1);
        if (!taken) { rc = -2; continue; }
        for (int k = 0; k < K; ++k) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                /* strictly greater: among equal logits the lower index stays */
                if (best < 0 || l[e] > l[best]) best = e;
            }
            taken[best] = 1;
            idx[(size_t)t * K + k] = best;
        }
        free(taken);
        double m = (double)l[idx[(size_t)t * K]];
        double denom = 0.0;
        if (renormalize) {
            for (int k = 0; k < K; ++k) denom += exp((double)l[idx[(size_t)t * K + k]] - m);
        } else {
            for (int e = 0; e < E; ++e) denom += exp((double)l[e] - m);
        }
        for (int k = 0; k < K; ++k)
            w[(size_t)t * K + k] = (float)(exp((double)l[idx[(size_t)t * K + k]] - m) / denom);
    }
    return rc;
}

int oracle_route_topk(int T, int H, int E, int K, int renormalize, const float *x,
                      const float *w_router, const float *bias, int32_t *idx, float *w)
{
    if (T < 0 || H < 1 || E < 1 || K < 1 || K > E) return -1;
    float *logits = (float *)malloc(sizeof(float) * (size_t)(T > 0 ? T : 1) * E);
    if (!logits) return -2;
    int rc = oracle_router_logits(T, H, E, x, w_router, bias, logits);
    if (rc == 0) rc = oracle_topk_from_logits(T, E, K, renormalize, logits, idx, w);
    free(logits);
    return rc;
}

/* Stable counting sort of the n = T*K assignments by expert.
 * off [E+1], row_to_assign [n], assign_to_row [n]. */
int oracle_permute(int n, int E, const int32_t *idx, int32_t *off, int32_t *row_to_assign,
                   int32_t *assign_to_row)
{
    if (n < 0 || E < 1 || !idx || !off || !row_to_assign || !assign_to_row) return -1;
    for (int e = 0; e <= E; ++e) off[e] = 0;
    for (int a = 0; a < n; ++a) {
        if (idx[a] < 0 || idx[a] >= E) return -3;
        off[idx[a] + 1] += 1;
    }
    for (int e = 0; e < E; ++e) off[e + 1] += off[e];
    int32_t *next = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    if (!next) return -2;
    memcpy(next, off, sizeof(int32_t) * (size_t)E);
    for (int a = 0; a < n; ++a) {
        int32_t r = next[idx[a]]++;
        row_to_assign[r] = a;
        assign_to_row[a] = r;
    }
    free(next);
    return 0;
}

/* x_perm[row(a),:] = x[a div K,:] */
int oracle_gather_rows(int n, int K, int H, const float *x, const int32_t *row_to_assign,
                       float *x_perm)
{
    if (n < 0 || K < 1 || H < 1 || !x || !row_to_assign || !x_perm) return -1;
    for (int r = 0; r < n; ++r)
        memcpy(x_perm + (size_t)r * H, x + (size_t)(row_to_assign[r] / K) * H, sizeof(float) * (size_t)H);
    return 0;
}

/* One expert applied to one input vector v[H]; y[H] double; scratch a[I]. */
static void expert_ffn(int H, int I, const float *v, const float *wg, const float *wu,
                       const float *wd, double *a, double *y)
{
    for (int i = 0; i < I; ++i) {
        double g = 0.0, u = 0.0;
        for (int h = 0; h < H; ++h) {
            g += (double)v[h] * (double)wg[(size_t)i * H + h];
            u += (double)v[h] * (double)wu[(size_t)i * H + h];
        }
        a[i] = g / (1.0 + exp(-g)) * u;
    }
    for (int j = 0; j < H; ++j) {
        double s = 0.0;
        for (int i = 0; i < I; ++i) s += a[i] * (double)wd[(size_t)j * I + i];
        y[j] = s;
    }
}

/* y_perm[r,:] = FFN_e(x_perm[r,:]) for r in [off[e], off[e+1]).  y_perm is [n,H] double. */
int oracle_grouped_swiglu(int n, int H, int E, int I, const float *x_perm, const int32_t *off,
                          const float *w_gate, const float *w_up, const float *w_down,
                          double *y_perm)
{
    if (n < 0 || H < 1 || E < 1 || I < 1 || !x_perm || !off || !w_gate || !w_up || !w_down || !y_perm)
        return -1;
    if (off[0] != 0 || off[E] != n) return -3;
    int32_t *row_expert = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    if (!row_expert) return -2;
    for (int e = 0; e < E; ++e)
        for (int r = off[e]; r < off[e + 1]; ++r) row_expert[r] = e;
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n; ++r) {
        int e = row_expert[r];
        double *a = (double *)malloc(sizeof(double) * (size_t)I);
        if (!a) { rc = -2; continue; }
        expert_ffn(H, I, x_perm + (size_t)r * H, w_gate + (size_t)e * I * H,
                   w_up + (size_t)e * I * H, w_down + (size_t)e * H * I, a, y_perm + (size_t)r * H);
        free(a);
    }
    free(row_expert);
    return rc;
}

/* out[t,:] = sum_k w[t,k] * y_perm[assign_to_row[t*K+k],:], k ascending. out [T,H] double. */
int oracle_combine(int T, int H, int K, const double *y_perm, const int32_t *assign_to_row,
                   const float *w, double *out)
{
    if (T < 0 || H < 1 || K < 1 || !y_perm || !assign_to_row || !w || !out) return -1;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int h = 0; h < H; ++h) {
            double s = 0.0;
            for (int k = 0; k < K; ++k)
                s += (double)w[(size_t)t * K + k] * y_perm[(size_t)assign_to_row[(size_t)t * K + k] * H + h];
            out[(size_t)t * H + h] = s;
        }
    }
    return 0;
}

/* The whole block, by composing the steps above.  Optional outputs may be NULL. */
int oracle_forward(int T, int H, int E, int K, int I, int renormalize, const float *x,
                   const float *w_router, const float *bias, const float *w_gate,
                   const float *w_up, const float *w_down, double *out, int32_t *idx_out,
                   float *w_out)
{
    if (T < 0 || H < 1 || E < 1 || K < 1 || K > E || I < 1 || !out) return -1;
    size_t n = (size_t)T * K, n1 = n ? n : 1;
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * n1);
    float *w = (float *)malloc(sizeof(float) * n1);
    int32_t *off = (int32_t *)malloc(sizeof(int32_t) * (size_t)(E + 1));
    int32_t *r2a = (int32_t *)malloc(sizeof(int32_t) * n1);
    int32_t *a2r = (int32_t *)malloc(sizeof(int32_t) * n1);
    float *xp = (float *)malloc(sizeof(float) * n1 * H);
    double *yp = (double *)malloc(sizeof(double) * n1 * H);
    int rc = (idx && w && off && r2a && a2r && xp && yp) ? 0 : -2;
    if (rc == 0) rc = oracle_route_topk(T, H, E, K, renormalize, x, w_router, bias, idx, w);
    if (rc == 0) rc = oracle_permute((int)n, E, idx, off, r2a, a2r);
    if (rc == 0) rc = oracle_gather_rows((int)n, K, H, x, r2a, xp);
    if (rc == 0) rc = oracle_grouped_swiglu((int)n, H, E, I, xp, off, w_gate, w_up, w_down, yp);
    if (rc == 0) rc = oracle_combine(T, H, K, yp, a2r, w, out);
    if (rc == 0 && idx_out) memcpy(idx_out, idx, sizeof(int32_t) * n);
    if (rc == 0 && w_out) memcpy(w_out, w, sizeof(float) * n);
    free(idx); free(w); free(off); free(r2a); free(a2r); free(xp); free(yp);
    return rc;
}

/* The block's output for a list of tokens only (for checking samples of a
 * large batch): out_rows[s,:] = out[tokens[s],:], given that batch's routing
 * (idx, w as produced by oracle_route_topk on the whole batch). */
int oracle_forward_tokens(int H, int K, int I, const float *x, const int32_t *idx, const float *w,
                          const float *w_gate, const float *w_up, const float *w_down,
                          int n_tokens, const int32_t *tokens, double *out_rows)
{
    if (H < 1 || K < 1 || I < 1 || n_tokens < 0 || !x || !idx || !w || !tokens || !out_rows) return -1;
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < n_tokens; ++s) {
        int t = tokens[s];
        double *a = (double *)malloc(sizeof(double) * (size_t)I);
        double *y = (double *)malloc(sizeof(double) * (size_t)H * K);
        if (!a || !y) { rc = -2; free(a); free(y); continue; }
        for (int k = 0; k < K; ++k) {
            int e = idx[(size_t)t * K + k];
            expert_ffn(H, I, x + (size_t)t * H, w_gate + (size_t)e * I * H, w_up + (size_t)e * I * H,
                       w_down + (size_t)e * H * I, a, y + (size_t)k * H);
        }
        for (int h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += (double)w[(size_t)t * K + k] * y[(size_t)k * H + h];
            out_rows[(size_t)s * H + h] = acc;
        }
        free(a); free(y);
    }
    return rc;
}
