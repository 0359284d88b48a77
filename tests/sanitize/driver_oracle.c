/* Runs every routine of the C oracle on small seeded inputs held in exactly sized heap buffers, so that a build with
 * -fsanitize=address,undefined reports any access outside them and any undefined arithmetic.  Exit code 0 = clean. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_router_logits(int T, int H, int E, const float *x, const float *w_router, const float *bias, float *logits);
int oracle_topk_from_logits(int T, int E, int K, int renormalize, const float *logits, int32_t *idx, float *w);
int oracle_route_topk(int T, int H, int E, int K, int renormalize, const float *x, const float *w_router, const float *bias,
                      int32_t *idx, float *w);
int oracle_permute(int n, int E, const int32_t *idx, int32_t *off, int32_t *row_to_assign, int32_t *assign_to_row);
int oracle_gather_rows(int n, int K, int H, const float *x, const int32_t *row_to_assign, float *x_perm);
int oracle_grouped_swiglu(int n, int H, int E, int I, const float *x_perm, const int32_t *off, const float *w_gate,
                          const float *w_up, const float *w_down, double *y_perm);
int oracle_combine(int T, int H, int K, const double *y_perm, const int32_t *assign_to_row, const float *w, double *out);
int oracle_forward(int T, int H, int E, int K, int I, int renormalize, const float *x, const float *w_router, const float *bias,
                   const float *w_gate, const float *w_up, const float *w_down, double *out, int32_t *idx_out, float *w_out);
int oracle_forward_tokens(int H, int K, int I, const float *x, const int32_t *idx, const float *w, const float *w_gate,
                          const float *w_up, const float *w_down, int n_tokens, const int32_t *tokens, double *out_rows);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static float draw(float scale) {      /* a small linear congruential generator: values in (-scale, scale) */
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return scale * ((float)((state >> 40) & 0xFFFFFF) / 8388608.0f - 1.0f);
}
static float *rand_floats(size_t n, float scale) {
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = draw(scale);
    return p;
}
#define CHECK(call) do { int rc_ = (call); if (rc_ != 0) { fprintf(stderr, "%s -> %d\n", #call, rc_); return 1; } } while (0)

static int one_shape(int T, int H, int E, int K, int I, int renorm, int with_bias) {
    size_t n = (size_t)T * K;
    float *x = rand_floats((size_t)T * H, 1.0f), *wr = rand_floats((size_t)E * H, 0.1f);
    float *bias = with_bias ? rand_floats((size_t)E, 0.5f) : NULL;
    float *wg = rand_floats((size_t)E * I * H, 0.1f), *wu = rand_floats((size_t)E * I * H, 0.1f), *wd = rand_floats((size_t)E * H * I, 0.1f);
    float *logits = (float *)malloc(sizeof(float) * ((size_t)T * E + 1));
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (n + 1)), *idx2 = (int32_t *)malloc(sizeof(int32_t) * (n + 1));
    float *w = (float *)malloc(sizeof(float) * (n + 1)), *w2 = (float *)malloc(sizeof(float) * (n + 1));
    int32_t *off = (int32_t *)malloc(sizeof(int32_t) * ((size_t)E + 1));
    int32_t *r2a = (int32_t *)malloc(sizeof(int32_t) * (n + 1)), *a2r = (int32_t *)malloc(sizeof(int32_t) * (n + 1));
    float *xp = (float *)malloc(sizeof(float) * (n * H + 1));
    double *yp = (double *)malloc(sizeof(double) * (n * H + 1));
    double *out = (double *)malloc(sizeof(double) * ((size_t)T * H + 1)), *out2 = (double *)malloc(sizeof(double) * ((size_t)T * H + 1));
    CHECK(oracle_router_logits(T, H, E, x, wr, bias, logits));
    CHECK(oracle_topk_from_logits(T, E, K, renorm, logits, idx, w));
    CHECK(oracle_route_topk(T, H, E, K, renorm, x, wr, bias, idx2, w2));
    if (memcmp(idx, idx2, sizeof(int32_t) * n) != 0) { fprintf(stderr, "routing differs between the two routes to it\n"); return 1; }
    CHECK(oracle_permute((int)n, E, idx, off, r2a, a2r));
    CHECK(oracle_gather_rows((int)n, K, H, x, r2a, xp));
    CHECK(oracle_grouped_swiglu((int)n, H, E, I, xp, off, wg, wu, wd, yp));
    CHECK(oracle_combine(T, H, K, yp, a2r, w, out));
    CHECK(oracle_forward(T, H, E, K, I, renorm, x, wr, bias, wg, wu, wd, out2, idx2, w2));
    for (size_t i = 0; i < (size_t)T * H; ++i)
        if (out[i] != out2[i]) { fprintf(stderr, "forward differs from its steps at %zu\n", i); return 1; }
    if (T > 0) {
        int32_t tokens[3] = {0, T - 1, T / 2};
        double *rows = (double *)malloc(sizeof(double) * 3 * (size_t)H);
        CHECK(oracle_forward_tokens(H, K, I, x, idx, w, wg, wu, wd, 3, tokens, rows));
        free(rows);
    }
    free(x); free(wr); free(bias); free(wg); free(wu); free(wd); free(logits); free(idx); free(idx2); free(w); free(w2);
    free(off); free(r2a); free(a2r); free(xp); free(yp); free(out); free(out2);
    return 0;
}

int main(void) {
    static const int shapes[][7] = {      /* T, H, E, K, I, renormalize, bias */
        {7, 16, 4, 2, 8, 1, 0}, {1, 8, 1, 1, 8, 1, 1}, {33, 24, 9, 9, 16, 0, 1}, {64, 32, 70, 3, 8, 1, 0},
        {0, 8, 4, 2, 8, 1, 0}, {5, 8, 300, 7, 8, 0, 0}, {40, 40, 6, 1, 24, 1, 1},
    };
    for (size_t i = 0; i < sizeof(shapes) / sizeof(shapes[0]); ++i)
        if (one_shape(shapes[i][0], shapes[i][1], shapes[i][2], shapes[i][3], shapes[i][4], shapes[i][5], shapes[i][6])) return 1;
    puts("oracle clean under the sanitizers");
    return 0;
}
