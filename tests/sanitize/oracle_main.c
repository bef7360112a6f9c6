/*
 * Driver for a -fsanitize=address,undefined build of the CPU oracle
 * (oracle/moepp_oracle.c): calls every oracle function on small seeded inputs,
 * among them the awkward ones (first layer without residual, forced selection,
 * an expert nobody selects, a token list in arbitrary order, zero capacities),
 * and prints one checksum per output.  tests/test_sanitizers_cpu.py builds it
 * with the sanitizers, requires a clean run, and compares the checksums with
 * the ones the ordinary build gives through its Python front end.
 * Test infrastructure, like the oracle itself.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
    int32_t T, D, F, n_ffn, n_zero, n_copy, n_const, k;
} oracle_shape;

int moepp_oracle_route(const oracle_shape *, const float *, const float *, const float *,
                       const float *, const float *, const int32_t *, float *, double *, int32_t *,
                       float *);
int moepp_oracle_permute(const oracle_shape *, const int32_t *, int32_t *, int32_t *, int32_t *,
                         int32_t *);
int moepp_oracle_capacity(const oracle_shape *, double, double, int32_t, int32_t *);
int moepp_oracle_permute_capacity(const oracle_shape *, const int32_t *, const int32_t *, int32_t *,
                                  int32_t *, int32_t *, int32_t *, int32_t *);
int moepp_oracle_balance(const oracle_shape *, const double *, const int32_t *, double, double *,
                         double *, double *);
int moepp_oracle_experts(const oracle_shape *, const float *, const int32_t *, const float *,
                         const float *, const float *, const float *, const float *, const float *,
                         const int32_t *, int32_t, const int32_t *, double *, double *, double *,
                         double *);
int moepp_oracle_dense(const oracle_shape *, const float *, const double *, const float *,
                       const float *, const float *, const float *, const float *, double *);

/* 64-bit linear congruential generator; value = top 24 bits mapped to [-1, 1) */
static uint64_t g_state;
static float next_unit(void)
{
    g_state = g_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (float)((double)(g_state >> 40) / 8388608.0 - 1.0);
}
static float *fill(size_t n, float scale)
{
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i)
        p[i] = scale * next_unit();
    return p;
}
static void sum_f(const char *name, const float *p, size_t n)
{
    double s = 0.0;
    for (size_t i = 0; i < n; ++i)
        s += (double)p[i] * (double)(1 + i % 7);
    printf("%s %.17g\n", name, s);
}
static void sum_d(const char *name, const double *p, size_t n)
{
    double s = 0.0;
    for (size_t i = 0; i < n; ++i)
        s += p[i] * (double)(1 + i % 7);
    printf("%s %.17g\n", name, s);
}
static void sum_i(const char *name, const int32_t *p, size_t n)
{
    long long s = 0;
    for (size_t i = 0; i < n; ++i)
        s += (long long)p[i] * (long long)(1 + i % 7);
    printf("%s %lld\n", name, s);
}

int main(void)
{
    const oracle_shape s = {37, 24, 16, 5, 1, 1, 2, 3};
    const int N = 9, T = s.T, K = s.k, D = s.D, F = s.F;
    g_state = 20241007ULL;
    float *x = fill((size_t)T * D, 1.0f);
    float *prev = fill((size_t)T * N, 1.0f);
    float *W_g = fill((size_t)N * D, 0.2f);
    float *W_res = fill((size_t)N * N, 0.2f);
    float *bias = fill(N, 0.5f);
    float *w1 = fill((size_t)s.n_ffn * F * D, 0.2f);
    float *w3 = fill((size_t)s.n_ffn * F * D, 0.2f);
    float *w2 = fill((size_t)s.n_ffn * D * F, 0.2f);
    float *cv = fill((size_t)s.n_const * D, 0.2f);
    float *W_c = fill((size_t)s.n_const * 2 * D, 0.2f);
    bias[2] = -100.0f;                       /* expert 2 is never selected: an empty group */

    float *gate = (float *)malloc(sizeof(float) * T * N);
    double *probs = (double *)malloc(sizeof(double) * T * N);
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * T * K);
    float *w = (float *)malloc(sizeof(float) * T * K);
    int rc = moepp_oracle_route(&s, x, prev, W_g, W_res, bias, NULL, gate, probs, idx, w);
    sum_f("route.out_gate", gate, (size_t)T * N);
    sum_d("route.probs", probs, (size_t)T * N);
    sum_i("route.topk_idx", idx, (size_t)T * K);
    sum_f("route.topk_w", w, (size_t)T * K);

    /* first layer (Eq.6, j = 1), no bias, no probabilities wanted */
    float *gate1 = (float *)malloc(sizeof(float) * T * N);
    int32_t *idx1 = (int32_t *)malloc(sizeof(int32_t) * T * K);
    float *w_1 = (float *)malloc(sizeof(float) * T * K);
    rc |= moepp_oracle_route(&s, x, NULL, W_g, NULL, NULL, NULL, gate1, NULL, idx1, w_1);
    sum_f("first.out_gate", gate1, (size_t)T * N);
    sum_i("first.topk_idx", idx1, (size_t)T * K);
    /* the first layer's selection forced onto the second call */
    float *w_f = (float *)malloc(sizeof(float) * T * K);
    int32_t *idx_f = (int32_t *)malloc(sizeof(int32_t) * T * K);
    rc |= moepp_oracle_route(&s, x, prev, W_g, W_res, bias, idx1, gate, NULL, idx_f, w_f);
    sum_i("forced.topk_idx", idx_f, (size_t)T * K);
    sum_f("forced.topk_w", w_f, (size_t)T * K);

    int32_t *counts = (int32_t *)malloc(sizeof(int32_t) * N);
    int32_t *kept = (int32_t *)malloc(sizeof(int32_t) * N);
    int32_t *offs = (int32_t *)malloc(sizeof(int32_t) * (s.n_ffn + 1));
    int32_t *row_of = (int32_t *)malloc(sizeof(int32_t) * T * K);
    int32_t *src_of = (int32_t *)malloc(sizeof(int32_t) * T * K);
    rc |= moepp_oracle_permute(&s, idx, counts, offs, row_of, src_of);
    sum_i("permute.counts", counts, N);
    sum_i("permute.offsets", offs, s.n_ffn + 1);
    sum_i("permute.row_of", row_of, (size_t)T * K);
    sum_i("permute.src_of", src_of, offs[s.n_ffn]);

    int32_t cap[9];
    rc |= moepp_oracle_capacity(&s, 1.1, 0.75, 1, cap);
    sum_i("capacity.assignments", cap, N);
    rc |= moepp_oracle_capacity(&s, 1.1, 0.75, 0, cap);
    sum_i("capacity.tokens", cap, N);
    cap[0] = 0;                                  /* an expert that keeps nothing */
    rc |= moepp_oracle_permute_capacity(&s, idx, cap, counts, kept, offs, row_of, src_of);
    sum_i("cap.kept", kept, N);
    sum_i("cap.offsets", offs, s.n_ffn + 1);
    sum_i("cap.row_of", row_of, (size_t)T * K);
    sum_i("cap.src_of", src_of, offs[s.n_ffn]);

    double *f = (double *)malloc(sizeof(double) * N);
    double *P = (double *)malloc(sizeof(double) * N);
    double loss = 0.0;
    rc |= moepp_oracle_balance(&s, probs, idx, 0.75, f, P, &loss);
    sum_d("balance.f", f, N);
    sum_d("balance.P", P, N);
    printf("balance.loss %.17g\n", loss);

    /* experts: a token list in arbitrary order with a repeat, dropped slots honoured */
    const int32_t toks[6] = {36, 0, 17, 17, 5, 30};
    double *out = (double *)malloc(sizeof(double) * 6 * D);
    double *slots = (double *)calloc((size_t)6 * K * D, sizeof(double));
    double *h = (double *)calloc((size_t)6 * K * F, sizeof(double));
    double *a1 = (double *)calloc((size_t)6 * s.n_const, sizeof(double));
    rc |= moepp_oracle_experts(&s, x, idx, w, w1, w3, w2, cv, W_c, row_of, 6, toks, out, slots, h, a1);
    sum_d("experts.out", out, (size_t)6 * D);
    sum_d("experts.slot_out", slots, (size_t)6 * K * D);
    sum_d("experts.h", h, (size_t)6 * K * F);
    sum_d("experts.alpha1", a1, (size_t)6 * s.n_const);
    /* all tokens, nothing optional */
    double *out_all = (double *)malloc(sizeof(double) * T * D);
    rc |= moepp_oracle_experts(&s, x, idx, w, w1, w3, w2, cv, W_c, NULL, T, NULL, out_all, NULL, NULL,
                               NULL);
    sum_d("experts.out_all", out_all, (size_t)T * D);
    /* a token index out of range is refused, not read */
    const int32_t bad_tok[2] = {3, 37};
    printf("experts.bad_token %d\n",
           moepp_oracle_experts(&s, x, idx, w, w1, w3, w2, cv, W_c, NULL, 2, bad_tok, out, NULL, NULL, NULL));

    /* Eq.1 literally, with the masked gate vector of the routing above */
    double *gv = (double *)calloc((size_t)T * N, sizeof(double));
    for (int t = 0; t < T; ++t)
        for (int sl = 0; sl < K; ++sl)
            gv[t * N + idx[t * K + sl]] = (double)w[t * K + sl];
    double *dense = (double *)malloc(sizeof(double) * T * D);
    rc |= moepp_oracle_dense(&s, x, gv, w1, w3, w2, cv, W_c, dense);
    sum_d("dense.out", dense, (size_t)T * D);
    printf("status %d\n", rc);

    free(x); free(prev); free(W_g); free(W_res); free(bias); free(w1); free(w3); free(w2);
    free(cv); free(W_c); free(gate); free(probs); free(idx); free(w); free(gate1); free(idx1);
    free(w_1); free(w_f); free(idx_f); free(counts); free(kept); free(offs); free(row_of);
    free(src_of); free(f); free(P); free(out); free(slots); free(h); free(a1); free(out_all);
    free(gv); free(dense);
    return rc;
}
