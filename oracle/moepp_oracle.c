/*
 * CPU oracle for the forward pass of one MoE++ layer (arXiv 2410.07348).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the layer computes, written from the paper's equations; it exists so that
 * the HIP library can be checked against it.  It shares no code, header,
 * table or helper with the HIP path and must never be called from it.  Only
 * tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Every floating-point quantity is evaluated in fp64 from float32-typed
 * inputs (bf16 inputs are passed as the float32 numbers they represent), one
 * token at a time, one expert at a time, sums running in index order.  The
 * only parallelism is an OpenMP loop over tokens, which are independent.
 *
 * Notation (paper, Sec. 3): T tokens, D hidden size, N = N_FFN + N_ZC experts,
 * K experts activated per token.  Expert index order inside the N-way
 * softmax: FFN experts [0, n_ffn), then zero, copy, constant experts (the
 * order in which the model table, Tab.2, lists them; the paper fixes none).
 *
 * Readings where the paper is silent (all listed again in the design notes):
 *  - gate weights are the softmax over all N experts, not renormalised over
 *    the selected K (Eq.1 writes Softmax(G(x))_i);
 *  - Top-K is taken on the logits G(x) (Eq.1), ties go to the lower index,
 *    the selected slots are ordered by descending logit;
 *  - the "routing scores of the previous layer" in Eq.6 are G(x^{j-1}), the
 *    pre-softmax logits (with that layer's own residual included);
 *  - each constant expert owns its vector v and its 2 x D matrix W_c (Eq.5);
 *  - an FFN expert is a bias-free SwiGLU: W2 (silu(W1 x) * (W3 x));
 *  - logits are rounded once to float32 (the type they are handed to the
 *    next layer in) and softmax / Top-K read those float32 values;
 *  - the optional per-expert additive router bias is a benchmark knob that
 *    the paper does not have; it is part of G(x) when present;
 *  - expert capacity (Eq.8): the "number of tokens T" of that equation is
 *    read as the number of (token, slot) assignments T*K (with T itself the
 *    capacities of Eq.8 sum to gamma*T for K*T assignments, so that at
 *    K = 2, gamma = 1.1 almost half of all assignments would be dropped);
 *    the literal form, T tokens, can be asked for as well;
 *    C_i is rounded up to an integer; an expert keeps the first C_i of the
 *    assignments it received in (token, slot) order and the others are
 *    dropped: a dropped assignment contributes nothing to y (the token
 *    reaches the next block through the residual connection around the
 *    layer), the gate weights of the kept ones are not renormalised;
 *  - f_i of Eq.7 counts the tokens that selected expert i before any drop.
 *
 * Pins: tests/test_oracle_*.py check this file against closed forms of
 * Eq.3-5, invariants of Eq.1 and Eq.6, hand-computed examples, a dense
 * "all experts then mask" evaluation of Eq.1 and a textbook top-k MoE; the
 * capacity and load-balance functions against Eq.7 / Eq.8 worked by hand,
 * their closed forms for uniform routing and the textbook token-dropping
 * rule they reduce to without zero-computation experts.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t T, D, F;
    int32_t n_ffn, n_zero, n_copy, n_const;
    int32_t k;
} oracle_shape;

static int n_experts(const oracle_shape *s)
{
    return s->n_ffn + s->n_zero + s->n_copy + s->n_const;
}

int moepp_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* silu(z) = z * sigmoid(z) */
static double silu(double z)
{
    return z / (1.0 + exp(-z));
}

/*
 * Router (Eq.2 / Eq.6), softmax and Top-K (Eq.1) for every token.
 *
 *   x         [T,D]  float32
 *   prev_gate [T,N]  float32 or NULL  (NULL = first layer, Eq.6 case j = 1)
 *   W_g       [N,D]  float32   the router matrix (the paper's W^j)
 *   W_res     [N,N]  float32 or NULL  (the paper's W_g^j), used iff prev_gate
 *   bias      [N]    float32 or NULL
 *   forced_idx[T,K]  int32 or NULL: if given, the selection is taken from it
 *                    instead of Top-K (gate weights still come from softmax)
 * outputs
 *   out_gate  [T,N]  float32   G(x^j)
 *   probs     [T,N]  float64 or NULL   Softmax(G(x))
 *   topk_idx  [T,K]  int32
 *   topk_w    [T,K]  float32   g_i of the selected experts
 * returns 0, or -1 on an invalid shape.
 */
int moepp_oracle_route(const oracle_shape *s, const float *x,
                       const float *prev_gate, const float *W_g,
                       const float *W_res, const float *bias,
                       const int32_t *forced_idx, float *out_gate,
                       double *probs, int32_t *topk_idx, float *topk_w)
{
    const int N = n_experts(s), D = s->D, K = s->k;
    if (N <= 0 || K <= 0 || K > N || D <= 0 || s->T < 0)
        return -1;
    if ((prev_gate == NULL) != (W_res == NULL))
        return -1;

#pragma omp parallel for schedule(static)
    for (int t = 0; t < s->T; ++t) {
        float *L32 = out_gate + (size_t)t * N;
        double *p = (double *)malloc(sizeof(double) * N);
        char *taken = (char *)calloc(N, 1);

        /* G(x) = W x (+ W_g G(x_prev)) (+ bias) */
        for (int i = 0; i < N; ++i) {
            double acc = 0.0;
            for (int d = 0; d < D; ++d)
                acc += (double)W_g[(size_t)i * D + d] * (double)x[(size_t)t * D + d];
            if (prev_gate) {
                double r = 0.0;
                for (int m = 0; m < N; ++m)
                    r += (double)W_res[(size_t)i * N + m] *
                         (double)prev_gate[(size_t)t * N + m];
                acc += r;
            }
            if (bias)
                acc += (double)bias[i];
            L32[i] = (float)acc;
        }

        /* softmax over all N experts */
        double mx = (double)L32[0];
        for (int i = 1; i < N; ++i)
            if ((double)L32[i] > mx)
                mx = (double)L32[i];
        double z = 0.0;
        for (int i = 0; i < N; ++i) {
            p[i] = exp((double)L32[i] - mx);
            z += p[i];
        }
        for (int i = 0; i < N; ++i)
            p[i] /= z;
        if (probs)
            memcpy(probs + (size_t)t * N, p, sizeof(double) * N);

        /* Top-K by repeated selection of the largest remaining logit;
         * a strict ">" scan from index 0 gives ties to the lower index. */
        for (int sl = 0; sl < K; ++sl) {
            int best;
            if (forced_idx) {
                best = forced_idx[(size_t)t * K + sl];
            } else {
                best = -1;
                for (int i = 0; i < N; ++i) {
                    if (taken[i])
                        continue;
                    if (best < 0 || L32[i] > L32[best])
                        best = i;
                }
                taken[best] = 1;
            }
            topk_idx[(size_t)t * K + sl] = best;
            topk_w[(size_t)t * K + sl] = (float)p[best];
        }
        free(p);
        free(taken);
    }
    return 0;
}

/*
 * Grouping of the (token, slot) pairs by FFN expert.
 *
 *   counts [N]        number of slots that selected expert i (all experts)
 *   offsets[n_ffn+1]  exclusive prefix sum of counts over the FFN experts;
 *                     offsets[n_ffn] = R, the number of rows that reach an FFN
 *   row_of [T*K]      row in [0,R) of slot t*K+s, or -1 if the slot selected a
 *                     zero-computation expert
 *   src_of [T*K]      first R entries: slot t*K+s held by each row
 * Rows of one expert are ordered by (token, slot) ascending.
 */
int moepp_oracle_permute(const oracle_shape *s, const int32_t *topk_idx,
                         int32_t *counts, int32_t *offsets, int32_t *row_of,
                         int32_t *src_of)
{
    const int N = n_experts(s), K = s->k, T = s->T;
    for (int i = 0; i < N; ++i)
        counts[i] = 0;
    for (int q = 0; q < T * K; ++q) {
        int e = topk_idx[q];
        if (e < 0 || e >= N)
            return -1;
        counts[e] += 1;
        row_of[q] = -1;
        src_of[q] = -1;
    }
    offsets[0] = 0;
    for (int e = 0; e < s->n_ffn; ++e)
        offsets[e + 1] = offsets[e] + counts[e];
    int row = 0;
    for (int e = 0; e < s->n_ffn; ++e)
        for (int t = 0; t < T; ++t)
            for (int sl = 0; sl < K; ++sl)
                if (topk_idx[t * K + sl] == e) {
                    src_of[row] = t * K + sl;
                    row_of[t * K + sl] = row;
                    ++row;
                }
    return 0;
}

/*
 * Expert capacity, Eq.8: C_i = gamma * tau * S / (tau N_FFN + N_ZC) for an FFN
 * expert and gamma * S / (tau N_FFN + N_ZC) for a zero-computation expert,
 * rounded up (a relative 1e-9 above an integer counts as that integer).
 * per_assignment != 0: S = T*K assignments (the reading in the header);
 * per_assignment == 0: S = T, the number of tokens, Eq.8 as it is printed.
 *   cap [N] int32
 */
int moepp_oracle_capacity(const oracle_shape *s, double gamma, double tau,
                          int32_t per_assignment, int32_t *cap)
{
    const int N = n_experts(s);
    const int n_zc = N - s->n_ffn;
    const double denom = tau * (double)s->n_ffn + (double)n_zc;
    if (!(gamma > 0.0) || !(tau > 0.0) || !(denom > 0.0))
        return -1;
    const double S = per_assignment ? (double)s->T * (double)s->k : (double)s->T;
    for (int i = 0; i < N; ++i) {
        const double c = i < s->n_ffn ? gamma * tau * S / denom : gamma * S / denom;
        /* round up, but take a value that exceeds an integer only by the
         * representation error of gamma and tau (1.1 * 200 / 10 evaluates
         * to 22.000000000000004) as that integer */
        cap[i] = (int32_t)ceil(c - 1e-9 * (c > 1.0 ? c : 1.0));
    }
    return 0;
}

/*
 * Grouping with expert capacities: as moepp_oracle_permute, but expert i
 * keeps only the first cap[i] of its assignments in (token, slot) order.
 *
 *   counts [N]        assignments per expert before any drop
 *   kept   [N]        min(counts[i], cap[i])
 *   offsets[n_ffn+1]  exclusive prefix sum of kept over the FFN experts
 *   row_of [T*K]      row of a kept FFN assignment; -1 for a kept assignment
 *                     of a zero-computation expert; -2 for a dropped one
 *   src_of [T*K]      first R = offsets[n_ffn] entries: assignment of each row
 */
int moepp_oracle_permute_capacity(const oracle_shape *s, const int32_t *topk_idx,
                                  const int32_t *cap, int32_t *counts,
                                  int32_t *kept, int32_t *offsets,
                                  int32_t *row_of, int32_t *src_of)
{
    const int N = n_experts(s), K = s->k, T = s->T;
    for (int i = 0; i < N; ++i) {
        counts[i] = 0;
        if (cap[i] < 0)
            return -1;
    }
    for (int q = 0; q < T * K; ++q) {
        int e = topk_idx[q];
        if (e < 0 || e >= N)
            return -1;
        counts[e] += 1;
        src_of[q] = -1;
    }
    for (int i = 0; i < N; ++i)
        kept[i] = counts[i] < cap[i] ? counts[i] : cap[i];
    offsets[0] = 0;
    for (int e = 0; e < s->n_ffn; ++e)
        offsets[e + 1] = offsets[e] + kept[e];
    /* walk the assignments in (token, slot) order, one running rank per expert */
    int32_t *rank = (int32_t *)calloc(N > 0 ? N : 1, sizeof(int32_t));
    for (int q = 0; q < T * K; ++q) {
        const int e = topk_idx[q];
        const int r = rank[e]++;
        if (r >= cap[e]) {
            row_of[q] = -2;
        } else if (e < s->n_ffn) {
            row_of[q] = offsets[e] + r;
            src_of[offsets[e] + r] = q;
        } else {
            row_of[q] = -1;
        }
    }
    free(rank);
    return 0;
}

/*
 * Heterogeneous load-balance statistics, Eq.7:
 *   f_i = (1/T) #{tokens that selected expert i},  P_i = (1/T) sum_t Softmax(G(x_t))_i,
 *   L_b = sum_i eta_i f_i P_i,  eta_i = 1 (FFN expert) or tau (zero-computation expert).
 *   probs [T,N] float64 (Softmax(G(x)) from moepp_oracle_route), topk_idx [T,K]
 *   f, P [N] float64; loss [1] float64
 */
int moepp_oracle_balance(const oracle_shape *s, const double *probs,
                         const int32_t *topk_idx, double tau, double *f,
                         double *P, double *loss)
{
    const int N = n_experts(s), K = s->k, T = s->T;
    if (T <= 0)
        return -1;
    for (int i = 0; i < N; ++i) {
        f[i] = 0.0;
        P[i] = 0.0;
    }
    for (int t = 0; t < T; ++t) {
        for (int sl = 0; sl < K; ++sl)
            f[topk_idx[(size_t)t * K + sl]] += 1.0;
        for (int i = 0; i < N; ++i)
            P[i] += probs[(size_t)t * N + i];
    }
    double L = 0.0;
    for (int i = 0; i < N; ++i) {
        f[i] /= (double)T;
        P[i] /= (double)T;
        L += (i < s->n_ffn ? 1.0 : tau) * f[i] * P[i];
    }
    *loss = L;
    return 0;
}

/* output of expert i for one token: e[D] (fp64).  xf is the token in fp64. */
static void expert_output(const oracle_shape *s, int i, const double *xf,
                          const float *w1, const float *w3, const float *w2,
                          const float *const_vecs, const float *W_c,
                          double *e, double *h, double *alpha1_out)
{
    const int D = s->D, F = s->F;
    if (i < s->n_ffn) {
        /* FFN expert: W2 ( silu(W1 x) * (W3 x) ) */
        const float *A = w1 + (size_t)i * F * D;
        const float *B = w3 + (size_t)i * F * D;
        const float *C = w2 + (size_t)i * D * F;
        for (int f = 0; f < F; ++f) {
            double g = 0.0, u = 0.0;
            for (int d = 0; d < D; ++d)
                g += (double)A[(size_t)f * D + d] * xf[d];
            for (int d = 0; d < D; ++d)
                u += (double)B[(size_t)f * D + d] * xf[d];
            h[f] = silu(g) * u;
        }
        for (int d = 0; d < D; ++d) {
            double acc = 0.0;
            for (int f = 0; f < F; ++f)
                acc += (double)C[(size_t)d * F + f] * h[f];
            e[d] = acc;
        }
    } else if (i < s->n_ffn + s->n_zero) {
        /* zero expert, Eq.3 */
        for (int d = 0; d < D; ++d)
            e[d] = 0.0;
    } else if (i < s->n_ffn + s->n_zero + s->n_copy) {
        /* copy expert, Eq.4 */
        for (int d = 0; d < D; ++d)
            e[d] = xf[d];
    } else {
        /* constant expert j, Eq.5: [a1,a2] = softmax(W_c x); a1 x + a2 v */
        int j = i - (s->n_ffn + s->n_zero + s->n_copy);
        const float *Wc = W_c + (size_t)j * 2 * D;
        const float *v = const_vecs + (size_t)j * D;
        double l1 = 0.0, l2 = 0.0;
        for (int d = 0; d < D; ++d)
            l1 += (double)Wc[d] * xf[d];
        for (int d = 0; d < D; ++d)
            l2 += (double)Wc[D + d] * xf[d];
        double m = l1 > l2 ? l1 : l2;
        double e1 = exp(l1 - m), e2 = exp(l2 - m);
        double a1 = e1 / (e1 + e2), a2 = e2 / (e1 + e2);
        for (int d = 0; d < D; ++d)
            e[d] = a1 * xf[d] + a2 * (double)v[d];
        if (alpha1_out)
            *alpha1_out = a1;
    }
}

/*
 * Expert evaluation and weighted sum (Eq.1) for the tokens in tok_list
 * (n_tok entries; NULL = tokens 0..n_tok-1).
 *
 *   w1, w3 [n_ffn,F,D], w2 [n_ffn,D,F], const_vecs [n_const,D],
 *   W_c [n_const,2,D]    float32
 *   topk_idx/topk_w [T,K] as written by moepp_oracle_route
 *   row_of [T*K] int32 or NULL: assignments with row_of == -2 were dropped by
 *                the expert capacity and contribute nothing
 * outputs (row u belongs to token tok_list[u])
 *   out     [n_tok,D]        float64  y = sum_s g_s E_s(x)
 *   slot_out[n_tok,K,D]      float64 or NULL  E_s(x) of each selected expert
 *   h       [n_tok,K,F]      float64 or NULL  SwiGLU intermediate of FFN slots
 *                                              (untouched for other slots)
 *   alpha1  [n_tok,n_const]  float64 or NULL  a1 of every constant expert,
 *                                              selected or not
 */
int moepp_oracle_experts(const oracle_shape *s, const float *x,
                         const int32_t *topk_idx, const float *topk_w,
                         const float *w1, const float *w3, const float *w2,
                         const float *const_vecs, const float *W_c,
                         const int32_t *row_of,
                         int32_t n_tok, const int32_t *tok_list, double *out,
                         double *slot_out, double *h_out, double *alpha1)
{
    const int D = s->D, F = s->F, K = s->k;
    const int zc0 = s->n_ffn + s->n_zero + s->n_copy;
    int bad = 0;

#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int u = 0; u < n_tok; ++u) {
        const int t = tok_list ? tok_list[u] : u;
        if (t < 0 || t >= s->T) {
            bad |= 1;
            continue;
        }
        double *xf = (double *)malloc(sizeof(double) * D);
        double *e = (double *)malloc(sizeof(double) * D);
        double *h = (double *)malloc(sizeof(double) * (F > 0 ? F : 1));
        double *y = out + (size_t)u * D;
        for (int d = 0; d < D; ++d) {
            xf[d] = (double)x[(size_t)t * D + d];
            y[d] = 0.0;
        }
        for (int sl = 0; sl < K; ++sl) {
            const int i = topk_idx[(size_t)t * K + sl];
            const double g = (double)topk_w[(size_t)t * K + sl];
            if (row_of && row_of[(size_t)t * K + sl] == -2)
                continue;                       /* dropped: over capacity */
            expert_output(s, i, xf, w1, w3, w2, const_vecs, W_c, e, h, NULL);
            for (int d = 0; d < D; ++d)
                y[d] += g * e[d];
            if (slot_out)
                memcpy(slot_out + ((size_t)u * K + sl) * D, e, sizeof(double) * D);
            if (h_out && i < s->n_ffn)
                memcpy(h_out + ((size_t)u * K + sl) * F, h, sizeof(double) * F);
        }
        if (alpha1)
            for (int j = 0; j < s->n_const; ++j)
                expert_output(s, zc0 + j, xf, w1, w3, w2, const_vecs, W_c, e, h,
                              alpha1 + (size_t)u * s->n_const + j);
        free(xf);
        free(e);
        free(h);
    }
    return bad ? -1 : 0;
}

/*
 * Eq.1 evaluated literally: every one of the N experts is applied to every
 * token and the results are summed with the gate vector g, which is zero
 * outside the selected experts.  Kept separate from the per-slot path above
 * (it shares only expert_output) and used on small inputs to cross-check it.
 *   gate [T,N] float64: g_i (already masked).   out [T,D] float64.
 */
int moepp_oracle_dense(const oracle_shape *s, const float *x, const double *gate,
                       const float *w1, const float *w3, const float *w2,
                       const float *const_vecs, const float *W_c, double *out)
{
    const int D = s->D, F = s->F, N = n_experts(s);
#pragma omp parallel for schedule(static)
    for (int t = 0; t < s->T; ++t) {
        double *xf = (double *)malloc(sizeof(double) * D);
        double *e = (double *)malloc(sizeof(double) * D);
        double *h = (double *)malloc(sizeof(double) * (F > 0 ? F : 1));
        double *y = out + (size_t)t * D;
        for (int d = 0; d < D; ++d) {
            xf[d] = (double)x[(size_t)t * D + d];
            y[d] = 0.0;
        }
        for (int i = 0; i < N; ++i) {
            expert_output(s, i, xf, w1, w3, w2, const_vecs, W_c, e, h, NULL);
            for (int d = 0; d < D; ++d)
                y[d] += gate[(size_t)t * N + i] * e[d];
        }
        free(xf);
        free(e);
        free(h);
    }
    return 0;
}
