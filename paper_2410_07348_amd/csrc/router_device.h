// Device-side piece of the router that more than one kernel uses.
#pragma once
#include "common.h"

namespace moepp {

// Softmax over all N experts, Top-K (paper Eq.1) and a1 of every constant expert
// (Eq.5) for token t by four neighbouring threads q = 0 .. 3 of a wave; thread q
// owns the experts i = q, q + 4, ... and shuffles combine the four.  Lr: the token's
// N + 2 n_const float32 logits (LDS).  Ties go to the lower index, slots are
// written in descending order of logit.  Every thread of the wave must call this
// (the shuffles are wave-wide); `valid` false: compute, store nothing.
// hist (LDS, may be null): selections per expert, counted with integer atomics.
// sel (LDS, may be null): sel[s] receives the expert of slot s.
// probs (LDS, may be null): probs[i] receives Softmax(G(x))_i, 0 when not valid.
__device__ inline void router_token_quad(const RouterArgs &a, size_t t, bool valid, int q, const float *Lr,
                                         int *hist, int *sel, float *probs = nullptr) {
    const int N = a.d.N, K = a.d.k, nc = a.d.n_const;
    float mx = -INFINITY;
    for (int i = q; i < N; i += 4) mx = fmaxf(mx, Lr[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 1, kWave));
    mx = fmaxf(mx, __shfl_xor(mx, 2, kWave));
    float sum = 0.f;
    for (int i = q; i < N; i += 4) sum += __expf(Lr[i] - mx);
    sum += __shfl_xor(sum, 1, kWave);
    sum += __shfl_xor(sum, 2, kWave);
    const float inv = 1.f / sum;
    unsigned long long taken = 0ull;            // of this thread's own experts
    for (int s = 0; s < K; ++s) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;                    // none yet
        for (int i = q; i < N; i += 4) {
            const float v = Lr[i];
            if (!((taken >> i) & 1ull) && (bi == 0x7fffffff || v > bv)) {
                bv = v;
                bi = i;
            }
        }
#pragma unroll
        for (int o = 1; o <= 2; o <<= 1) {
            const float ov = __shfl_xor(bv, o, kWave);
            const int oi = __shfl_xor(bi, o, kWave);
            // larger logit wins, equal logits go to the lower index
            if (oi != 0x7fffffff && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi))) {
                bv = ov;
                bi = oi;
            }
        }
        if ((bi & 3) == q) taken |= 1ull << bi;
        if (valid && q == 0) {
            a.topk_idx[t * K + s] = bi;
            a.topk_w[t * K + s] = __expf(bv - mx) * inv;
            if (hist) atomicAdd(&hist[bi], 1);   // integer counts: the same on every run
            if (sel) sel[s] = bi;
        }
    }
    if (valid)
        for (int j = q; j < nc; j += 4)
            a.alpha1[t * nc + j] = 1.f / (1.f + expf(Lr[N + 2 * j + 1] - Lr[N + 2 * j]));
    if (probs)
        for (int i = q; i < N; i += 4) probs[i] = valid ? __expf(Lr[i] - mx) * inv : 0.f;
}

}  // namespace moepp
