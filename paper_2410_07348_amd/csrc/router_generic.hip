// Router for any supported shape and activation type, plain fp32 FMA.
//
// One wavefront per token computes, in one pass over x:
//   G(x) = W x (+ W_g G(x_prev)) (+ bias)            (paper Eq.2 / Eq.6)
//   Softmax over all N experts and Top-K of G(x)     (Eq.1)
//   a1 of every constant expert, Softmax(W_c x)_1    (Eq.5)
// Top-K runs on the float32 logits; ties go to the lower index and slots are
// written in descending order of logit.
#include "common.h"

namespace moepp {

constexpr int kRouterWaves = 4;
constexpr int kMaxRouterRows = kMaxExperts + 2 * kMaxConst;

template <typename AT>
__global__ __launch_bounds__(kRouterWaves *kWave) void k_router_generic(RouterArgs a) {
    __shared__ float dots[kRouterWaves][kMaxRouterRows];
    const int lane = threadIdx.x % kWave;
    const int w = threadIdx.x / kWave;
    const int t = blockIdx.x * kRouterWaves + w;
    const int D = a.d.D, N = a.d.N, K = a.d.k, nc = a.d.n_const;
    const bool active = t < a.d.T;
    const int rows = N + 2 * nc;
    constexpr int V = ActVec<AT>::N;

    if (active) {
        const AT *xt = static_cast<const AT *>(a.x) + (size_t)t * D;
        for (int r = 0; r < rows; ++r) {
            const float *wr = r < N ? a.W_g + (size_t)r * D : a.W_c + (size_t)(r - N) * D;
            float acc = 0.f;
            for (int d = lane * V; d < D; d += kWave * V) {
                ActVec<AT> xv = load_vec(xt + d);
#pragma unroll
                for (int i = 0; i < V; ++i) acc = fmaf(wr[d + i], xv.get(i), acc);
            }
            acc = wave_sum(acc);
            if (lane == 0) dots[w][r] = acc;
        }
    }
    __syncthreads();
    if (!active) return;

    // logits: lane i owns expert i
    float L = -INFINITY;
    if (lane < N) {
        L = dots[w][lane];
        if (a.prev_gate) {
            float r = 0.f;
            for (int m = 0; m < N; ++m)
                r = fmaf(a.W_res[lane * N + m], a.prev_gate[(size_t)t * N + m], r);
            L += r;
        }
        if (a.bias) L += a.bias[lane];
        a.out_gate[(size_t)t * N + lane] = L;
    }
    const float mx = wave_max(L);
    const float e = lane < N ? expf(L - mx) : 0.f;
    const float p = e / wave_sum(e);

    // Top-K by K rounds of wave-wide argmax on (logit desc, index asc)
    float cand = L;
    for (int s = 0; s < K; ++s) {
        float bv = cand;
        int bi = lane;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            float ov = __shfl_xor(bv, o, kWave);
            int oi = __shfl_xor(bi, o, kWave);
            if (ov > bv || (ov == bv && oi < bi)) {
                bv = ov;
                bi = oi;
            }
        }
        float pw = __shfl(p, bi, kWave);
        if (lane == bi) cand = -INFINITY;
        if (lane == 0) {
            a.topk_idx[(size_t)t * K + s] = bi;
            a.topk_w[(size_t)t * K + s] = pw;
        }
    }

    if (lane < nc) {
        float l1 = dots[w][N + 2 * lane], l2 = dots[w][N + 2 * lane + 1];
        a.alpha1[(size_t)t * nc + lane] = 1.f / (1.f + expf(l2 - l1));
    }
}

hipError_t launch_router_generic(const RouterArgs &a, bool bf16, hipStream_t s) {
    if (a.d.T == 0) return hipSuccess;
    dim3 grid((a.d.T + kRouterWaves - 1) / kRouterWaves), block(kRouterWaves * kWave);
    if (bf16)
        hipLaunchKernelGGL(k_router_generic<bf16_t>, grid, block, 0, s, a);
    else
        hipLaunchKernelGGL(k_router_generic<float>, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace moepp
