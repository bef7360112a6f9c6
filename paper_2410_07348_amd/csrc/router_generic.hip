// Router for any supported shape and activation type, plain fp32 FMA.
//
// One wavefront per token computes, in one pass over x:
//   G(x) = W x (+ W_g G(x_prev)) (+ bias)            (paper Eq.2 / Eq.6)
//   Softmax over all N experts and Top-K of G(x)     (Eq.1)
//   a1 of every constant expert, Softmax(W_c x)_1    (Eq.5)
// Top-K runs on the float32 logits; ties go to the lower index and slots are
// written in descending order of logit.
#include "common.h"
#include "perm_device.h"
#include "router_device.h"

#include <type_traits>

namespace moepp {

constexpr int kRouterWaves = 4;
constexpr int kMaxRouterRows = kMaxExperts + 2 * kMaxConst;

// W_res into LDS with all threads of the workgroup (the caller synchronises).
__device__ inline void stage_wres(const RouterArgs &a, float *wres) {
    if (!a.prev_gate) return;
    for (int c = threadIdx.x; c < a.d.N * a.d.N; c += blockDim.x) wres[c] = a.W_res[c];
}

// Gating residual, bias, softmax, Top-K and a1 for token t by one wave; `dots`
// holds the token's N + 2 n_const dot products with x, `wres` W_res (both LDS).
__device__ inline void router_tail(const RouterArgs &a, int t, int lane, const float *dots,
                                   const float *wres) {
    const int N = a.d.N, K = a.d.k, nc = a.d.n_const;
    // logits: lane i owns expert i
    float L = -INFINITY;
    const bool mine = lane < N;
    float r = 0.f;
    if (a.prev_gate) {
        const float pg = mine ? a.prev_gate[(size_t)t * N + lane] : 0.f;
        for (int m = 0; m < N; ++m) {
            const float pm = __shfl(pg, m, kWave);
            if (mine) r = fmaf(wres[lane * N + m], pm, r);
        }
    }
    if (mine) {
        L = dots[lane] + r;
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
        float l1 = dots[N + 2 * lane], l2 = dots[N + 2 * lane + 1];
        a.alpha1[(size_t)t * nc + lane] = 1.f / (1.f + expf(l2 - l1));
    }
}

template <typename AT>
__global__ __launch_bounds__(kRouterWaves *kWave) void k_router_generic(RouterArgs a) {
    __shared__ float dots[kRouterWaves][kMaxRouterRows];
    __shared__ float wres[kMaxExperts * kMaxExperts];
    const int lane = threadIdx.x % kWave;
    const int w = threadIdx.x / kWave;
    const int t = blockIdx.x * kRouterWaves + w;
    const int D = a.d.D, N = a.d.N, nc = a.d.n_const;
    const bool active = t < a.d.T;
    const int rows = N + 2 * nc;
    constexpr int V = ActVec<AT>::N;
    stage_wres(a, wres);

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
    if (active) router_tail(a, t, lane, dots[w], wres);
}

// ---- few tokens -------------------------------------------------------------
// With a few hundred tokens at most, one workgroup per block of tokens leaves
// the chip empty and the pass over x and the router weights runs at one CU's
// load rate.  Here the reduction over D is cut into up to kRsSplits slices:
// workgroup (slice, token block) writes the partial dot products of its slice,
// and a second kernel adds the slices of a token in slice order (the result is
// the same on every run) and finishes as above.
constexpr int kRsTok = 64;      // tokens per workgroup
constexpr int kRsBK = 64;       // K elements per LDS tile
constexpr int kRsStr = kRsBK + 4;   // floats per LDS tile row: 16-byte reads of 16 consecutive rows cover all banks
constexpr int kRsSplits = 32;   // slices at most

// RPT: weight rows per thread; the four waves share 4 RPT >= N + 2 n_const rows
// (rows past the last are zero in LDS, so the inner loop has no conditions).
template <typename AT, int RPT>
__global__ __launch_bounds__(4 * kWave) void k_router_small_partial(RouterArgs a, int slice,
                                                                    float *partial) {
    __shared__ __attribute__((aligned(16))) float sx[kRsTok][kRsStr];
    __shared__ __attribute__((aligned(16))) float sw[4 * RPT][kRsStr];
    const int tid = threadIdx.x, tok = tid % kWave, rg = tid / kWave;
    const int D = a.d.D, N = a.d.N, T = a.d.T, rows = N + 2 * a.d.n_const;
    const int t0 = blockIdx.y * kRsTok;
    const int k_begin = blockIdx.x * slice, k_end = min(k_begin + slice, D);
    constexpr int V = ActVec<AT>::N;
    const AT *x = static_cast<const AT *>(a.x);
    f32x4 acc[RPT];
#pragma unroll
    for (int j = 0; j < RPT; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int k0 = k_begin; k0 < k_end; k0 += kRsBK) {
        // x tile [64 tokens][64 k] and weight tile [4 RPT rows][64 k], zero past k_end and past the last row
        for (int c = tid; c < kRsTok * (kRsBK / V); c += 4 * kWave) {
            const int tt = c / (kRsBK / V), kk = (c % (kRsBK / V)) * V;
            const int t = min(t0 + tt, T - 1);
            ActVec<AT> xv;
#pragma unroll
            for (int i = 0; i < V; ++i) xv.set(i, 0.f);
            if (k0 + kk < k_end) xv = load_vec(x + (size_t)t * D + k0 + kk);
#pragma unroll
            for (int i = 0; i < V; i += 4)
                *reinterpret_cast<f32x4 *>(&sx[tt][kk + i]) =
                    f32x4{xv.get(i), xv.get(i + 1), xv.get(i + 2), xv.get(i + 3)};
        }
        for (int c = tid; c < 4 * RPT * (kRsBK / 4); c += 4 * kWave) {
            const int r = c / (kRsBK / 4), kk = (c % (kRsBK / 4)) * 4;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (r < rows && k0 + kk < k_end) {
                const float *wr = r < N ? a.W_g + (size_t)r * D : a.W_c + (size_t)(r - N) * D;
                v = *reinterpret_cast<const f32x4 *>(wr + k0 + kk);
            }
            *reinterpret_cast<f32x4 *>(&sw[r][kk]) = v;
        }
        __syncthreads();
        // wave rg owns rows rg, rg + 4, ...: the weight reads are broadcasts.
        // acc[j][i] collects the k with k % 4 == i.
#pragma unroll 4
        for (int kk = 0; kk < kRsBK; kk += 4) {
            const f32x4 xv = *reinterpret_cast<const f32x4 *>(&sx[tok][kk]);
#pragma unroll
            for (int j = 0; j < RPT; ++j) {
                const f32x4 wv = *reinterpret_cast<const f32x4 *>(&sw[rg + 4 * j][kk]);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[j][i] = fmaf(wv[i], xv[i], acc[j][i]);
            }
        }
        __syncthreads();
    }
    if (t0 + tok < T) {
        float *dst = partial + ((size_t)blockIdx.x * T + t0 + tok) * rows;
#pragma unroll
        for (int j = 0; j < RPT; ++j)
            if (rg + 4 * j < rows) dst[rg + 4 * j] = (acc[j][0] + acc[j][1]) + (acc[j][2] + acc[j][3]);
    }
}

__global__ __launch_bounds__(kRouterWaves *kWave) void k_router_small_final(RouterArgs a, int n_splits,
                                                                           const float *partial) {
    __shared__ float dots[kRouterWaves][kMaxRouterRows];
    __shared__ float wres[kMaxExperts * kMaxExperts];
    const int lane = threadIdx.x % kWave;
    const int w = threadIdx.x / kWave;
    const int t = blockIdx.x * kRouterWaves + w;
    const int rows = a.d.N + 2 * a.d.n_const;
    const bool active = t < a.d.T;
    stage_wres(a, wres);
    if (active) {
        for (int r = lane; r < rows; r += kWave) {
            // all loads first (a fixed trip count lets them be issued together), then the sum in slice order
            float v[kRsSplits];
#pragma unroll
            for (int sp = 0; sp < kRsSplits; ++sp)
                v[sp] = sp < n_splits ? partial[((size_t)sp * a.d.T + t) * rows + r] : 0.f;
            float sum = 0.f;
#pragma unroll
            for (int sp = 0; sp < kRsSplits; ++sp) sum += v[sp];
            dots[w][r] = sum;
        }
    }
    __syncthreads();
    if (active) router_tail(a, t, lane, dots[w], wres);
}

// The second kernel and the permutation in one launch, for T <= kRouterFusedT: one
// workgroup adds the slices of every dot product (in slice order), finishes the
// logits (gating residual, bias) with all threads, does softmax / Top-K / a1 with
// four threads per token, and then groups the T*k selections, which it still
// holds in LDS, by expert like k_perm_small does.
__global__ __launch_bounds__(kPermSmallWaves *kWave) void k_router_small_final_perm(RouterArgs a, int n_splits,
                                                                                  const float *partial, Workspace w,
                                                                                  CapArgs cap) {
    constexpr int NT = kPermSmallWaves * kWave;
    constexpr int DSTR = kMaxRouterRows + 1;
    __shared__ float dots[kRouterFusedT * DSTR];
    __shared__ float prevs[kRouterFusedT * (kMaxExperts + 1)];
    __shared__ float wres[kMaxExperts * kMaxExperts];
    __shared__ float sbias[kMaxExperts];
    __shared__ int s_idx[kRouterFusedT * kMaxTopK];
    __shared__ int s_rank[kPermSmallWaves][kMaxExperts];
    __shared__ int s_first[kMaxExperts], s_limit[kMaxExperts];
    const int tid = threadIdx.x;
    const int T = a.d.T, N = a.d.N, K = a.d.k, rows = N + 2 * a.d.n_const;
    for (int c = tid; c < T * rows; c += NT) {
        // element c = (token c / rows, row c % rows) of every slice; all loads first, then the sum in slice order
        float v[kRsSplits];
#pragma unroll
        for (int sp = 0; sp < kRsSplits; ++sp) v[sp] = sp < n_splits ? partial[(size_t)sp * T * rows + c] : 0.f;
        float sum = 0.f;
#pragma unroll
        for (int sp = 0; sp < kRsSplits; ++sp) sum += v[sp];
        dots[(c / rows) * DSTR + c % rows] = sum;
    }
    if (a.prev_gate) {
        for (int c = tid; c < T * N; c += NT) prevs[(c / N) * (kMaxExperts + 1) + c % N] = a.prev_gate[c];
        for (int c = tid; c < N * N; c += NT) wres[c] = a.W_res[c];
    }
    if (tid < N) sbias[tid] = a.bias ? a.bias[tid] : 0.f;
    __syncthreads();
    for (int c = tid; c < T * N; c += NT) {
        const int tt = c / N, i = c % N;
        float L = dots[tt * DSTR + i];
        if (a.prev_gate) {
            const float *pr = prevs + tt * (kMaxExperts + 1);
            const float *wr = wres + i * N;
            float r = 0.f;
            for (int m = 0; m < N; ++m) r = fmaf(wr[m], pr[m], r);
            L += r;
        }
        L += sbias[i];
        dots[tt * DSTR + i] = L;        // only this thread reads or writes the element
        a.out_gate[c] = L;
    }
    __syncthreads();
    {
        // every thread runs this (the shuffles are wave-wide); threads past the last token
        // compute on the last token and store nothing
        const int tok = tid >> 2;
        const int tk = tok < T ? tok : T - 1;
        router_token_quad(a, (size_t)tk, tok < T, tid & 3, dots + tk * DSTR, nullptr, s_idx + tk * K);
    }
    __syncthreads();
    perm_small_body(a.d, w, cap, s_idx, s_rank, s_first, s_limit);
}

size_t router_small_bytes() {
    return (size_t)kRsSplits * kRouterSmallT * kMaxRouterRows * sizeof(float);
}

hipError_t launch_router_small(const RouterArgs &a, bool bf16, float *partial, hipStream_t s,
                               const Workspace *perm_ws, const CapArgs *perm_cap) {
    if (a.d.T == 0) return hipSuccess;
    if (a.d.T > kRouterSmallT) return hipErrorInvalidValue;
    const int tiles = (a.d.D + kRsBK - 1) / kRsBK;
    const int per = (tiles + kRsSplits - 1) / kRsSplits;        // K tiles per slice
    const int slice = per * kRsBK;
    const int n_splits = (a.d.D + slice - 1) / slice;           // <= kRsSplits
    const dim3 grid(n_splits, (a.d.T + kRsTok - 1) / kRsTok), block(4 * kWave);
    const int rows = a.d.N + 2 * a.d.n_const;
    auto go = [&](auto rpt) {
        constexpr int RPT = decltype(rpt)::value;
        if (bf16)
            hipLaunchKernelGGL((k_router_small_partial<bf16_t, RPT>), grid, block, 0, s, a, slice, partial);
        else
            hipLaunchKernelGGL((k_router_small_partial<float, RPT>), grid, block, 0, s, a, slice, partial);
    };
    static_assert(kMaxRouterRows <= 80, "rows per thread");
    if (rows <= 24) go(std::integral_constant<int, 6>());
    else if (rows <= 40) go(std::integral_constant<int, 10>());
    else go(std::integral_constant<int, 20>());
    if (perm_ws) {
        if (a.d.T > kRouterFusedT || perm_cap == nullptr) return hipErrorInvalidValue;
        hipLaunchKernelGGL(k_router_small_final_perm, dim3(1), dim3(kPermSmallWaves * kWave), 0, s, a, n_splits,
                           partial, *perm_ws, *perm_cap);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_router_small_final, dim3((a.d.T + kRouterWaves - 1) / kRouterWaves),
                       dim3(kRouterWaves * kWave), 0, s, a, n_splits, partial);
    return hipGetLastError();
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
