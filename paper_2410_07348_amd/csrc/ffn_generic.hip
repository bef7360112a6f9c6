// Grouped SwiGLU FFN for any supported shape and activation type, plain fp32
// FMA: one thread per output element.  FFN_e(x) = W2_e (silu(W1_e x) * (W3_e x))
// for the rows of every FFN expert e (the FFN experts of paper Eq.2).  This is
// the path of the float32 layers and the fallback for shapes the MFMA kernels
// do not cover.
#include "common.h"

namespace moepp {

__device__ inline int expert_of_row(const int32_t *offsets, int n_ffn, int r) {
    int e = 0;
    while (e + 1 < n_ffn && r >= offsets[e + 1]) ++e;
    return e;
}

__device__ inline float silu_f(float z) { return z / (1.f + expf(-z)); }

// h[r,f] = silu(W1_e[f,:] x_r) * (W3_e[f,:] x_r), x_r = x[src_of[r] / k]
template <typename AT>
__global__ __launch_bounds__(256) void k_ffn1_generic(FfnArgs a) {
    const int r = blockIdx.x;
    const int f = blockIdx.y * blockDim.x + threadIdx.x;
    const int R = a.offsets[a.d.n_ffn];
    if (r >= R || f >= a.d.F) return;
    const int D = a.d.D, F = a.d.F;
    const int e = expert_of_row(a.offsets, a.d.n_ffn, r);
    const int t = a.src_of[r] / a.d.k;
    const AT *x = static_cast<const AT *>(a.x) + (size_t)t * D;
    const AT *W = static_cast<const AT *>(a.w13) + (size_t)e * 2 * F * D;
    const int rg = packed_row(f, 0, F), ru = packed_row(f, 1, F);
    constexpr int V = ActVec<AT>::N;
    float g = 0.f, u = 0.f;
    for (int s = 0; s * kSlab < D; ++s) {          // the packed weights: panels of K slabs
        const AT *wg = W + panel_row(rg, s, 2 * F, D);
        const AT *wu = W + panel_row(ru, s, 2 * F, D);
        const int kw = slab_width(s, D);
        for (int d = 0; d < kw; d += V) {
            ActVec<AT> xv = load_vec(x + s * kSlab + d), gv = load_vec(wg + d), uv = load_vec(wu + d);
#pragma unroll
            for (int i = 0; i < V; ++i) {
                g = fmaf(gv.get(i), xv.get(i), g);
                u = fmaf(uv.get(i), xv.get(i), u);
            }
        }
    }
    static_cast<AT *>(a.h)[slab_row(r, f / kSlab, a.h_rows, F) + f % kSlab] = (AT)(silu_f(g) * u);
}

// yffn[r,d] = W2_e[d,:] h[r,:]
template <typename AT>
__global__ __launch_bounds__(256) void k_ffn2_generic(FfnArgs a) {
    const int r = blockIdx.x;
    const int dd = blockIdx.y * blockDim.x + threadIdx.x;
    const int R = a.offsets[a.d.n_ffn];
    if (r >= R || dd >= a.d.D) return;
    const int D = a.d.D, F = a.d.F;
    const int e = expert_of_row(a.offsets, a.d.n_ffn, r);
    const AT *hb = static_cast<const AT *>(a.h);
    const AT *wb = static_cast<const AT *>(a.w2) + (size_t)e * D * F;
    constexpr int V = ActVec<AT>::N;
    float acc = 0.f;
    for (int s = 0; s * kSlab < F; ++s) {          // h is K-slab-major, the packed weights are panels of K slabs
        const AT *h = hb + slab_row(r, s, a.h_rows, F);
        const AT *w = wb + panel_row(dd, s, D, F);
        const int kw = slab_width(s, F);
        for (int f = 0; f < kw; f += V) {
            ActVec<AT> hv = load_vec(h + f), wv = load_vec(w + f);
#pragma unroll
            for (int i = 0; i < V; ++i) acc = fmaf(wv.get(i), hv.get(i), acc);
        }
    }
    static_cast<AT *>(a.yffn)[(size_t)r * D + dd] = (AT)acc;
}

hipError_t launch_ffn_generic(const FfnArgs &a, bool bf16, int which, hipStream_t s) {
    const int rows = a.d.T * a.d.k;   // upper bound of R; surplus blocks exit at once
    if (rows == 0 || a.d.n_ffn == 0) return hipSuccess;
    const int cols = which == 0 ? a.d.F : a.d.D;
    dim3 grid(rows, (cols + 255) / 256), block(256);
    if (which == 0) {
        if (bf16) hipLaunchKernelGGL(k_ffn1_generic<bf16_t>, grid, block, 0, s, a);
        else hipLaunchKernelGGL(k_ffn1_generic<float>, grid, block, 0, s, a);
    } else {
        if (bf16) hipLaunchKernelGGL(k_ffn2_generic<bf16_t>, grid, block, 0, s, a);
        else hipLaunchKernelGGL(k_ffn2_generic<float>, grid, block, 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace moepp
