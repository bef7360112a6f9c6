// Weighted combine (paper Eq.1) with the zero, copy and constant experts
// (Eq.3-5) evaluated in place: tokens routed to those experts never enter a
// GEMM, their contribution is elementwise work on x and the constant vectors.
//
//   y_t = sum over slots s = 0..K-1, in that order, of g_s * E_s(x_t)
//     FFN expert      : E = yffn[row_of[t,s]]
//     zero expert     : E = 0                          (nothing is read)
//     copy expert     : E = x_t
//     constant expert : E = a1 x_t + (1 - a1) v_j
//     any expert, slot dropped by the expert capacity (row_of = -2): nothing
// fp32 accumulation, one rounding to the activation type.  HBM-bound: one
// wavefront streams one token with 16-byte accesses per lane.
#include "common.h"

namespace moepp {

constexpr int kCombineWaves = 4;

// KMAX: slots the kernel is unrolled for (2: the paper's Top-2 layers keep their
// per-slot plan in a handful of registers; kMaxTopK: any k).
template <typename AT, int KMAX>
__global__ __launch_bounds__(kCombineWaves *kWave) void k_combine(CombineArgs a) {
    const int lane = threadIdx.x % kWave;
    const int t = blockIdx.x * kCombineWaves + threadIdx.x / kWave;
    if (t >= a.d.T) return;
    const int D = a.d.D, K = a.d.k;
    const int zero0 = a.d.n_ffn, copy0 = zero0 + a.d.n_zero, const0 = copy0 + a.d.n_copy;
    constexpr int V = ActVec<AT>::N;

    // Per-slot plan (wave-uniform): coefficient of a gathered row, of x, of v_j.
    float g_row[KMAX], g_x[KMAX], g_v[KMAX];
    const AT *p_row[KMAX];
    const AT *p_v[KMAX];
    bool need_x = false;
#pragma unroll
    for (int s = 0; s < KMAX; ++s) {
        g_row[s] = g_x[s] = g_v[s] = 0.f;
        p_row[s] = p_v[s] = nullptr;
        if (s < K) {
            const int i = a.topk_idx[(size_t)t * K + s];
            const float g = a.topk_w[(size_t)t * K + s];
            const int row = a.row_of[(size_t)t * K + s];
            if (row == -2) {
                // over the expert's capacity: dropped
            } else if (i < zero0) {
                g_row[s] = g;
                p_row[s] = static_cast<const AT *>(a.yffn) + (size_t)row * D;
            } else if (i < copy0) {
                // zero expert: contributes nothing
            } else if (i < const0) {
                g_x[s] = g;
                need_x = true;
            } else {
                const int j = i - const0;
                const float a1 = a.alpha1[(size_t)t * a.d.n_const + j];
                g_x[s] = g * a1;
                g_v[s] = g * (1.f - a1);
                p_v[s] = static_cast<const AT *>(a.const_vecs) + (size_t)j * D;
                need_x = true;
            }
        }
    }
    const AT *xt = static_cast<const AT *>(a.x) + (size_t)t * D;
    AT *ot = static_cast<AT *>(a.out) + (size_t)t * D;
#pragma unroll 4
    for (int d = lane * V; d < D; d += kWave * V) {
        float acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.f;
        ActVec<AT> xv;
        if (need_x) xv = load_vec_stream(xt + d);
#pragma unroll
        for (int s = 0; s < KMAX; ++s) {
            if (s < K) {
                if (p_row[s]) {
                    ActVec<AT> rv = load_vec_stream(p_row[s] + d);   // read once
#pragma unroll
                    for (int i = 0; i < V; ++i) acc[i] = fmaf(g_row[s], rv.get(i), acc[i]);
                } else if (p_v[s]) {
                    ActVec<AT> vv = load_vec(p_v[s] + d);
#pragma unroll
                    for (int i = 0; i < V; ++i)
                        acc[i] += g_x[s] * xv.get(i) + g_v[s] * vv.get(i);
                } else if (g_x[s] != 0.f) {
#pragma unroll
                    for (int i = 0; i < V; ++i) acc[i] = fmaf(g_x[s], xv.get(i), acc[i]);
                }
            }
        }
        ActVec<AT> ov;
#pragma unroll
        for (int i = 0; i < V; ++i) ov.set(i, acc[i]);
        store_vec_stream(ot + d, ov);
    }
}

hipError_t launch_combine(const CombineArgs &a, bool bf16, hipStream_t s) {
    if (a.d.T == 0) return hipSuccess;
    dim3 grid((a.d.T + kCombineWaves - 1) / kCombineWaves), block(kCombineWaves * kWave);
    if (a.d.k <= 2) {
        if (bf16) hipLaunchKernelGGL((k_combine<bf16_t, 2>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_combine<float, 2>), grid, block, 0, s, a);
    } else {
        if (bf16) hipLaunchKernelGGL((k_combine<bf16_t, kMaxTopK>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_combine<float, kMaxTopK>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// One-time repacking of the expert weights (not part of the forward pass).
template <typename AT>
__global__ __launch_bounds__(256) void k_pack(Dims d, const AT *w1, const AT *w3, const AT *w2,
                                              AT *w13, AT *w2o) {
    constexpr int V = ActVec<AT>::N;
    const size_t per = (size_t)d.F * d.D / V;            // vectors per matrix
    const size_t n = (size_t)d.n_ffn * per;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x) {
        const size_t e = i / per, v = i % per;
        {   // W1 / W3 row f, columns dv..: packed rows of the [2F, D] matrix, in panels
            const int f = (int)(v / (d.D / V));
            const int dv = (int)(v % (d.D / V)) * V;
            AT *dst = w13 + e * 2 * d.F * d.D;
            const int sl = dv / kSlab, in = dv % kSlab;
            store_vec(dst + panel_row(packed_row(f, 0, d.F), sl, 2 * d.F, d.D) + in, load_vec(w1 + i * V));
            store_vec(dst + panel_row(packed_row(f, 1, d.F), sl, 2 * d.F, d.D) + in, load_vec(w3 + i * V));
        }
        {   // W2 row dd, columns fv..: the [D, F] matrix, in panels
            const int dd = (int)(v / (d.F / V));
            const int fv = (int)(v % (d.F / V)) * V;
            AT *dst = w2o + e * d.D * d.F;
            store_vec(dst + panel_row(dd, fv / kSlab, d.D, d.F) + fv % kSlab, load_vec(w2 + i * V));
        }
    }
}

hipError_t launch_pack(const Dims &d, bool bf16, const void *w1, const void *w3, const void *w2,
                       void *w13_out, void *w2_out, hipStream_t s) {
    if (d.n_ffn == 0) return hipSuccess;
    dim3 grid(4096), block(256);
    if (bf16)
        hipLaunchKernelGGL(k_pack<bf16_t>, grid, block, 0, s, d, (const bf16_t *)w1,
                           (const bf16_t *)w3, (const bf16_t *)w2, (bf16_t *)w13_out,
                           (bf16_t *)w2_out);
    else
        hipLaunchKernelGGL(k_pack<float>, grid, block, 0, s, d, (const float *)w1,
                           (const float *)w3, (const float *)w2, (float *)w13_out,
                           (float *)w2_out);
    return hipGetLastError();
}

}  // namespace moepp
