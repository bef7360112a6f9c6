// Grouping of the (token, slot) pairs by FFN expert: a stable counting sort in
// three kernels (histogram per chunk, exclusive scan, scatter).  Integer work
// only, no atomics, so the result is the same on every run: rows of one
// expert are ordered by ascending slot index q = t*k + s.
//
// The paper does not describe this step; it is how the K selected experts of
// Eq.1 are turned into contiguous row groups for the grouped FFN GEMM.
//
// With expert capacities (Sec. 3.3, Eq.8) expert i keeps the first cap[i] of
// its slots in that order; the others are dropped (row_of = -2) and take no
// part in the GEMMs or in the combine.  The same file holds the reduction for
// the load-balance statistics of Eq.7.
#include "common.h"

namespace moepp {

constexpr int kPermWaves = 4;

__device__ inline int slot_expert(const int32_t *idx, int q, int total) {
    return q < total ? idx[q] : -1;
}

// chunk_hist[c][e] = number of slots of chunk c that selected expert e.
__global__ __launch_bounds__(kPermWaves *kWave) void k_perm_hist(Dims d, Workspace w) {
    const int lane = threadIdx.x % kWave;
    const int c = blockIdx.x * kPermWaves + threadIdx.x / kWave;
    const int total = d.T * d.k;
    if (c * kPermChunk >= total) return;
    int cnt = 0;
    for (int it = 0; it < kPermIters; ++it) {
        const int e_mine = slot_expert(w.topk_idx, c * kPermChunk + it * kWave + lane, total);
        for (int e = 0; e < d.N; ++e) {
            unsigned long long m = __ballot(e_mine == e);
            if (lane == e) cnt += __popcll(m);
        }
    }
    if (lane < d.N) w.chunk_hist[c * d.N + lane] = cnt;
}

// chunk_base[c][e] = slots of expert e in chunks before c; counts; kept; offsets.
__global__ __launch_bounds__(kPermWaves *kWave) void k_perm_scan(Dims d, Workspace w, CapArgs cap) {
    const int lane = threadIdx.x % kWave;
    const int wv = threadIdx.x / kWave;
    const int total = d.T * d.k;
    const int n_chunks = (total + kPermChunk - 1) / kPermChunk;
    __shared__ int s_counts[kMaxExperts];
    for (int e = wv; e < d.N; e += kPermWaves) {
        int running = 0;
        for (int c0 = 0; c0 < n_chunks; c0 += kWave) {
            const int c = c0 + lane;
            const int v = c < n_chunks ? w.chunk_hist[c * d.N + e] : 0;
            int incl = v;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                int up = __shfl_up(incl, o, kWave);
                if (lane >= o) incl += up;
            }
            if (c < n_chunks) w.chunk_base[c * d.N + e] = running + incl - v;
            running += __shfl(incl, kWave - 1, kWave);
        }
        if (lane == 0) {
            const int keep = cap.on && cap.cap[e] < running ? cap.cap[e] : running;
            s_counts[e] = keep;
            w.counts[e] = running;
            w.kept[e] = keep;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int acc = 0;
        w.offsets[0] = 0;
        for (int e = 0; e < d.n_ffn; ++e) {
            acc += s_counts[e];
            w.offsets[e + 1] = acc;
        }
    }
}

// row_of / src_of.  CAP: expert capacities apply (every expert's rank is
// tracked, not only the FFN experts').
template <bool CAP>
__global__ __launch_bounds__(kPermWaves *kWave) void k_perm_scatter(Dims d, Workspace w, CapArgs cap) {
    const int lane = threadIdx.x % kWave;
    const int c = blockIdx.x * kPermWaves + threadIdx.x / kWave;
    const int total = d.T * d.k;
    if (c * kPermChunk >= total) return;
    const int n_track = CAP ? d.N : d.n_ffn;
    // lane e tracks the rank of the next slot of expert e within its expert
    int rank = 0, first_row = 0, limit = 0x7fffffff;
    if (lane < n_track) {
        rank = w.chunk_base[c * d.N + lane];
        if (lane < d.n_ffn) first_row = w.offsets[lane];
        if (CAP) limit = cap.cap[lane];
    }
    const unsigned long long lt = (1ull << lane) - 1ull;
    for (int it = 0; it < kPermIters; ++it) {
        const int q = c * kPermChunk + it * kWave + lane;
        const int e_mine = slot_expert(w.topk_idx, q, total);
        int row = -1;
        for (int e = 0; e < n_track; ++e) {
            unsigned long long m = __ballot(e_mine == e);
            // (all lanes take part in the shuffles; only the slots of expert e use them)
            const int r = __shfl(rank, e, kWave) + __popcll(m & lt);
            const int lim_e = CAP ? __shfl(limit, e, kWave) : 0x7fffffff;
            const int row_e = __shfl(first_row, e, kWave) + r;
            if (e_mine == e) {
                if (r >= lim_e) row = -2;
                else if (e < d.n_ffn) row = row_e;
            }
            if (lane == e) rank += __popcll(m);
        }
        if (q < total) {
            w.row_of[q] = row;
            if (row >= 0) w.src_of[row] = q;
        }
    }
}

// ---- load-balance statistics (Eq.7) ---------------------------------------
// Pass 1: wave g takes tokens g, g + kBalWaves, ...; lane i owns expert i,
// recomputes Softmax(G(x_t))_i from the logits the router wrote and adds it
// up in fp64.  Pass 2: one workgroup adds the per-wave sums in a fixed order
// (the result is the same on every run), P_i = sum / T, f_i = counts_i / T,
// L_b = sum_i eta_i f_i P_i with eta = 1 for FFN experts, tau for the others.
__global__ __launch_bounds__(4 * kWave) void k_balance_partial(Dims d, Workspace w, const float *out_gate) {
    const int lane = threadIdx.x % kWave;
    const int g = blockIdx.x * 4 + threadIdx.x / kWave;
    double acc = 0.0;
    for (int t = g; t < d.T; t += kBalWaves) {
        const float L = lane < d.N ? out_gate[(size_t)t * d.N + lane] : -INFINITY;
        const float mx = wave_max(L);
        const float e = lane < d.N ? expf(L - mx) : 0.f;
        acc += (double)(e / wave_sum(e));
    }
    w.bal_partial[(size_t)g * kMaxExperts + lane] = acc;
}

constexpr int kBalFinalWaves = 16;
__global__ __launch_bounds__(kBalFinalWaves *kWave) void k_balance_final(Dims d, Workspace w, float tau) {
    __shared__ double part[kBalFinalWaves][kWave];
    const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
    // wave wv adds its block of per-wave sums in index order, wave 0 the 16 block sums in order
    constexpr int per = kBalWaves / kBalFinalWaves;
    double sum = 0.0;
    for (int g = wv * per; g < (wv + 1) * per; ++g) sum += w.bal_partial[(size_t)g * kMaxExperts + lane];
    part[wv][lane] = sum;
    __syncthreads();
    if (wv != 0) return;
    sum = 0.0;
    for (int q = 0; q < kBalFinalWaves; ++q) sum += part[q][lane];
    const double P = lane < d.N ? sum / (double)d.T : 0.0;
    const double f = lane < d.N ? (double)w.counts[lane] / (double)d.T : 0.0;
    double term = (lane < d.n_ffn ? 1.0 : (double)tau) * f * P;
    // sum over lanes in index order
    double loss = 0.0;
    for (int i = 0; i < d.N; ++i) loss += __shfl(term, i, kWave);
    if (lane < d.N) {
        w.bal[lane] = (float)f;
        w.bal[d.N + lane] = (float)P;
    }
    if (lane == 0) w.bal[2 * d.N] = (float)loss;
}

static int perm_blocks(const Dims &d) {
    const int total = d.T * d.k;
    const int n_chunks = (total + kPermChunk - 1) / kPermChunk;
    return (n_chunks + kPermWaves - 1) / kPermWaves;
}

hipError_t launch_perm_hist(const Dims &d, const Workspace &w, hipStream_t s) {
    if (d.T == 0) return hipSuccess;
    hipLaunchKernelGGL(k_perm_hist, dim3(perm_blocks(d)), dim3(kPermWaves * kWave), 0, s, d, w);
    return hipGetLastError();
}
hipError_t launch_perm_scan(const Dims &d, const Workspace &w, const CapArgs &cap, hipStream_t s) {
    hipLaunchKernelGGL(k_perm_scan, dim3(1), dim3(kPermWaves * kWave), 0, s, d, w, cap);
    return hipGetLastError();
}
hipError_t launch_perm_scatter(const Dims &d, const Workspace &w, const CapArgs &cap, hipStream_t s) {
    if (d.T == 0) return hipSuccess;
    const dim3 grid(perm_blocks(d)), block(kPermWaves * kWave);
    if (cap.on) hipLaunchKernelGGL(k_perm_scatter<true>, grid, block, 0, s, d, w, cap);
    else hipLaunchKernelGGL(k_perm_scatter<false>, grid, block, 0, s, d, w, cap);
    return hipGetLastError();
}
hipError_t launch_balance(const Dims &d, const Workspace &w, const float *out_gate, float tau,
                          hipStream_t s) {
    if (d.T == 0) return hipSuccess;
    hipLaunchKernelGGL(k_balance_partial, dim3(kBalWaves / 4), dim3(4 * kWave), 0, s, d, w, out_gate);
    hipLaunchKernelGGL(k_balance_final, dim3(1), dim3(kBalFinalWaves * kWave), 0, s, d, w, tau);
    return hipGetLastError();
}

}  // namespace moepp
