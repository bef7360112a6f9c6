// Grouping of the (token, slot) pairs by FFN expert: a stable counting sort in
// three kernels (histogram per chunk, exclusive scan, scatter).  Integer work
// only, no atomics, so the result is the same on every run: rows of one
// expert are ordered by ascending slot index q = t*k + s.
//
// The paper does not describe this step; it is how the K selected experts of
// Eq.1 are turned into contiguous row groups for the grouped FFN GEMM.
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

// chunk_base[c][e] = slots of expert e in chunks before c; counts; offsets.
__global__ __launch_bounds__(kPermWaves *kWave) void k_perm_scan(Dims d, Workspace w) {
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
            s_counts[e] = running;
            w.counts[e] = running;
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

// row_of / src_of.
__global__ __launch_bounds__(kPermWaves *kWave) void k_perm_scatter(Dims d, Workspace w) {
    const int lane = threadIdx.x % kWave;
    const int c = blockIdx.x * kPermWaves + threadIdx.x / kWave;
    const int total = d.T * d.k;
    if (c * kPermChunk >= total) return;
    // lane e tracks the next free row of FFN expert e
    int running = 0;
    if (lane < d.n_ffn) running = w.offsets[lane] + w.chunk_base[c * d.N + lane];
    const unsigned long long lt = (1ull << lane) - 1ull;
    for (int it = 0; it < kPermIters; ++it) {
        const int q = c * kPermChunk + it * kWave + lane;
        const int e_mine = slot_expert(w.topk_idx, q, total);
        int row = -1;
        for (int e = 0; e < d.n_ffn; ++e) {
            unsigned long long m = __ballot(e_mine == e);
            int base = __shfl(running, e, kWave);
            if (e_mine == e) row = base + __popcll(m & lt);
            if (lane == e) running += __popcll(m);
        }
        if (q < total) {
            w.row_of[q] = row;
            if (row >= 0) w.src_of[row] = q;
        }
    }
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
hipError_t launch_perm_scan(const Dims &d, const Workspace &w, hipStream_t s) {
    hipLaunchKernelGGL(k_perm_scan, dim3(1), dim3(kPermWaves * kWave), 0, s, d, w);
    return hipGetLastError();
}
hipError_t launch_perm_scatter(const Dims &d, const Workspace &w, hipStream_t s) {
    if (d.T == 0) return hipSuccess;
    hipLaunchKernelGGL(k_perm_scatter, dim3(perm_blocks(d)), dim3(kPermWaves * kWave), 0, s, d, w);
    return hipGetLastError();
}

}  // namespace moepp
