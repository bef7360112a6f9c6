// Grouping of the (token, slot) pairs by FFN expert: a stable counting sort in
// three kernels (histogram per chunk, exclusive scan, scatter), or in one
// workgroup when there are few slots.  Integer work
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

// Expert of slot q, or -1 past the last slot (and for an index outside
// [0, N), which only a workspace that no routing call has filled can hold).
__device__ inline int slot_expert(const int32_t *idx, int q, int total, int N) {
    const int e = q < total ? idx[q] : -1;
    return (unsigned)e < (unsigned)N ? e : -1;
}

// The lanes of the wave that hold the same expert as this lane, among the
// lanes with a slot (e >= 0): six ballots, one per bit of the expert index.
static_assert(kMaxExperts <= 64, "six index bits");
__device__ inline unsigned long long same_expert_lanes(int e) {
    unsigned long long m = __ballot(e >= 0);
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        const bool bit = (e >> b) & 1;
        const unsigned long long bal = __ballot(bit);
        m &= bit ? bal : ~bal;
    }
    return m;
}

// cnt[e] (LDS, this wave's own 64 counters) = slots of chunk c on expert e.
// The lowest lane of every group of equal experts adds the group's size; LDS
// operations of one wave execute in program order.
__device__ inline void chunk_histogram(const int32_t *idx, int c, int total, int N, int lane,
                                       volatile int *cnt) {
    cnt[lane] = 0;
    for (int it = 0; it < kPermIters; ++it) {
        const int e = slot_expert(idx, c * kPermChunk + it * kWave + lane, total, N);
        const unsigned long long m = same_expert_lanes(e);
        if (e >= 0 && lane == __ffsll((long long)m) - 1) cnt[e] += __popcll(m);
    }
}

// chunk_hist[c][e] = number of slots of chunk c that selected expert e.
__global__ __launch_bounds__(kPermWaves *kWave) void k_perm_hist(Dims d, Workspace w) {
    __shared__ int s_cnt[kPermWaves][kMaxExperts];
    const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
    const int c = blockIdx.x * kPermWaves + wv;
    const int total = d.T * d.k;
    if (c * kPermChunk >= total) return;
    chunk_histogram(w.topk_idx, c, total, d.N, lane, s_cnt[wv]);
    if (lane < d.N) w.chunk_hist[c * d.N + lane] = ((volatile int *)s_cnt[wv])[lane];
}

// chunk_base[c][e] = slots of expert e in chunks before c; counts; kept; offsets.
constexpr int kScanWaves = 16;   // one workgroup; its waves share the experts
__global__ __launch_bounds__(kScanWaves *kWave) void k_perm_scan(Dims d, Workspace w, CapArgs cap) {
    const int lane = threadIdx.x % kWave;
    const int wv = threadIdx.x / kWave;
    const int total = d.T * d.k;
    const int n_chunks = (total + kPermChunk - 1) / kPermChunk;
    __shared__ int s_counts[kMaxExperts];
    for (int e = wv; e < d.N; e += kScanWaves) {
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

// row_of / src_of of chunk c.  rank[e] (LDS, this wave's own 64 counters)
// enters with the rank, within expert e, of the chunk's first slot on e;
// first_row[e] is the first row of FFN expert e and limit[e] the capacity of
// expert e (both LDS, read only).  A slot's rank is rank[e] plus the number of
// lower lanes on the same expert; the lowest lane of the group then moves
// rank[e] past the group.
__device__ inline void scatter_chunk(const Dims &d, const Workspace &w, int c, int lane,
                                     volatile int *rank, const int *first_row, const int *limit) {
    const int total = d.T * d.k;
    const unsigned long long lt = (1ull << lane) - 1ull;
    for (int it = 0; it < kPermIters; ++it) {
        const int q = c * kPermChunk + it * kWave + lane;
        const int e = slot_expert(w.topk_idx, q, total, d.N);
        const unsigned long long m = same_expert_lanes(e);
        if (e >= 0) {
            const int old = rank[e];
            const int r = old + __popcll(m & lt);
            if (lane == __ffsll((long long)m) - 1) rank[e] = old + __popcll(m);
            int row = -1;
            if (r >= limit[e]) row = -2;
            else if (e < d.n_ffn) row = first_row[e] + r;
            w.row_of[q] = row;
            if (row >= 0) w.src_of[row] = q;
        } else if (q < total) {
            w.row_of[q] = -2;                              // no valid expert: the combine skips the slot
        }
    }
}

__global__ __launch_bounds__(kPermWaves *kWave) void k_perm_scatter(Dims d, Workspace w, CapArgs cap) {
    __shared__ int s_rank[kPermWaves][kMaxExperts];
    __shared__ int s_first[kMaxExperts], s_limit[kMaxExperts];
    const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
    const int c = blockIdx.x * kPermWaves + wv;
    const bool active = c * kPermChunk < d.T * d.k;
    if (wv == 0) {
        s_first[lane] = lane < d.n_ffn ? w.offsets[lane] : 0;
        s_limit[lane] = cap.on && lane < d.N ? cap.cap[lane] : 0x7fffffff;
    }
    if (active) s_rank[wv][lane] = lane < d.N ? w.chunk_base[c * d.N + lane] : 0;
    __syncthreads();
    if (active) scatter_chunk(d, w, c, lane, s_rank[wv], s_first, s_limit);
}

// The three steps in one workgroup, for calls with at most kPermSmallSlots
// slots (one launch instead of three; same results).  Wave c owns chunk c.
__global__ __launch_bounds__(kPermSmallWaves *kWave) void k_perm_small(Dims d, Workspace w, CapArgs cap) {
    __shared__ int s_rank[kPermSmallWaves][kMaxExperts];   // counts, then ranks of the chunk's first slots
    __shared__ int s_first[kMaxExperts], s_limit[kMaxExperts];
    const int lane = threadIdx.x % kWave, c = threadIdx.x / kWave;
    const int total = d.T * d.k;
    chunk_histogram(w.topk_idx, c, total, d.N, lane, s_rank[c]);
    __syncthreads();
    if (c == 0) {                                          // wave 0: lane e scans expert e over the chunks
        int running = 0;
        for (int q = 0; q < kPermSmallWaves; ++q) {
            const int v = s_rank[q][lane];
            s_rank[q][lane] = running;
            running += v;
        }
        int keep = 0, lim = 0x7fffffff;
        if (lane < d.N) {
            if (cap.on) lim = cap.cap[lane];
            keep = lim < running ? lim : running;
            w.counts[lane] = running;
            w.kept[lane] = keep;
        }
        const int kf = lane < d.n_ffn ? keep : 0;
        int incl = kf;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            int up = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += up;
        }
        s_first[lane] = incl - kf;
        s_limit[lane] = lim;
        if (lane < d.n_ffn) w.offsets[lane + 1] = incl;
        if (lane == 0) w.offsets[0] = 0;
    }
    __syncthreads();
    if (c * kPermChunk < total) scatter_chunk(d, w, c, lane, s_rank[c], s_first, s_limit);
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
    hipLaunchKernelGGL(k_perm_scan, dim3(1), dim3(kScanWaves * kWave), 0, s, d, w, cap);
    return hipGetLastError();
}
hipError_t launch_perm_scatter(const Dims &d, const Workspace &w, const CapArgs &cap, hipStream_t s) {
    if (d.T == 0) return hipSuccess;
    const dim3 grid(perm_blocks(d)), block(kPermWaves * kWave);
    hipLaunchKernelGGL(k_perm_scatter, grid, block, 0, s, d, w, cap);
    return hipGetLastError();
}
hipError_t launch_perm_small(const Dims &d, const Workspace &w, const CapArgs &cap, hipStream_t s) {
    if (d.T <= 0 || d.T * d.k > kPermSmallSlots) return hipErrorInvalidValue;
    const dim3 grid(1), block(kPermSmallWaves * kWave);
    hipLaunchKernelGGL(k_perm_small, grid, block, 0, s, d, w, cap);
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
