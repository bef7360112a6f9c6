// Grouping of the (token, slot) pairs by FFN expert: a stable counting sort.
// The slots are cut into chunks (one wave each); a histogram per chunk, an
// exclusive scan over the chunks and a scatter give every slot its row.  The
// histogram comes from the router kernel when that one counted its own
// workgroup's selections (then a chunk is the slots of one router workgroup),
// else from k_perm_hist; scan and scatter are one kernel in which every
// workgroup adds up the histogram rows its waves need itself (a few thousand
// chunks at most: the rows are 4 N bytes each and sit in L2), or two kernels
// with a single-workgroup scan when there are more chunks than that; calls with
// few slots do all of it in one workgroup (k_perm_small, or, with a handful of
// tokens, the last kernel of the few-token router).  Integer work only and no ordering left
// to atomics, so the result is the same on every run: rows of one expert are
// ordered by ascending slot index q = t*k + s.
//
// The paper does not describe this step; it is how the K selected experts of
// Eq.1 are turned into contiguous row groups for the grouped FFN GEMM.
//
// With expert capacities (Sec. 3.3, Eq.8) expert i keeps the first cap[i] of
// its slots in that order; the others are dropped (row_of = -2) and take no
// part in the GEMMs or in the combine.  The same file holds the reduction for
// the load-balance statistics of Eq.7.
#include "common.h"
#include "perm_device.h"

namespace moepp {

constexpr int kPermWaves = 4;

// chunk_hist[c][e] = number of slots of chunk c that selected expert e.
__global__ __launch_bounds__(kPermWaves *kWave) void k_perm_hist(Dims d, Workspace w, int chunk_slots) {
    __shared__ int s_cnt[kPermWaves][kMaxExperts];
    const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
    const int c = blockIdx.x * kPermWaves + wv;
    const int total = d.T * d.k;
    if ((long long)c * chunk_slots >= total) return;
    chunk_histogram(w.topk_idx, c, chunk_slots, total, d.N, lane, s_cnt[wv]);
    if (lane < d.N) w.chunk_hist[c * d.N + lane] = ((volatile int *)s_cnt[wv])[lane];
}

// chunk_base[c][e] = slots of expert e in chunks before c; counts; kept; offsets.
constexpr int kScanWaves = 16;   // one workgroup; its waves share the experts
__global__ __launch_bounds__(kScanWaves *kWave) void k_perm_scan(Dims d, Workspace w, CapArgs cap,
                                                                 int n_chunks) {
    const int lane = threadIdx.x % kWave;
    const int wv = threadIdx.x / kWave;
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

__global__ __launch_bounds__(kPermWaves *kWave) void k_perm_scatter(Dims d, Workspace w, CapArgs cap,
                                                                   int chunk_slots) {
    __shared__ int s_rank[kPermWaves][kMaxExperts];
    __shared__ int s_first[kMaxExperts], s_limit[kMaxExperts];
    const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
    const int c = blockIdx.x * kPermWaves + wv;
    const bool active = (long long)c * chunk_slots < d.T * d.k;
    if (wv == 0) {
        s_first[lane] = lane < d.n_ffn ? w.offsets[lane] : 0;
        s_limit[lane] = cap.on && lane < d.N ? cap.cap[lane] : 0x7fffffff;
    }
    int ex[kPermMaxRounds];
    if (active) {
        chunk_experts(d, w.topk_idx, c, chunk_slots, lane, ex);
        s_rank[wv][lane] = lane < d.N ? w.chunk_base[c * d.N + lane] : 0;
    }
    __syncthreads();
    if (active) scatter_chunk(d, w, c, chunk_slots, lane, ex, s_rank[wv], s_first, s_limit);
}

// Scan and scatter in one kernel, for at most kPermDirectChunks chunks.  Every
// wave needs, per expert, the selections in the chunks before its own (the ranks
// its chunk starts at) and in all chunks (the counts, from which it derives kept
// and the first row of every FFN expert like the scan kernel does).  The
// workgroup passes the whole table chunk_hist through LDS in pieces of
// kScanTileInts integers with coalesced 16-byte loads, and its threads share
// the additions: thread i looks after expert i % NP of the rows i / NP,
// i / NP + 256 / NP, ... of a piece (NP = N rounded up to a power of two) and
// adds up all of them and those before the workgroup's first chunk; the partial
// sums meet in LDS, and a wave adds the rows of the workgroup's chunks before
// its own.  The wave of chunk 0 also writes counts, kept and offsets.
constexpr int kScanTileInts = 8192;               // 32 KB of LDS
__global__ __launch_bounds__(kPermWaves *kWave) void k_perm_scan_scatter(Dims d, Workspace w, CapArgs cap,
                                                                        int chunk_slots, int n_chunks) {
    constexpr int NT = kPermWaves * kWave;
    __shared__ __attribute__((aligned(16))) int s_tab[kScanTileInts];
    __shared__ int s_all[NT], s_before[NT];        // [row group][expert slot]: NT / NP groups of NP
    __shared__ int s_rank[kPermWaves][kMaxExperts];
    __shared__ int s_first[kPermWaves][kMaxExperts], s_limit[kPermWaves][kMaxExperts];
    const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
    const int c0 = blockIdx.x * kPermWaves;        // first chunk of the workgroup
    const int c = c0 + wv;                         // may be past the last chunk: such a wave only helps adding
    const int N = d.N;
    int NP = 1, lg = 0;
    while (NP < N) NP <<= 1, ++lg;
    const int e = threadIdx.x & (NP - 1), grp = threadIdx.x >> lg, ngrp = NT >> lg;   // >= 4 row groups
    int ex[kPermMaxRounds];                        // this chunk's slots: in flight while the table is added up
    if (c < n_chunks) chunk_experts(d, w.topk_idx, c, chunk_slots, lane, ex);
    // the rows of the workgroup's own chunks before this wave's (the table pass stops short of them)
    int own[kPermWaves - 1];
#pragma unroll
    for (int i = 0; i < kPermWaves - 1; ++i)
        own[i] = i < wv && c0 + i < n_chunks && lane < N ? w.chunk_hist[(c0 + i) * N + lane] : 0;
    const int tile_rows = kScanTileInts / N;       // whole rows per piece (N <= 64: at least 128)
    const int total_ints = n_chunks * N;           // <= kPermDirectChunks * 64
    // thread (grp, e) adds up expert e over the rows grp, grp + ngrp, ... of every piece:
    // all of them, and those before the workgroup's first chunk
    int before = 0, all = 0;
    for (int row0 = 0; row0 < n_chunks; row0 += tile_rows) {
        const int base = row0 * N;
        const int n_ints = min(tile_rows * N, total_ints - base);
        // the workspace regions are 256-byte aligned and whole pieces start at multiples of N * tile_rows
        // integers; pieces are copied 16 bytes at a time where the alignment allows, else by integers
        if (((base | n_ints) & 3) == 0) {
            // all loads of the piece first, then the LDS writes: one memory latency, not one per load
            constexpr int PER = kScanTileInts / (NT * 4);
            int4 v[PER];
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int i = (threadIdx.x + u * NT) * 4;
                v[u] = make_int4(0, 0, 0, 0);      // (every element defined: the array stays in registers)
                if (i < n_ints) v[u] = *reinterpret_cast<const int4 *>(&w.chunk_hist[base + i]);
            }
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int i = (threadIdx.x + u * NT) * 4;
                if (i < n_ints) *reinterpret_cast<int4 *>(&s_tab[i]) = v[u];
            }
        } else {
            for (int i = threadIdx.x; i < n_ints; i += NT) s_tab[i] = w.chunk_hist[base + i];
        }
        __syncthreads();
        const int rows = n_ints / N;
        if (e < N) {
            constexpr int U = 4;                   // reads in flight: the sums would otherwise wait for each one
            for (int r0 = grp; r0 < rows; r0 += U * ngrp) {
                int v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = r0 + u * ngrp < rows ? s_tab[(r0 + u * ngrp) * N + e] : 0;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    all += v[u];
                    if (row0 + r0 + u * ngrp < c0) before += v[u];
                }
            }
        }
        __syncthreads();
    }
    s_all[threadIdx.x] = all;                      // index = grp * NP + e
    s_before[threadIdx.x] = before;
    __syncthreads();
    if (c >= n_chunks) return;
    // lane l < N: expert l's sums over the row groups (in group order), plus the
    // workgroup's own chunks before this wave's
    all = 0;
    before = 0;
    if (lane < N) {
        for (int g = 0; g < ngrp; ++g) {
            all += s_all[g * NP + lane];
            before += s_before[g * NP + lane];
        }
#pragma unroll
        for (int i = 0; i < kPermWaves - 1; ++i) before += own[i];
    }
    const int lim = cap.on && lane < N ? cap.cap[lane] : 0x7fffffff;
    const int keep = lane < N ? (lim < all ? lim : all) : 0;
    const int kf = lane < d.n_ffn ? keep : 0;
    int incl = kf;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int up = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += up;
    }
    if (c == 0) {
        if (lane < N) {
            w.counts[lane] = all;
            w.kept[lane] = keep;
        }
        if (lane < d.n_ffn) w.offsets[lane + 1] = incl;
        if (lane == 0) w.offsets[0] = 0;
    }
    ((volatile int *)s_rank[wv])[lane] = lane < N ? before : 0;
    ((volatile int *)s_first[wv])[lane] = incl - kf;
    ((volatile int *)s_limit[wv])[lane] = lim;
    // (this wave's own LDS rows: LDS operations of one wave execute in order; the
    // fence keeps the compiler from moving the reads below above these writes)
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    scatter_chunk(d, w, c, chunk_slots, lane, ex, s_rank[wv], s_first[wv], s_limit[wv]);
}

// The three steps in one workgroup, for calls with at most kPermSmallSlots
// slots (one launch instead of three; same results).
__global__ __launch_bounds__(kPermSmallWaves *kWave) void k_perm_small(Dims d, Workspace w, CapArgs cap) {
    __shared__ int s_rank[kPermSmallWaves][kMaxExperts];   // counts, then ranks of the chunk's first slots
    __shared__ int s_first[kMaxExperts], s_limit[kMaxExperts];
    perm_small_body(d, w, cap, w.topk_idx, s_rank, s_first, s_limit);
}

// ---- load-balance statistics (Eq.7) ---------------------------------------
// Pass 1: wave g takes tokens g, g + kBalWaves, ...; lane i owns expert i,
// recomputes Softmax(G(x_t))_i from the logits the router wrote and adds it
// up in fp64 (not needed when the matrix-core router has left the sums of its
// workgroups' tokens itself).  Pass 2: one workgroup adds the per-wave sums in a fixed order
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
__global__ __launch_bounds__(kBalFinalWaves *kWave) void k_balance_final(Dims d, Workspace w, float tau,
                                                                        int n_rows) {
    __shared__ double part[kBalFinalWaves][kWave];
    const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
    // wave wv adds its block of the n_rows partial sums in index order, wave 0 the 16 block sums in order
    // (rows written by the router kernel hold nothing for lanes >= N: those lanes' sums are not used)
    const int per = (n_rows + kBalFinalWaves - 1) / kBalFinalWaves;
    double sum = 0.0;
    const int g_end = min((wv + 1) * per, n_rows);
    for (int g0 = wv * per; g0 < g_end; g0 += 8) {         // eight loads in flight, added in index order
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = g0 + u < g_end ? w.bal_partial[(size_t)(g0 + u) * kMaxExperts + lane] : 0.0;
#pragma unroll
        for (int u = 0; u < 8; ++u) sum += v[u];
    }
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

int perm_chunks(const Dims &d, int chunk_slots) {
    const long long total = (long long)d.T * d.k;
    return (int)((total + chunk_slots - 1) / chunk_slots);
}
static int perm_blocks(int n_chunks) { return (n_chunks + kPermWaves - 1) / kPermWaves; }

hipError_t launch_perm_hist(const Dims &d, const Workspace &w, int chunk_slots, hipStream_t s) {
    if (d.T == 0) return hipSuccess;
    hipLaunchKernelGGL(k_perm_hist, dim3(perm_blocks(perm_chunks(d, chunk_slots))), dim3(kPermWaves * kWave),
                       0, s, d, w, chunk_slots);
    return hipGetLastError();
}
hipError_t launch_perm_scan(const Dims &d, const Workspace &w, const CapArgs &cap, int chunk_slots,
                            hipStream_t s) {
    hipLaunchKernelGGL(k_perm_scan, dim3(1), dim3(kScanWaves * kWave), 0, s, d, w, cap,
                       perm_chunks(d, chunk_slots));
    return hipGetLastError();
}
hipError_t launch_perm_scatter(const Dims &d, const Workspace &w, const CapArgs &cap, int chunk_slots,
                               hipStream_t s) {
    if (d.T == 0) return hipSuccess;
    if (chunk_slots > kPermMaxRounds * kWave) return hipErrorInvalidValue;
    const dim3 grid(perm_blocks(perm_chunks(d, chunk_slots))), block(kPermWaves * kWave);
    hipLaunchKernelGGL(k_perm_scatter, grid, block, 0, s, d, w, cap, chunk_slots);
    return hipGetLastError();
}
hipError_t launch_perm_scan_scatter(const Dims &d, const Workspace &w, const CapArgs &cap, int chunk_slots,
                                    hipStream_t s) {
    if (d.T == 0) return hipSuccess;
    const int n_chunks = perm_chunks(d, chunk_slots);
    if (n_chunks > kPermDirectChunks || chunk_slots > kPermMaxRounds * kWave) return hipErrorInvalidValue;
    const dim3 grid(perm_blocks(n_chunks)), block(kPermWaves * kWave);
    hipLaunchKernelGGL(k_perm_scan_scatter, grid, block, 0, s, d, w, cap, chunk_slots, n_chunks);
    return hipGetLastError();
}
hipError_t launch_perm_small(const Dims &d, const Workspace &w, const CapArgs &cap, hipStream_t s) {
    if (d.T <= 0 || d.T * d.k > kPermSmallSlots) return hipErrorInvalidValue;
    const dim3 grid(1), block(kPermSmallWaves * kWave);
    hipLaunchKernelGGL(k_perm_small, grid, block, 0, s, d, w, cap);
    return hipGetLastError();
}
hipError_t launch_balance(const Dims &d, const Workspace &w, const float *out_gate, float tau,
                          hipStream_t s, int router_rows) {
    if (d.T == 0) return hipSuccess;
    if (router_rows > kBalWaves) return hipErrorInvalidValue;
    if (router_rows <= 0)
        hipLaunchKernelGGL(k_balance_partial, dim3(kBalWaves / 4), dim3(4 * kWave), 0, s, d, w, out_gate);
    hipLaunchKernelGGL(k_balance_final, dim3(1), dim3(kBalFinalWaves * kWave), 0, s, d, w, tau,
                       router_rows > 0 ? router_rows : kBalWaves);
    return hipGetLastError();
}

}  // namespace moepp
