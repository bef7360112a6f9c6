// Device-side pieces of the permutation (a stable counting sort of the (token,
// slot) pairs by FFN expert) that more than one kernel uses: the kernels of
// permute.hip, and the few-token router kernel that finishes with the
// permutation of its own selections.
#pragma once
#include "common.h"

namespace moepp {

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
__device__ inline void chunk_histogram(const int32_t *idx, int c, int chunk_slots, int total, int N,
                                       int lane, volatile int *cnt) {
    cnt[lane] = 0;
    const int end = min(total, (c + 1) * chunk_slots);
    for (int q0 = c * chunk_slots; q0 < end; q0 += kWave) {
        const int e = slot_expert(idx, q0 + lane, end, N);
        const unsigned long long m = same_expert_lanes(e);
        if (e >= 0 && lane == __ffsll((long long)m) - 1) cnt[e] += __popcll(m);
    }
}

// row_of / src_of of chunk c.  rank[e] (LDS, this wave's own 64 counters)
// enters with the rank, within expert e, of the chunk's first slot on e;
// first_row[e] is the first row of FFN expert e and limit[e] the capacity of
// expert e (both LDS, read only).  A slot's rank is rank[e] plus the number of
// lower lanes on the same expert; the lowest lane of the group then moves
// rank[e] past the group.
constexpr int kPermMaxRounds = 16;     // a chunk has at most 1024 slots (128 tokens x 8)

// The experts of this lane's slots of chunk c, one per round of 64 slots (-1: no
// slot): all loads are issued here, before anything waits for one.
__device__ inline void chunk_experts(const Dims &d, const int32_t *idx, int c, int chunk_slots, int lane,
                                     int (&ex)[kPermMaxRounds]) {
    const int end = min(d.T * d.k, (c + 1) * chunk_slots);
#pragma unroll
    for (int it = 0; it < kPermMaxRounds; ++it) {
        const int q = c * chunk_slots + it * kWave + lane;
        ex[it] = it * kWave < chunk_slots ? slot_expert(idx, q, end, d.N) : -1;
    }
}

__device__ inline void scatter_chunk(const Dims &d, const Workspace &w, int c, int chunk_slots, int lane,
                                     const int (&ex)[kPermMaxRounds], volatile int *rank,
                                     const int *first_row, const int *limit) {
    const int total = min(d.T * d.k, (c + 1) * chunk_slots);     // end of this chunk
    const unsigned long long lt = (1ull << lane) - 1ull;
#pragma unroll
    for (int it = 0; it < kPermMaxRounds; ++it) {
        if (it * kWave >= chunk_slots) break;
        const int q = c * chunk_slots + it * kWave + lane;
        const int e = ex[it];
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

// The three steps of the permutation in one workgroup of kPermSmallWaves waves,
// for calls with at most kPermSmallSlots slots; wave c owns chunk c.  `idx` holds
// the T*k selected experts (global memory or LDS); s_rank [kPermSmallWaves][kMaxExperts],
// s_first and s_limit [kMaxExperts] are LDS.  Every thread of the workgroup calls it.
__device__ inline void perm_small_body(const Dims &d, const Workspace &w, const CapArgs &cap, const int32_t *idx,
                                       int (*s_rank)[kMaxExperts], int *s_first, int *s_limit) {
    const int lane = threadIdx.x % kWave, c = threadIdx.x / kWave;
    const int total = d.T * d.k;
    chunk_histogram(idx, c, kPermChunk, total, d.N, lane, s_rank[c]);
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
    if (c * kPermChunk < total) {
        int ex[kPermMaxRounds];
        chunk_experts(d, idx, c, kPermChunk, lane, ex);
        scatter_chunk(d, w, c, kPermChunk, lane, ex, s_rank[c], s_first, s_limit);
    }
}

}  // namespace moepp
