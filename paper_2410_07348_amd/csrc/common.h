// Internal declarations shared by the HIP sources of libmoepp (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moepp {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kMaxExperts = 64;   // N
constexpr int kMaxTopK = 8;       // K
constexpr int kMaxConst = 8;      // constant experts
constexpr int kWave = 64;         // CDNA wavefront

// Calls with at most this many tokens take the router that splits the
// reduction over D across workgroups.
constexpr int kRouterSmallT = 256;
// ... and up to this many its second kernel also does the permutation
constexpr int kRouterFusedT = 64;

// Permutation: one wave owns a chunk of consecutive slots: kPermChunk of them,
// or the slots of one workgroup of the MFMA router when that kernel has
// counted them (at least 64 tokens).
constexpr int kPermChunk = 4 * kWave;
constexpr int kPermMinChunkTokens = 64;
// Up to this many chunks every scatter wave adds up the histogram rows itself
// (work grows with the square of the chunk count); beyond it a scan kernel does.
constexpr int kPermDirectChunks = 2048;

// Rows of W1 and W3 are interleaved in blocks of this many rows in the packed
// expert buffer: [kPackBlk rows of W1][kPackBlk rows of W3] ...
constexpr int kPackBlk = 32;

// Row of the packed W1/W3 matrix [2F, D] that holds row f of W1 (up = 0) or
// of W3 (up = 1).  The last block may be partial when F % kPackBlk != 0.
__host__ __device__ inline int packed_row(int f, int up, int F) {
    int b = f / kPackBlk;
    int rem = F - b * kPackBlk;
    int bs = rem < kPackBlk ? rem : kPackBlk;
    return b * 2 * kPackBlk + up * bs + (f - b * kPackBlk);
}

// K-slab-major storage of a matrix [N rows, K columns]: slab s holds columns
// [s*kSlab, (s+1)*kSlab) of every row, rows consecutive, so that the part of
// the matrix a GEMM tile needs for one K step (some consecutive rows x one
// slab) is one consecutive piece of memory.  The last slab is narrower when
// K % kSlab != 0.  Used for h.
constexpr int kSlab = 32;
__host__ __device__ inline int slab_width(int s, int K) {
    const int rem = K - s * kSlab;
    return rem < kSlab ? rem : kSlab;
}
// element offset of (row n, first column of slab s)
__host__ __device__ inline size_t slab_row(int n, int s, int N, int K) {
    return (size_t)s * N * kSlab + (size_t)n * slab_width(s, K);
}

// The packed expert weight matrices [N rows, K columns] are stored in panels
// of kPanel rows (the GEMM's tile height), each panel K-slab-major: all that
// one GEMM tile reads of the matrix, in the order it reads it, is one
// consecutive run of memory.  The last panel has fewer rows when
// N % kPanel != 0.  Element offset of (row n, first column of slab s):
constexpr int kPanel = 256;
__host__ __device__ inline size_t panel_row(int n, int s, int N, int K) {
    const int p = n / kPanel;
    const int rem = N - p * kPanel;
    const int rows = rem < kPanel ? rem : kPanel;
    return (size_t)p * kPanel * K + slab_row(n - p * kPanel, s, rows, K);
}

struct Dims {
    int T, D, F;
    int n_ffn, n_zero, n_copy, n_const, N;
    int k;
};

// Device pointers into the caller's workspace.
struct Workspace {
    int32_t *topk_idx;   // [T_max*k]
    float *topk_w;       // [T_max*k]
    float *alpha1;       // [T_max*n_const]
    int32_t *counts;     // [N] assignments per expert, before any drop
    int32_t *kept;       // [N] min(counts, capacity)
    int32_t *offsets;    // [n_ffn+1]
    int32_t *row_of;     // [T_max*k]
    int32_t *src_of;     // [T_max*k]
    int32_t *chunk_hist; // [n_chunks*N]
    int32_t *chunk_base; // [n_chunks*N]
    void *h;             // [T_max*k, F] act, K-slab-major
    void *yffn;          // [T_max*k, D] act
    double *bal_partial; // [kBalWaves][kMaxExperts] partial sums of Softmax(G(x))
    float *bal;          // f [N], P [N], L_b [1]  (Eq.7)
    float *router_partial; // router_small_bytes(): per-slice dot products of the few-token router
};

// Expert capacities (Eq.8), by value in the kernel arguments.  on = false: unlimited.
struct CapArgs {
    bool on;
    int32_t cap[kMaxExperts];
};

constexpr int kBalWaves = 2048;   // waves of the load-balance reduction (its partial sums)

struct RouterArgs {
    Dims d;
    const void *x;
    const float *prev_gate, *W_g, *W_res, *bias, *W_c;
    float *out_gate;
    int32_t *topk_idx;
    float *topk_w;
    float *alpha1;
    int32_t *chunk_hist;  // MFMA router: [workgroup][N] selections per expert, or null
    double *bal_partial;  // MFMA router: [workgroup][kMaxExperts] sums of Softmax(G(x))_i over the
                          // workgroup's tokens (for P_i of Eq.7), or null
};

struct FfnArgs {
    Dims d;
    const void *x;        // [T,D]
    const void *w13;      // packed: [n_ffn] matrices [2F, D] in panels (panel_row), rows in packed_row order
    const void *w2;       // packed: [n_ffn] matrices [D, F] in panels (panel_row)
    const int32_t *offsets;
    const int32_t *src_of;
    void *h;              // [h_rows, F] K-slab-major; rows < R are written
    void *yffn;           // [R,D] row-major
    int h_rows;           // T_max * k
    bool no_tail;         // tests: leave a sparsely filled last round of tiles to the main launch
};

struct CombineArgs {
    Dims d;
    const void *x, *const_vecs, *yffn;
    const int32_t *topk_idx, *row_of;
    const float *topk_w, *alpha1;
    void *out;
};

// Launchers (each returns hipGetLastError() after its launches).
// `bf16` selects the activation type; `which` selects GEMM1 / GEMM2.
hipError_t launch_router_generic(const RouterArgs &a, bool bf16, hipStream_t s);
// T <= kRouterSmallT only; partial: router_small_bytes() of scratch.  With perm_ws
// (T <= kRouterFusedT only) the second kernel also does the permutation of the
// call's T*k slots (counts, kept, offsets, row_of, src_of of *perm_ws, capacities
// *perm_cap), as launch_perm_small would.
hipError_t launch_router_small(const RouterArgs &a, bool bf16, float *partial, hipStream_t s,
                               const Workspace *perm_ws = nullptr, const CapArgs *perm_cap = nullptr);
size_t router_small_bytes();
bool router_mfma_supported(const Dims &d);
hipError_t launch_router_mfma(const RouterArgs &a, hipStream_t s);
int router_mfma_block_tokens(const Dims &d);

// chunk_slots: slots per chunk (kPermChunk, or tokens per router workgroup x k)
int perm_chunks(const Dims &d, int chunk_slots);
hipError_t launch_perm_hist(const Dims &d, const Workspace &w, int chunk_slots, hipStream_t s);
hipError_t launch_perm_scan(const Dims &d, const Workspace &w, const CapArgs &cap, int chunk_slots,
                            hipStream_t s);
hipError_t launch_perm_scatter(const Dims &d, const Workspace &w, const CapArgs &cap, int chunk_slots,
                               hipStream_t s);
// scan + scatter in one kernel; at most kPermDirectChunks chunks
hipError_t launch_perm_scan_scatter(const Dims &d, const Workspace &w, const CapArgs &cap, int chunk_slots,
                                    hipStream_t s);
// all three steps in one workgroup, for 0 < T*k <= kPermSmallSlots
constexpr int kPermSmallWaves = 16;
constexpr int kPermSmallSlots = kPermSmallWaves * kPermChunk;
hipError_t launch_perm_small(const Dims &d, const Workspace &w, const CapArgs &cap, hipStream_t s);
// f_i, P_i and L_b of Eq.7 from the logits of the routed call and the counts of the permutation.
// router_rows > 0: the router kernel has already left that many rows of per-workgroup sums of
// Softmax(G(x)) in w.bal_partial (at most kBalWaves), and only the final reduction runs.
hipError_t launch_balance(const Dims &d, const Workspace &w, const float *out_gate, float tau,
                          hipStream_t s, int router_rows = 0);

hipError_t launch_ffn_generic(const FfnArgs &a, bool bf16, int which, hipStream_t s);
bool ffn_mfma_supported(const Dims &d);
hipError_t launch_ffn_mfma(const FfnArgs &a, int which, hipStream_t s);

// few rows per expert (T * k <= 16 n_ffn): weight-streaming kernels
bool ffn_decode_supported(const Dims &d);
hipError_t launch_ffn_decode(const FfnArgs &a, int which, hipStream_t s);

hipError_t launch_combine(const CombineArgs &a, bool bf16, hipStream_t s);

hipError_t launch_pack(const Dims &d, bool bf16, const void *w1, const void *w3,
                       const void *w2, void *w13_out, void *w2_out, hipStream_t s);

hipError_t launch_mfma_ceiling(float *scratch, int iters, hipStream_t s);
double mfma_ceiling_flops(int iters);
size_t mfma_ceiling_scratch_bytes();
hipError_t launch_stream(void *buf, size_t bytes, int mode, hipStream_t s);

// ---- small device helpers -------------------------------------------------
// Workgroup barrier that orders LDS accesses only: global loads (including
// loads that write LDS directly, which the caller waits for with vmcnt) stay
// in flight across it, unlike __syncthreads().
__device__ inline void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

__device__ inline float to_f32(float v) { return v; }
__device__ inline float to_f32(bf16_t v) { return (float)v; }

template <typename T> struct ActVec;   // 16 bytes of activations
template <> struct ActVec<float> {
    static constexpr int N = 4;
    f32x4 v;
    __device__ float get(int i) const { return v[i]; }
    __device__ void set(int i, float f) { v[i] = f; }
};
template <> struct ActVec<bf16_t> {
    static constexpr int N = 8;
    bf16x8 v;
    __device__ float get(int i) const { return (float)v[i]; }
    __device__ void set(int i, float f) { v[i] = (bf16_t)f; }
};

template <typename T>
__device__ inline ActVec<T> load_vec(const T *p) {
    ActVec<T> r;
    r.v = *reinterpret_cast<const decltype(r.v) *>(p);
    return r;
}
template <typename T>
__device__ inline void store_vec(T *p, const ActVec<T> &r) {
    *reinterpret_cast<decltype(r.v) *>(p) = r.v;
}
// The same with the non-temporal hint, for data this library does not touch
// again (a layer's output) or reads exactly once (a row of the FFN output):
// such lines then do not displace, or sit dirty in, the caches that the
// following kernels read through (measured: the router that follows a combine
// runs 20 % faster).
template <typename T>
__device__ inline ActVec<T> load_vec_stream(const T *p) {
    ActVec<T> r;
    r.v = __builtin_nontemporal_load(reinterpret_cast<const decltype(r.v) *>(p));
    return r;
}
template <typename T>
__device__ inline void store_vec_stream(T *p, const ActVec<T> &r) {
    __builtin_nontemporal_store(r.v, reinterpret_cast<decltype(r.v) *>(p));
}

}  // namespace moepp
