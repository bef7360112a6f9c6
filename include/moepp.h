/*
 * moepp.h - C ABI of the MI355X (gfx950) forward pass of one MoE++ layer.
 *
 * The layer (arXiv 2410.07348, Sec. 3) maps (x^j, G(x^{j-1})) to
 * (y^j, G(x^j)):
 *
 *   G(x)  = W x  (+ W_g G(x_prev) for layers j > 1)              Eq.2, Eq.6
 *   g_i   = Softmax(G(x))_i if G(x)_i is among the Top-K, else 0   Eq.1
 *   y     = sum_i g_i E_i(x)                                       Eq.1
 *   E_i   = FFN_i | 0 (zero) | x (copy) | a1 x + a2 v (constant),
 *           [a1,a2] = Softmax(W_c x)                               Eq.2-5
 *
 * Expert index order inside the N-way softmax (N = n_ffn + n_zero + n_copy +
 * n_const): FFN experts first, then zero, copy and constant experts.  An FFN
 * expert is a bias-free SwiGLU, W2 (silu(W1 x) * (W3 x)).  Gate weights are
 * the softmax over all N experts (not renormalised over the selected K);
 * Top-K is taken on the float32 logits, ties go to the lower index and the K
 * slots of a token are ordered by descending logit.
 *
 * Conventions
 *  - Every data pointer is a DEVICE pointer owned by the caller, contiguous,
 *    row-major and 16-byte aligned, unless a parameter says "host".
 *  - The library never allocates or frees device memory: scratch space is the
 *    caller's workspace (size from moepp_workspace_bytes).
 *  - `stream` is a hipStream_t passed as void*; all work is enqueued on it
 *    asynchronously and no call synchronises with the host, except
 *    moepp_get_timing.
 *  - No exception crosses the boundary.  Every call returns a moepp_status;
 *    arguments are validated before anything is launched, so MOEPP_EINVAL,
 *    MOEPP_EUNSUPPORTED and MOEPP_ENOMEM can be provoked on a machine without
 *    a GPU.  A HIP launch error is returned as MOEPP_EHIP.
 *  - Calls on one context must not overlap (they share its workspace).
 */
#ifndef MOEPP_H
#define MOEPP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moepp_ctx moepp_ctx; /* opaque; host bookkeeping only */

typedef enum {
    MOEPP_OK = 0,
    MOEPP_EINVAL = -1,       /* bad argument: null, misaligned, out of range   */
    MOEPP_EUNSUPPORTED = -2, /* valid request outside the implemented limits   */
    MOEPP_ENOMEM = -3,       /* caller's buffer is smaller than required       */
    MOEPP_EHIP = -4          /* the HIP runtime reported an error              */
} moepp_status;

typedef enum {
    MOEPP_F32 = 0, /* activations and expert weights float32 */
    MOEPP_BF16 = 1 /* activations and expert weights bfloat16; router-side
                      tensors stay float32, accumulation is float32 */
} moepp_dtype;

/*
 * Static description of a layer.  Limits: 1 <= k <= min(N, 8), N <= 64,
 * n_const <= 8, D % 8 == 0, F % 8 == 0, 1 <= T_max, T_max * k < 2^30.
 */
typedef struct {
    int32_t T_max;   /* largest token count of a forward call                 */
    int32_t D;       /* hidden size                                           */
    int32_t F;       /* SwiGLU intermediate size                              */
    int32_t n_ffn;   /* FFN experts (may be 0)                                */
    int32_t n_zero;  /* zero experts,     Eq.3                                */
    int32_t n_copy;  /* copy experts,     Eq.4                                */
    int32_t n_const; /* constant experts, Eq.5                                */
    int32_t k;       /* experts activated per token (Top-K of Eq.1)           */
    int32_t act;     /* moepp_dtype of x, out, expert weights, const_vecs     */
} moepp_desc;

/* Logical expert weights: w1, w3 [n_ffn][F][D], w2 [n_ffn][D][F], act type. */
typedef struct {
    const void *w1;
    const void *w3;
    const void *w2;
} moepp_experts;

/* Bytes of workspace a context for `desc` needs; 0 if desc is invalid. */
size_t moepp_workspace_bytes(const moepp_desc *desc);

/* Bytes of the packed expert buffer for `desc`; 0 if desc is invalid. */
size_t moepp_packed_bytes(const moepp_desc *desc);

/*
 * Create a context over a caller-owned device workspace (256-byte aligned,
 * at least moepp_workspace_bytes(desc) bytes, alive until moepp_destroy).
 * Host-only: touches neither the workspace nor the GPU.
 * EINVAL: null pointer, invalid desc, misaligned workspace.
 * EUNSUPPORTED: desc outside the limits above.  ENOMEM: bytes too small.
 */
moepp_status moepp_create(const moepp_desc *desc, void *workspace, size_t bytes,
                          moepp_ctx **ctx);
moepp_status moepp_destroy(moepp_ctx *ctx);

/*
 * One-time repacking of the FFN expert weights into the layout the FFN
 * kernels read (weights are static across forward calls, so this is not part
 * of the forward pass): W1 and W3 of an expert are interleaved in blocks of
 * 32 rows ([32 rows of W1][32 rows of W3]...) so that one output tile holds
 * silu's argument and its multiplier for the same columns, and every matrix
 * is stored in panels of 256 rows, each panel in slabs of 32 columns (slab s
 * = columns 32s..32s+31 of the panel's rows, rows consecutive), so that what
 * a GEMM tile reads of a weight matrix is one consecutive run of memory, in
 * the order it is read.  The packed layout is private to the library.
 * `packed` must hold moepp_packed_bytes(desc) bytes (ENOMEM otherwise).
 */
moepp_status moepp_pack_experts(moepp_ctx *ctx, void *stream,
                                const moepp_experts *experts, void *packed,
                                size_t bytes);

/*
 * Optional additive per-expert router bias, bias[N] float32 on the device
 * (NULL = none, the default).  Not part of the paper; the benchmark's ragged
 * and skewed workloads use it.  It is added to G(x) before softmax / Top-K
 * and is included in out_gate.  The pointer is kept, not copied.
 */
moepp_status moepp_set_router_bias(moepp_ctx *ctx, const float *bias);

/*
 * Forward pass of the layer for T tokens (0 <= T <= T_max); the whole path of
 * Eq.1-6.  Equivalent to moepp_route, moepp_permute, moepp_expert_ffn and
 * moepp_combine in that order.
 *
 *   x          [T,D]          act      input tokens x^j
 *   prev_gate  [T,N]          float32  G(x^{j-1}), or NULL for the first layer
 *   W_g        [N,D]          float32  router matrix (the paper's W^j)
 *   W_res      [N,N]          float32  gating-residual matrix (the paper's
 *                                      W_g^j); NULL iff prev_gate is NULL
 *   experts                   act      buffer written by moepp_pack_experts
 *   const_vecs [n_const,D]    act      v of each constant expert
 *   W_c        [n_const,2,D]  float32  W_c of each constant expert
 *   k                                  1 <= k <= desc.k
 *   out        [T,D]          act      y^j
 *   out_gate   [T,N]          float32  G(x^j), residual (and bias) included
 *
 * const_vecs / W_c may be NULL iff n_const == 0; experts may be NULL iff
 * n_ffn == 0.  EINVAL on null / misaligned pointers, T or k out of range,
 * prev_gate / W_res not given together.  T == 0 is a no-op that reads no
 * pointer (they may all be NULL).
 */
moepp_status moepp_layer_forward(moepp_ctx *ctx, void *stream, int32_t T,
                                 const void *x, const float *prev_gate,
                                 const float *W_g, const float *W_res,
                                 const void *experts, const void *const_vecs,
                                 const float *W_c, int32_t k, void *out,
                                 float *out_gate);

/*
 * moepp_layer_forward for callers that cannot allocate device memory and have
 * no workspace to bring: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments and results as
 * moepp_layer_forward on a fresh context for `desc` (automatic kernel choice,
 * no router bias, no capacities, no statistics, no timing), but the scratch
 * space is an array of MOEPP_STATIC_SCRATCH_BYTES that the library holds in
 * the memory of every GPU it runs on, from the first use of the library on
 * that GPU until the process ends.  The call allocates and frees nothing, on
 * the device or through any library, and keeps no state between calls.
 * ENOMEM: moepp_workspace_bytes(desc) exceeds MOEPP_STATIC_SCRATCH_BYTES (size
 * desc.T_max for the call: at D = 4096, F = 5632, k = 2 the limit is reached
 * near T_max = 1000).  EHIP: the array's address on the current device could
 * not be obtained.  Other errors as moepp_layer_forward.  All calls on one
 * GPU share that GPU's array: calls that overlap in time on one GPU (other
 * streams, other threads) race on it, and the array keeps what the last call
 * left (every kernel writes what it later reads, nothing needs to start at
 * zero).  The first call on a GPU asks the runtime for the array's address on
 * that GPU (once per GPU; the runtime may set the array up at that moment), so
 * make one call on each GPU before capturing a graph.  moepp_get_routing and
 * the other state queries do not apply.
 */
#define MOEPP_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
moepp_status moepp_layer_forward_static(const moepp_desc *desc, void *stream, int32_t T,
                                        const void *x, const float *prev_gate,
                                        const float *W_g, const float *W_res,
                                        const void *experts, const void *const_vecs,
                                        const float *W_c, int32_t k, void *out,
                                        float *out_gate);

/*
 * The four steps of moepp_layer_forward as separate calls (same argument
 * meaning).  Each reads what the previous step left in the workspace.
 *
 * moepp_route: router GEMM + gating residual (Eq.2, Eq.6), softmax and Top-K
 *   (Eq.1), and a1 of every constant expert (Eq.5).  Writes out_gate and, in
 *   the workspace, topk_idx, topk_w, alpha1.
 * moepp_permute: groups the (token, slot) pairs by FFN expert: histogram,
 *   exclusive scan, stable scatter.  Writes counts, offsets, row_of, src_of.
 * moepp_expert_ffn: grouped SwiGLU FFN over the rows of every FFN expert
 *   (the FFN_i of Eq.2); writes h [R,F] and yffn [R,D] in the workspace.
 * moepp_combine: y = sum over the K slots of g * E(x) (Eq.1) with the zero,
 *   copy and constant experts (Eq.3-5) evaluated in place.
 */
moepp_status moepp_route(moepp_ctx *ctx, void *stream, int32_t T, const void *x,
                         const float *prev_gate, const float *W_g,
                         const float *W_res, const float *W_c, int32_t k,
                         float *out_gate);
moepp_status moepp_permute(moepp_ctx *ctx, void *stream, int32_t T, int32_t k);
moepp_status moepp_expert_ffn(moepp_ctx *ctx, void *stream, int32_t T,
                              const void *x, const void *experts, int32_t k);
moepp_status moepp_combine(moepp_ctx *ctx, void *stream, int32_t T,
                           const void *x, const void *const_vecs, int32_t k,
                           void *out);

/*
 * Device pointers (into the workspace) to the routing state left by the last
 * forward / route / permute call on `ctx`; valid until the next one.  Any
 * output pointer may be NULL.  With T and k of that call:
 *   topk_idx [T,k] int32   selected experts, descending logit
 *   topk_w   [T,k] float32 their gate weights g_i
 *   counts   [N]   int32   slots per expert (sum = T*k), before any drop
 *   offsets  [n_ffn+1] int32  exclusive scan of the kept slots (= counts
 *                             without capacities) over the FFN experts;
 *                             offsets[n_ffn] = R = rows that reach an FFN
 *   row_of   [T*k] int32   row in [0,R) of slot t*k+s, -1 for zero-computation
 *                          experts, -2 for a slot dropped by an expert capacity
 *   src_of   [T*k] int32   first R entries: the slot t*k+s of each row; rows of
 *                          one expert are in ascending slot order
 */
moepp_status moepp_get_routing(moepp_ctx *ctx, const int32_t **topk_idx,
                               const float **topk_w, const int32_t **counts,
                               const int32_t **offsets, const int32_t **row_of,
                               const int32_t **src_of);

/*
 * Device pointers to intermediates of the last call: alpha1 [T,n_const]
 * float32 (a1 of Eq.5), h (SwiGLU intermediate, rows in the order of src_of)
 * and yffn [R,D] act row-major (FFN expert outputs).  h is stored in slabs
 * of 32 columns over T_max*k rows: element (r, f) is at
 * (f/32)*(T_max*k)*32 + r*w + f%32 with w = min(32, F - 32*(f/32)); rows
 * r < R hold data.  Any pointer may be NULL.
 */
moepp_status moepp_get_intermediates(moepp_ctx *ctx, const float **alpha1,
                                     const void **h, const void **yffn);

/*
 * Per-kernel timing.  With timing enabled, every call records HIP events on
 * its stream around each kernel it launches (up to 64 calls are kept, later
 * ones overwrite the oldest).  moepp_get_timing waits for the recorded events
 * (host synchronisation), writes into ms[MOEPP_NUM_KERNELS] (host array) the
 * duration in milliseconds of each kernel averaged over the calls recorded
 * since timing was enabled or last read (0 for kernels that did not run), and
 * starts a new average.
 */
enum {
    MOEPP_K_ROUTER = 0,  /* router GEMM + residual + softmax + top-k         */
    MOEPP_K_HIST = 1,    /* permute: per-chunk histogram; 0 when the router kernel
                            has counted its own selections (bf16 layers on the
                            matrix-core router) and for calls with at most 4096
                            slots, where one kernel does all three steps and is
                            reported as MOEPP_K_SCATTER                       */
    MOEPP_K_SCAN = 2,    /* permute: exclusive scan as a kernel of its own; 0 up to
                            2048 chunks (scan and scatter are one kernel)    */
    MOEPP_K_SCATTER = 3, /* permute: (scan and) stable scatter; 0 for calls with at
                            most 64 tokens on the automatic variant, where the
                            router's second kernel also groups the slots and the
                            time is part of MOEPP_K_ROUTER                    */
    MOEPP_K_GEMM1 = 4,   /* grouped GEMM W1/W3 + SwiGLU                       */
    MOEPP_K_GEMM2 = 5,   /* grouped GEMM W2                                   */
    MOEPP_K_COMBINE = 6, /* weighted combine + zero-computation experts       */
    MOEPP_K_BALANCE = 7, /* load-balance statistics (only when switched on)    */
    MOEPP_NUM_KERNELS = 8
};
moepp_status moepp_set_timing(moepp_ctx *ctx, int32_t enable);
moepp_status moepp_get_timing(moepp_ctx *ctx, float *ms);

/*
 * Expert capacity (Sec. 3.3, Eq.8).  moepp_capacity is host arithmetic: it
 * writes into cap_host[N] (host array)
 *   C_i = ceil(gamma * tau * S / (tau N_FFN + N_ZC))   for an FFN expert,
 *   C_i = ceil(gamma * S / (tau N_FFN + N_ZC))         for a zero-computation expert.
 * per_assignment != 0 (the reading this library's benchmark and tests use):
 * S = T * k, the number of (token, slot) assignments of a call; with T itself
 * the capacities add up to gamma*T places for k*T assignments.
 * per_assignment == 0: S = T, the number of tokens, Eq.8 as it is printed
 * (capacities k times smaller).  A value that exceeds an integer by less than
 * 1e-9 relative counts as that integer.
 * EINVAL: null pointer, T or k outside the descriptor, gamma or tau not positive.
 *
 * moepp_set_capacity copies cap_host[N] into the context (NULL switches the
 * capacities off, the default).  From then on moepp_permute and
 * moepp_layer_forward let expert i keep only the first cap_host[i] of its
 * assignments in (token, slot) order; the others are dropped: they get
 * row_of = -2, reach no GEMM and add nothing to `out` (the token continues
 * through the residual connection around the layer); gate weights are not
 * renormalised.  counts (moepp_get_routing) stay the numbers before the drop,
 * moepp_get_kept gives min(counts, cap) [N] int32 on the device, offsets
 * are the prefix sums of the kept FFN rows.  EINVAL: a negative capacity.
 */
moepp_status moepp_capacity(const moepp_desc *desc, int32_t T, int32_t k, double gamma,
                            double tau, int32_t per_assignment, int32_t *cap_host);
moepp_status moepp_set_capacity(moepp_ctx *ctx, const int32_t *cap_host);
moepp_status moepp_get_kept(moepp_ctx *ctx, const int32_t **kept);

/*
 * Heterogeneous load-balance statistics (Sec. 3.3, Eq.7), by-products of the
 * routing: f_i = fraction of the tokens that selected expert i (before any
 * drop), P_i = mean of Softmax(G(x))_i over the tokens, L_b = sum_i eta_i
 * f_i P_i with eta_i = 1 for FFN experts and tau for zero-computation
 * experts.  moepp_set_balance(tau > 0) switches them on (tau <= 0: off, the
 * default); moepp_permute / moepp_layer_forward then compute them after the
 * permutation from the logits of the routed call the permutation belongs to
 * (out_gate of that call must still be intact; moepp_permute without a
 * preceding moepp_route of the same T is EINVAL while they are on).
 * moepp_get_balance returns device pointers: f [N], P [N], loss [1] float32.
 */
moepp_status moepp_set_balance(moepp_ctx *ctx, double tau);
moepp_status moepp_get_balance(moepp_ctx *ctx, const float **f, const float **P,
                               const float **loss);

/*
 * Kernel-variant selection, for tests and tuning: 0 = automatic (default;
 * calls with at most 256 tokens use a router that splits the reduction over
 * D across workgroups, in plain fp32 FMA, for either activation type),
 * 1 = force the generic kernels (any supported shape, plain fp32 FMA),
 * 2 = require the MFMA kernels (EUNSUPPORTED at call time if the shape or
 * type has none), 3 = as 2, and the grouped GEMM leaves a sparsely filled last
 * round of tiles to its main launch instead of a second launch with tiles of
 * half the height (same results bit for bit; lets a test compare the two).
 */
moepp_status moepp_set_variant(moepp_ctx *ctx, int32_t variant);

/*
 * Measurement aid, not part of the layer: enqueues a kernel that does nothing
 * but bf16 MFMAs on pseudo-random register operands (2 waves per SIMD, no
 * memory traffic) and writes the number of floating-point operations it
 * performs to *flops (host).  Timed by the caller, it gives the matrix rate
 * this GPU sustains on real operand bits, which is below the published peak
 * because the clock drops under matrix load.  `scratch` is a device buffer of
 * at least 512 KiB (ENOMEM if smaller); iters >= 1 (about 0.1 ms per 200).
 */
moepp_status moepp_mfma_ceiling(void *stream, void *scratch, size_t scratch_bytes,
                                int32_t iters, double *flops);

/*
 * Measurement aid, not part of the layer: enqueues a kernel that only moves
 * data with 16-byte accesses, whole 1 KB pieces per wave: mode 0 reads `bytes`
 * of `buf`, mode 1 copies the first half of `buf` over the second half.
 * *moved_bytes (host) = bytes read + bytes written.  Timed by the caller, it
 * gives the rate the memory system delivers to a kernel that does nothing
 * else, which is below the published 8 TB/s.  bytes: a multiple of 32 KiB, at
 * least 64 MiB (use more than the 256 MB of the memory-side cache).
 * EINVAL otherwise, and for null / misaligned buf.
 */
moepp_status moepp_stream_ceiling(void *stream, void *buf, size_t bytes, int32_t mode,
                                  double *moved_bytes);

/* Text of a status code (any integer: unknown values give "unknown status"). */
const char *moepp_status_str(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* MOEPP_H */
