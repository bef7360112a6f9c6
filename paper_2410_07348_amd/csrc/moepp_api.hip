// Host side of libmoepp: the extern "C" boundary declared in include/moepp.h.
// Argument validation, workspace partitioning and kernel dispatch; no
// arithmetic of the layer happens on the host.
#include "../../include/moepp.h"
#include "common.h"

#include <math.h>

#include <mutex>
#include <new>

using namespace moepp;

constexpr int kTimingSlots = 64;

struct moepp_ctx {
    moepp_desc desc;
    Workspace ws;
    size_t ws_bytes;
    const float *bias;
    int variant;          // 0 auto, 1 generic, 2 require MFMA, 3 as 2 without the GEMM tail launch
    CapArgs cap;          // expert capacities (Eq.8); cap.on = false: unlimited
    double bal_tau;       // > 0: collect the load-balance statistics (Eq.7) with this tau
    const float *last_out_gate;   // logits of the last routed call (read by the statistics)
    int last_T, last_k;
    // the MFMA router leaves a histogram per workgroup for the permutation of the same call
    int bal_rows;         // > 0: the router kernel of call (bal_T) left this many rows of Softmax sums
    int bal_T;
    bool perm_valid;      // the few-token router kernel has already grouped the slots of call (perm_T, perm_k)
    int perm_T, perm_k;
    bool hist_valid;
    int hist_T, hist_k, hist_chunk_slots;
    bool timing;
    bool have_events;
    // ring of event pairs: one slot per recorded call
    hipEvent_t ev[kTimingSlots][MOEPP_NUM_KERNELS][2];
    bool ran[kTimingSlots][MOEPP_NUM_KERNELS];
    int slot;             // slot of the call being recorded
    int n_recorded;       // calls recorded since the last moepp_get_timing
};

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

int n_experts(const moepp_desc *d) { return d->n_ffn + d->n_zero + d->n_copy + d->n_const; }
size_t elt(const moepp_desc *d) { return d->act == MOEPP_BF16 ? 2 : 4; }

// 0 = ok, else the status to return
moepp_status check_desc(const moepp_desc *d) {
    if (!d) return MOEPP_EINVAL;
    if (d->T_max < 1 || d->D < 1 || d->F < 1 || d->n_ffn < 0 || d->n_zero < 0 ||
        d->n_copy < 0 || d->n_const < 0 || d->k < 1)
        return MOEPP_EINVAL;
    if (d->act != MOEPP_F32 && d->act != MOEPP_BF16) return MOEPP_EINVAL;
    const long long N = (long long)d->n_ffn + d->n_zero + d->n_copy + d->n_const;
    if (N < 1 || d->k > N) return MOEPP_EINVAL;
    if (N > kMaxExperts || d->k > kMaxTopK || d->n_const > kMaxConst) return MOEPP_EUNSUPPORTED;
    if (d->D % 8 != 0 || d->F % 8 != 0) return MOEPP_EUNSUPPORTED;
    if ((long long)d->T_max * d->k >= (1ll << 30)) return MOEPP_EUNSUPPORTED;
    return MOEPP_OK;
}

// Lays the workspace out from `base` (may be null to size it); returns bytes.
size_t layout(const moepp_desc *d, char *base, Workspace *ws) {
    const size_t N = n_experts(d);
    const size_t slots = (size_t)d->T_max * d->k;
    // chunks of the permutation: kPermChunk slots each, or one per router workgroup
    const size_t by_slots = (slots + kPermChunk - 1) / kPermChunk;
    const size_t by_tokens = ((size_t)d->T_max + kPermMinChunkTokens - 1) / kPermMinChunkTokens;
    const size_t chunks = by_slots > by_tokens ? by_slots : by_tokens;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += align_up(bytes);
        return p;
    };
    Workspace w;
    w.topk_idx = (int32_t *)take(slots * 4);
    w.topk_w = (float *)take(slots * 4);
    w.alpha1 = (float *)take((size_t)d->T_max * (d->n_const ? d->n_const : 1) * 4);
    w.counts = (int32_t *)take(N * 4);
    w.kept = (int32_t *)take(N * 4);
    w.offsets = (int32_t *)take(((size_t)d->n_ffn + 1) * 4);
    w.row_of = (int32_t *)take(slots * 4);
    w.src_of = (int32_t *)take(slots * 4);
    w.chunk_hist = (int32_t *)take(chunks * N * 4);
    w.chunk_base = (int32_t *)take(chunks * N * 4);
    w.h = take(d->n_ffn ? slots * d->F * elt(d) : 0);
    w.yffn = take(d->n_ffn ? slots * d->D * elt(d) : 0);
    w.bal_partial = (double *)take((size_t)kBalWaves * kMaxExperts * sizeof(double));
    w.bal = (float *)take((2 * N + 1) * 4);
    w.router_partial = (float *)take(router_small_bytes());
    if (ws) *ws = w;
    return off;
}

bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

Dims dims_of(const moepp_ctx *c, int T, int k) {
    Dims d;
    d.T = T;
    d.D = c->desc.D;
    d.F = c->desc.F;
    d.n_ffn = c->desc.n_ffn;
    d.n_zero = c->desc.n_zero;
    d.n_copy = c->desc.n_copy;
    d.n_const = c->desc.n_const;
    d.N = n_experts(&c->desc);
    d.k = k;
    return d;
}

moepp_status check_call(const moepp_ctx *c, int T, int k) {
    if (!c) return MOEPP_EINVAL;
    if (T < 0 || T > c->desc.T_max) return MOEPP_EINVAL;
    if (k < 1 || k > c->desc.k) return MOEPP_EINVAL;
    return MOEPP_OK;
}

struct KernelTimer {
    moepp_ctx *c;
    hipStream_t s;
    int which;
    KernelTimer(moepp_ctx *c_, hipStream_t s_, int which_) : c(c_), s(s_), which(which_) {
        if (c->timing && c->have_events) {
            (void)hipEventRecord(c->ev[c->slot][which][0], s);
        }
    }
    ~KernelTimer() {
        if (c->timing && c->have_events) {
            (void)hipEventRecord(c->ev[c->slot][which][1], s);
            c->ran[c->slot][which] = true;
        }
    }
};

// Start recording a new call: take the next slot of the ring.
void reset_ran(moepp_ctx *c) {
    if (!(c->timing && c->have_events)) return;
    c->slot = (c->slot + 1) % kTimingSlots;
    if (c->n_recorded < kTimingSlots) c->n_recorded += 1;
    for (int i = 0; i < MOEPP_NUM_KERNELS; ++i) c->ran[c->slot][i] = false;
}

void clear_timing(moepp_ctx *c) {
    c->slot = kTimingSlots - 1;
    c->n_recorded = 0;
    for (int q = 0; q < kTimingSlots; ++q)
        for (int i = 0; i < MOEPP_NUM_KERNELS; ++i) c->ran[q][i] = false;
}

bool use_mfma_router(const moepp_ctx *c, const Dims &d, moepp_status *st) {
    const bool ok = c->desc.act == MOEPP_BF16 && router_mfma_supported(d);
    if (c->variant >= 2 && !ok) *st = MOEPP_EUNSUPPORTED;
    return ok && c->variant != 1;
}
bool use_mfma_ffn(const moepp_ctx *c, const Dims &d, moepp_status *st) {
    const bool ok = c->desc.act == MOEPP_BF16 && ffn_mfma_supported(d);
    if (c->variant >= 2 && !ok) *st = MOEPP_EUNSUPPORTED;
    return ok && c->variant != 1;
}

const void *packed_w2(const moepp_ctx *c, const void *packed) {
    const size_t w13 = (size_t)c->desc.n_ffn * 2 * c->desc.F * c->desc.D * elt(&c->desc);
    return (const char *)packed + w13;
}

// ---- the four steps, arguments already validated ---------------------------
moepp_status do_route(moepp_ctx *c, hipStream_t s, int T, const void *x, const float *prev_gate,
                      const float *W_g, const float *W_res, const float *W_c, int k,
                      float *out_gate) {
    RouterArgs a;
    a.d = dims_of(c, T, k);
    a.x = x;
    a.prev_gate = prev_gate;
    a.W_g = W_g;
    a.W_res = W_res;
    a.bias = c->bias;
    a.W_c = W_c;
    a.out_gate = out_gate;
    a.topk_idx = c->ws.topk_idx;
    a.topk_w = c->ws.topk_w;
    a.alpha1 = c->ws.alpha1;
    a.chunk_hist = nullptr;
    a.bal_partial = nullptr;
    moepp_status st = MOEPP_OK;
    const bool mfma = use_mfma_router(c, a.d, &st);
    if (st != MOEPP_OK) return st;
    c->last_T = T;
    c->last_k = k;
    c->last_out_gate = out_gate;
    c->hist_valid = false;
    c->perm_valid = false;
    c->bal_rows = 0;
    if (T == 0) return MOEPP_OK;
    KernelTimer kt(c, s, MOEPP_K_ROUTER);
    const bool bf16 = c->desc.act == MOEPP_BF16;
    hipError_t e;
    if (c->variant == 0 && T <= kRouterFusedT) {
        // a handful of tokens: the router's second kernel also groups the slots by expert
        e = launch_router_small(a, bf16, c->ws.router_partial, s, &c->ws, &c->cap);
        c->perm_valid = e == hipSuccess;
        c->perm_T = T;
        c->perm_k = k;
    } else if (c->variant == 0 && T <= kRouterSmallT) {
        e = launch_router_small(a, bf16, c->ws.router_partial, s);
    } else if (mfma) {
        // the permutation of a call with few slots runs in one workgroup and counts for itself
        if ((long long)T * k > kPermSmallSlots) {
            a.chunk_hist = c->ws.chunk_hist;
            c->hist_valid = true;
            c->hist_T = T;
            c->hist_k = k;
            c->hist_chunk_slots = router_mfma_block_tokens(a.d) * k;
        }
        // with the load-balance statistics on, the kernel also adds up the softmax of its tokens
        const int tok = router_mfma_block_tokens(a.d);
        const int wgs = (T + tok - 1) / tok;
        if (c->bal_tau > 0.0 && wgs <= kBalWaves) {
            a.bal_partial = c->ws.bal_partial;
            c->bal_rows = wgs;
            c->bal_T = T;
        }
        e = launch_router_mfma(a, s);
    } else {
        e = launch_router_generic(a, bf16, s);
    }
    return e == hipSuccess ? MOEPP_OK : MOEPP_EHIP;
}

moepp_status do_permute(moepp_ctx *c, hipStream_t s, int T, int k) {
    const Dims d = dims_of(c, T, k);
    c->last_T = T;
    c->last_k = k;
    hipError_t e = hipSuccess;
    if (T > 0 && T * k <= kPermSmallSlots) {
        // (nothing to do when the router kernel of this very call has done it; the
        // capacities it used are still the current ones, see moepp_set_capacity)
        if (!(c->perm_valid && c->perm_T == T && c->perm_k == k)) {
            KernelTimer kt(c, s, MOEPP_K_SCATTER);
            e = launch_perm_small(d, c->ws, c->cap, s);
        }
        if (e != hipSuccess) return MOEPP_EHIP;
        if (c->bal_tau > 0.0) {
            KernelTimer kt(c, s, MOEPP_K_BALANCE);
            e = launch_balance(d, c->ws, c->last_out_gate, (float)c->bal_tau, s,
                               c->bal_rows > 0 && c->bal_T == T ? c->bal_rows : 0);
        }
        return e == hipSuccess ? MOEPP_OK : MOEPP_EHIP;
    }
    // chunks: the router's workgroups when it has counted this call's selections
    const bool counted = c->hist_valid && c->hist_T == T && c->hist_k == k;
    const int chunk_slots = counted ? c->hist_chunk_slots : kPermChunk;
    c->hist_valid = false;
    if (!counted) {
        KernelTimer kt(c, s, MOEPP_K_HIST);
        e = launch_perm_hist(d, c->ws, chunk_slots, s);
        if (e != hipSuccess) return MOEPP_EHIP;
    }
    if (perm_chunks(d, chunk_slots) <= kPermDirectChunks) {
        KernelTimer kt(c, s, MOEPP_K_SCATTER);
        e = launch_perm_scan_scatter(d, c->ws, c->cap, chunk_slots, s);
    } else {
        {
            KernelTimer kt(c, s, MOEPP_K_SCAN);
            e = launch_perm_scan(d, c->ws, c->cap, chunk_slots, s);
        }
        if (e != hipSuccess) return MOEPP_EHIP;
        KernelTimer kt(c, s, MOEPP_K_SCATTER);
        e = launch_perm_scatter(d, c->ws, c->cap, chunk_slots, s);
    }
    if (e != hipSuccess) return MOEPP_EHIP;
    if (c->bal_tau > 0.0 && T > 0) {
        KernelTimer kt(c, s, MOEPP_K_BALANCE);
        e = launch_balance(d, c->ws, c->last_out_gate, (float)c->bal_tau, s,
                           c->bal_rows > 0 && c->bal_T == T ? c->bal_rows : 0);
    }
    return e == hipSuccess ? MOEPP_OK : MOEPP_EHIP;
}

moepp_status do_ffn(moepp_ctx *c, hipStream_t s, int T, const void *x, const void *experts,
                    int k) {
    FfnArgs a;
    a.d = dims_of(c, T, k);
    moepp_status st = MOEPP_OK;
    const bool mfma = use_mfma_ffn(c, a.d, &st);
    if (st != MOEPP_OK) return st;
    if (T == 0 || a.d.n_ffn == 0) return MOEPP_OK;
    a.x = x;
    a.w13 = experts;
    a.w2 = packed_w2(c, experts);
    a.offsets = c->ws.offsets;
    a.src_of = c->ws.src_of;
    a.h = c->ws.h;
    a.yffn = c->ws.yffn;
    a.h_rows = c->desc.T_max * c->desc.k;
    a.no_tail = c->variant == 3;
    const bool bf = c->desc.act == MOEPP_BF16;
    // a handful of rows per expert: the kernels that only stream the weights
    // (variant 3 keeps the tiled kernels, so that tests can compare the two)
    const bool decode = mfma && c->variant != 3 && ffn_decode_supported(a.d);
    hipError_t e;
    {
        KernelTimer kt(c, s, MOEPP_K_GEMM1);
        e = decode ? launch_ffn_decode(a, 0, s) : mfma ? launch_ffn_mfma(a, 0, s) : launch_ffn_generic(a, bf, 0, s);
    }
    if (e != hipSuccess) return MOEPP_EHIP;
    {
        KernelTimer kt(c, s, MOEPP_K_GEMM2);
        e = decode ? launch_ffn_decode(a, 1, s) : mfma ? launch_ffn_mfma(a, 1, s) : launch_ffn_generic(a, bf, 1, s);
    }
    return e == hipSuccess ? MOEPP_OK : MOEPP_EHIP;
}

moepp_status do_combine(moepp_ctx *c, hipStream_t s, int T, const void *x, const void *const_vecs,
                        int k, void *out) {
    if (T == 0) return MOEPP_OK;
    CombineArgs a;
    a.d = dims_of(c, T, k);
    a.x = x;
    a.const_vecs = const_vecs;
    a.yffn = c->ws.yffn;
    a.topk_idx = c->ws.topk_idx;
    a.row_of = c->ws.row_of;
    a.topk_w = c->ws.topk_w;
    a.alpha1 = c->ws.alpha1;
    a.out = out;
    KernelTimer kt(c, s, MOEPP_K_COMBINE);
    hipError_t e = launch_combine(a, c->desc.act == MOEPP_BF16, s);
    return e == hipSuccess ? MOEPP_OK : MOEPP_EHIP;
}

// T == 0: nothing to compute and no pointer is read
moepp_status note_empty_call(moepp_ctx *c, int k) {
    c->last_T = 0;
    c->last_k = k;
    reset_ran(c);
    return MOEPP_OK;
}

moepp_status check_route_args(const moepp_ctx *c, const void *x, const float *prev_gate,
                              const float *W_g, const float *W_res, const float *W_c,
                              const float *out_gate) {
    if (!x || !W_g || !out_gate) return MOEPP_EINVAL;
    if ((prev_gate == nullptr) != (W_res == nullptr)) return MOEPP_EINVAL;
    if (c->desc.n_const > 0 && !W_c) return MOEPP_EINVAL;
    if (misaligned(x) || misaligned(W_g) || misaligned(out_gate) || misaligned(prev_gate) ||
        misaligned(W_res) || misaligned(W_c))
        return MOEPP_EINVAL;
    return MOEPP_OK;
}

// Argument checks of moepp_layer_forward for T > 0 (nothing is launched).
moepp_status check_forward(const moepp_ctx *ctx, int32_t T, const void *x, const float *prev_gate,
                           const float *W_g, const float *W_res, const void *experts,
                           const void *const_vecs, const float *W_c, int32_t k, const void *out,
                           const float *out_gate) {
    moepp_status st = check_route_args(ctx, x, prev_gate, W_g, W_res, W_c, out_gate);
    if (st != MOEPP_OK) return st;
    if (!out || misaligned(out)) return MOEPP_EINVAL;
    if (ctx->desc.n_ffn > 0 && (!experts || misaligned(experts))) return MOEPP_EINVAL;
    if (ctx->desc.n_const > 0 && (!const_vecs || misaligned(const_vecs))) return MOEPP_EINVAL;
    // a required kernel family that does not cover the shape must fail before anything is launched
    const Dims d = dims_of(ctx, T, k);
    moepp_status s2 = MOEPP_OK;
    (void)use_mfma_router(ctx, d, &s2);
    (void)use_mfma_ffn(ctx, d, &s2);
    return s2;
}

// The four steps, arguments already checked.
moepp_status run_forward(moepp_ctx *ctx, void *stream, int32_t T, const void *x,
                         const float *prev_gate, const float *W_g, const float *W_res,
                         const void *experts, const void *const_vecs, const float *W_c, int32_t k,
                         void *out, float *out_gate) {
    reset_ran(ctx);
    hipStream_t s = (hipStream_t)stream;
    moepp_status st = do_route(ctx, s, T, x, prev_gate, W_g, W_res, W_c, k, out_gate);
    if (st != MOEPP_OK) return st;
    st = do_permute(ctx, s, T, k);
    if (st != MOEPP_OK) return st;
    st = do_ffn(ctx, s, T, x, experts, k);
    if (st != MOEPP_OK) return st;
    return do_combine(ctx, s, T, x, const_vecs, k, out);
}

// Fresh host-side state of a context over `workspace` (already validated).
void init_ctx(moepp_ctx *c, const moepp_desc *desc, void *workspace) {
    c->desc = *desc;
    c->ws_bytes = layout(desc, (char *)workspace, &c->ws);
    c->bias = nullptr;
    c->variant = 0;
    c->cap.on = false;
    for (int i = 0; i < kMaxExperts; ++i) c->cap.cap[i] = 0;
    c->bal_tau = 0.0;
    c->last_out_gate = nullptr;
    c->last_T = 0;
    c->last_k = desc->k;
    c->hist_valid = false;
    c->perm_valid = false;
    c->bal_rows = c->bal_T = 0;
    c->hist_T = c->hist_k = c->hist_chunk_slots = 0;
    c->timing = false;
    c->have_events = false;
    clear_timing(c);
}

// ---- scratch of moepp_layer_forward_static ----------------------------------
// One array per GPU, in that GPU's memory from the moment the library's code
// object is loaded there until the process ends.  In host code the name
// `scratch` is only a handle of the symbol, not a device address: the address
// on the current device is asked for once per device and kept.
constexpr size_t kStaticScratchBytes = MOEPP_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];       // per device; null until first asked for

// Device address of `scratch` on the current device (null + status on failure).
moepp_status static_scratch(void **ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return MOEPP_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return MOEPP_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MOEPP_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return MOEPP_OK;
}

}  // namespace

// ---------------------------------------------------------------------------
extern "C" {

size_t moepp_workspace_bytes(const moepp_desc *desc) {
    if (check_desc(desc) != MOEPP_OK) return 0;
    return layout(desc, nullptr, nullptr);
}

size_t moepp_packed_bytes(const moepp_desc *desc) {
    if (check_desc(desc) != MOEPP_OK) return 0;
    const size_t b = (size_t)desc->n_ffn * 3 * desc->F * desc->D * elt(desc);
    return b ? b : 16;
}

moepp_status moepp_create(const moepp_desc *desc, void *workspace, size_t bytes, moepp_ctx **ctx) {
    if (!desc || !workspace || !ctx) return MOEPP_EINVAL;
    moepp_status st = check_desc(desc);
    if (st != MOEPP_OK) return st;
    if (((uintptr_t)workspace & (kAlign - 1)) != 0) return MOEPP_EINVAL;
    if (bytes < layout(desc, nullptr, nullptr)) return MOEPP_ENOMEM;
    moepp_ctx *c = new (std::nothrow) moepp_ctx();
    if (!c) return MOEPP_ENOMEM;
    init_ctx(c, desc, workspace);
    *ctx = c;
    return MOEPP_OK;
}

moepp_status moepp_destroy(moepp_ctx *ctx) {
    if (!ctx) return MOEPP_EINVAL;
    if (ctx->have_events)
        for (int q = 0; q < kTimingSlots; ++q)
            for (int i = 0; i < MOEPP_NUM_KERNELS; ++i) {
                (void)hipEventDestroy(ctx->ev[q][i][0]);
                (void)hipEventDestroy(ctx->ev[q][i][1]);
            }
    delete ctx;
    return MOEPP_OK;
}

moepp_status moepp_pack_experts(moepp_ctx *ctx, void *stream, const moepp_experts *experts,
                                void *packed, size_t bytes) {
    if (!ctx || !packed) return MOEPP_EINVAL;
    if (bytes < moepp_packed_bytes(&ctx->desc)) return MOEPP_ENOMEM;
    if (ctx->desc.n_ffn == 0) return MOEPP_OK;
    if (!experts || !experts->w1 || !experts->w3 || !experts->w2) return MOEPP_EINVAL;
    if (misaligned(experts->w1) || misaligned(experts->w3) || misaligned(experts->w2) ||
        misaligned(packed))
        return MOEPP_EINVAL;
    const Dims d = dims_of(ctx, 0, ctx->desc.k);
    hipError_t e = launch_pack(d, ctx->desc.act == MOEPP_BF16, experts->w1, experts->w3,
                               experts->w2, packed, const_cast<void *>(packed_w2(ctx, packed)),
                               (hipStream_t)stream);
    return e == hipSuccess ? MOEPP_OK : MOEPP_EHIP;
}

moepp_status moepp_set_router_bias(moepp_ctx *ctx, const float *bias) {
    if (!ctx || misaligned(bias)) return MOEPP_EINVAL;
    ctx->bias = bias;
    return MOEPP_OK;
}

moepp_status moepp_capacity(const moepp_desc *desc, int32_t T, int32_t k, double gamma, double tau,
                            int32_t per_assignment, int32_t *cap_host) {
    moepp_status st = check_desc(desc);
    if (st != MOEPP_OK) return st;
    if (!cap_host || T < 0 || T > desc->T_max || k < 1 || k > desc->k) return MOEPP_EINVAL;
    if (!(gamma > 0.0) || !(tau > 0.0) || !isfinite(gamma) || !isfinite(tau)) return MOEPP_EINVAL;
    const int N = n_experts(desc);
    const double units = per_assignment ? (double)T * (double)k : (double)T;
    // places per unit of eta: gamma * S / (tau N_FFN + N_ZC); an FFN expert gets tau of them
    const double per_eta = gamma * units / (tau * (double)desc->n_ffn + (double)(N - desc->n_ffn));
    for (int i = 0; i < N; ++i) {
        const double c = i < desc->n_ffn ? tau * per_eta : per_eta;
        // the next integer at or above c; a c that sits above an integer only by the
        // representation error of gamma and tau (relative 1e-9) is that integer
        const double near = nearbyint(c);
        const double tol = 1e-9 * (c > 1.0 ? c : 1.0);
        const double r = (c > near && c - near <= tol) ? near : ceil(c);
        cap_host[i] = r > 2147483647.0 ? 2147483647 : (int32_t)r;
    }
    return MOEPP_OK;
}

moepp_status moepp_set_capacity(moepp_ctx *ctx, const int32_t *cap_host) {
    if (!ctx) return MOEPP_EINVAL;
    ctx->perm_valid = false;      // a permutation done under the old capacities does not stand in for a new one
    if (!cap_host) {
        ctx->cap.on = false;
        return MOEPP_OK;
    }
    const int N = n_experts(&ctx->desc);
    for (int i = 0; i < N; ++i)
        if (cap_host[i] < 0) return MOEPP_EINVAL;
    for (int i = 0; i < kMaxExperts; ++i) ctx->cap.cap[i] = i < N ? cap_host[i] : 0;
    ctx->cap.on = true;
    return MOEPP_OK;
}

moepp_status moepp_set_balance(moepp_ctx *ctx, double tau) {
    if (!ctx || !(tau == tau) || !isfinite(tau)) return MOEPP_EINVAL;
    ctx->bal_tau = tau > 0.0 ? tau : 0.0;
    return MOEPP_OK;
}

moepp_status moepp_get_balance(moepp_ctx *ctx, const float **f, const float **P,
                               const float **loss) {
    if (!ctx) return MOEPP_EINVAL;
    const int N = n_experts(&ctx->desc);
    if (f) *f = ctx->ws.bal;
    if (P) *P = ctx->ws.bal + N;
    if (loss) *loss = ctx->ws.bal + 2 * N;
    return MOEPP_OK;
}

moepp_status moepp_get_kept(moepp_ctx *ctx, const int32_t **kept) {
    if (!ctx || !kept) return MOEPP_EINVAL;
    *kept = ctx->ws.kept;
    return MOEPP_OK;
}

moepp_status moepp_set_variant(moepp_ctx *ctx, int32_t variant) {
    if (!ctx || variant < 0 || variant > 3) return MOEPP_EINVAL;
    ctx->variant = variant;
    return MOEPP_OK;
}

moepp_status moepp_route(moepp_ctx *ctx, void *stream, int32_t T, const void *x,
                         const float *prev_gate, const float *W_g, const float *W_res,
                         const float *W_c, int32_t k, float *out_gate) {
    moepp_status st = check_call(ctx, T, k);
    if (st != MOEPP_OK) return st;
    if (T == 0) return note_empty_call(ctx, k);
    st = check_route_args(ctx, x, prev_gate, W_g, W_res, W_c, out_gate);
    if (st != MOEPP_OK) return st;
    reset_ran(ctx);
    return do_route(ctx, (hipStream_t)stream, T, x, prev_gate, W_g, W_res, W_c, k, out_gate);
}

moepp_status moepp_permute(moepp_ctx *ctx, void *stream, int32_t T, int32_t k) {
    moepp_status st = check_call(ctx, T, k);
    if (st != MOEPP_OK) return st;
    // the statistics read the logits of the routed call this permutation belongs to
    if (ctx->bal_tau > 0.0 && T > 0 && (!ctx->last_out_gate || ctx->last_T != T)) return MOEPP_EINVAL;
    reset_ran(ctx);
    return do_permute(ctx, (hipStream_t)stream, T, k);
}

moepp_status moepp_expert_ffn(moepp_ctx *ctx, void *stream, int32_t T, const void *x,
                              const void *experts, int32_t k) {
    moepp_status st = check_call(ctx, T, k);
    if (st != MOEPP_OK) return st;
    if (T == 0) return note_empty_call(ctx, k);
    if (!x || misaligned(x)) return MOEPP_EINVAL;
    if (ctx->desc.n_ffn > 0 && (!experts || misaligned(experts))) return MOEPP_EINVAL;
    reset_ran(ctx);
    return do_ffn(ctx, (hipStream_t)stream, T, x, experts, k);
}

moepp_status moepp_combine(moepp_ctx *ctx, void *stream, int32_t T, const void *x,
                           const void *const_vecs, int32_t k, void *out) {
    moepp_status st = check_call(ctx, T, k);
    if (st != MOEPP_OK) return st;
    if (T == 0) return note_empty_call(ctx, k);
    if (!x || !out || misaligned(x) || misaligned(out)) return MOEPP_EINVAL;
    if (ctx->desc.n_const > 0 && (!const_vecs || misaligned(const_vecs))) return MOEPP_EINVAL;
    reset_ran(ctx);
    return do_combine(ctx, (hipStream_t)stream, T, x, const_vecs, k, out);
}

moepp_status moepp_layer_forward(moepp_ctx *ctx, void *stream, int32_t T, const void *x,
                                 const float *prev_gate, const float *W_g, const float *W_res,
                                 const void *experts, const void *const_vecs, const float *W_c,
                                 int32_t k, void *out, float *out_gate) {
    moepp_status st = check_call(ctx, T, k);
    if (st != MOEPP_OK) return st;
    if (T == 0) return note_empty_call(ctx, k);
    st = check_forward(ctx, T, x, prev_gate, W_g, W_res, experts, const_vecs, W_c, k, out, out_gate);
    if (st != MOEPP_OK) return st;
    return run_forward(ctx, stream, T, x, prev_gate, W_g, W_res, experts, const_vecs, W_c, k, out,
                       out_gate);
}

moepp_status moepp_layer_forward_static(const moepp_desc *desc, void *stream, int32_t T,
                                        const void *x, const float *prev_gate, const float *W_g,
                                        const float *W_res, const void *experts,
                                        const void *const_vecs, const float *W_c, int32_t k,
                                        void *out, float *out_gate) {
    moepp_status st = check_desc(desc);
    if (st != MOEPP_OK) return st;
    if (layout(desc, nullptr, nullptr) > kStaticScratchBytes) return MOEPP_ENOMEM;
    // Host-side bookkeeping of this call only: no device memory, nothing allocated.
    static thread_local moepp_ctx c;
    init_ctx(&c, desc, nullptr);
    st = check_call(&c, T, k);
    if (st != MOEPP_OK) return st;
    if (T == 0) return MOEPP_OK;
    st = check_forward(&c, T, x, prev_gate, W_g, W_res, experts, const_vecs, W_c, k, out, out_gate);
    if (st != MOEPP_OK) return st;
    void *ws = nullptr;
    st = static_scratch(&ws);
    if (st != MOEPP_OK) return st;
    init_ctx(&c, desc, ws);
    return run_forward(&c, stream, T, x, prev_gate, W_g, W_res, experts, const_vecs, W_c, k, out,
                       out_gate);
}

moepp_status moepp_get_routing(moepp_ctx *ctx, const int32_t **topk_idx, const float **topk_w,
                               const int32_t **counts, const int32_t **offsets,
                               const int32_t **row_of, const int32_t **src_of) {
    if (!ctx) return MOEPP_EINVAL;
    if (topk_idx) *topk_idx = ctx->ws.topk_idx;
    if (topk_w) *topk_w = ctx->ws.topk_w;
    if (counts) *counts = ctx->ws.counts;
    if (offsets) *offsets = ctx->ws.offsets;
    if (row_of) *row_of = ctx->ws.row_of;
    if (src_of) *src_of = ctx->ws.src_of;
    return MOEPP_OK;
}

moepp_status moepp_get_intermediates(moepp_ctx *ctx, const float **alpha1, const void **h,
                                     const void **yffn) {
    if (!ctx) return MOEPP_EINVAL;
    if (alpha1) *alpha1 = ctx->ws.alpha1;
    if (h) *h = ctx->ws.h;
    if (yffn) *yffn = ctx->ws.yffn;
    return MOEPP_OK;
}

moepp_status moepp_set_timing(moepp_ctx *ctx, int32_t enable) {
    if (!ctx) return MOEPP_EINVAL;
    if (enable && !ctx->have_events) {
        for (int q = 0; q < kTimingSlots; ++q)
            for (int i = 0; i < MOEPP_NUM_KERNELS; ++i)
                for (int j = 0; j < 2; ++j)
                    // timing only: without the system-scope fence (and cache flush) an ordinary
                    // event puts behind the kernel it follows, which costs ~10 us per event
                    if (hipEventCreateWithFlags(&ctx->ev[q][i][j], hipEventDisableSystemFence) != hipSuccess)
                        return MOEPP_EHIP;
        ctx->have_events = true;
    }
    ctx->timing = enable != 0;
    clear_timing(ctx);
    return MOEPP_OK;
}

moepp_status moepp_get_timing(moepp_ctx *ctx, float *ms) {
    if (!ctx || !ms) return MOEPP_EINVAL;
    for (int i = 0; i < MOEPP_NUM_KERNELS; ++i) {
        ms[i] = 0.f;
        if (!ctx->have_events) continue;
        double sum = 0.0;
        int n = 0;
        for (int q = 0; q < kTimingSlots; ++q) {
            if (!ctx->ran[q][i]) continue;
            float t = 0.f;
            if (hipEventSynchronize(ctx->ev[q][i][1]) != hipSuccess) return MOEPP_EHIP;
            if (hipEventElapsedTime(&t, ctx->ev[q][i][0], ctx->ev[q][i][1]) != hipSuccess)
                return MOEPP_EHIP;
            sum += t;
            n += 1;
        }
        if (n) ms[i] = (float)(sum / n);
    }
    clear_timing(ctx);
    return MOEPP_OK;
}

moepp_status moepp_mfma_ceiling(void *stream, void *scratch, size_t scratch_bytes, int32_t iters,
                                double *flops) {
    if (!scratch || !flops || iters < 1 || misaligned(scratch)) return MOEPP_EINVAL;
    if (scratch_bytes < mfma_ceiling_scratch_bytes()) return MOEPP_ENOMEM;
    *flops = mfma_ceiling_flops(iters);
    return launch_mfma_ceiling((float *)scratch, iters, (hipStream_t)stream) == hipSuccess
               ? MOEPP_OK
               : MOEPP_EHIP;
}

moepp_status moepp_stream_ceiling(void *stream, void *buf, size_t bytes, int32_t mode,
                                  double *moved_bytes) {
    if (!buf || !moved_bytes || misaligned(buf) || (mode != 0 && mode != 1)) return MOEPP_EINVAL;
    if (bytes < ((size_t)64 << 20) || bytes % 32768 != 0) return MOEPP_EINVAL;
    *moved_bytes = (double)bytes;       // mode 1: half of the buffer read and half of it written
    return launch_stream(buf, bytes, mode, (hipStream_t)stream) == hipSuccess ? MOEPP_OK : MOEPP_EHIP;
}

const char *moepp_status_str(int32_t status) {
    switch (status) {
        case MOEPP_OK: return "ok";
        case MOEPP_EINVAL: return "invalid argument";
        case MOEPP_EUNSUPPORTED: return "unsupported configuration";
        case MOEPP_ENOMEM: return "buffer too small";
        case MOEPP_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
