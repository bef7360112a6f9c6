// Router for bf16 activations on the matrix cores.
//
//   G(x) = W x (+ W_g G(x_prev)) (+ bias)           (paper Eq.2 / Eq.6)
//   Softmax over all N experts, Top-K of G(x)       (Eq.1)
//   a1 = Softmax(W_c x)_1 of every constant expert  (Eq.5)
//
// The pass over x is HBM-bound only if the N + 2 n_const dot products per
// token do not run on the vector ALUs (about 24 flop per byte of x).  x is
// exactly bf16, so each float32 router weight is split into three bf16 pieces
// w = hi + mid + lo (24 significand bits, the split is exact) and the
// contraction runs as three bf16 MFMAs with float32 accumulation: products
// are exact, logits keep float32-class accuracy.
//
// The kernel is a skinny GEMM [128 tokens x K] x [K x (N + 2 n_const)] per
// workgroup of 8 waves.  x tiles of 64 K-elements are written into a ring of
// LDS stages by the loads themselves (row-contiguous 16-byte chunks, so every
// wave-wide load covers whole 128-byte lines).  The weight rows (router rows,
// then the W_c rows) are split once per call by a small kernel into a scratch
// buffer that already has the byte order of an LDS weight tile, so the weight
// tile of a stage is filled by the same kind of load.  (A float32 load mixed
// into the loop would have to be waited for with vmcnt, and loads complete in
// order: it would drag every younger x load with it.)  Wave w owns tokens
// 32 (w % 4) .. +31 and the K steps of parity w / 4 of every tile; the two
// halves are added at the end.
// Epilogue: gating residual and bias with all threads, then one thread per
// token does softmax and Top-K on the float32 logits (ties to the lower
// index, slots in descending order).
#include "common.h"

#include <type_traits>

namespace moepp {

constexpr int kRtThreads = 512;
constexpr int kRtTok = 128;                // tokens per workgroup
constexpr int kRtBK = 64;                  // K elements per stage
constexpr int kRtRow = kRtBK * 2;          // bytes per tile row
constexpr int kRtXBytes = kRtTok * kRtRow; // x part of a stage

typedef const __attribute__((address_space(1))) void *rt_gptr_t;
typedef __attribute__((address_space(3))) void *rt_lptr_t;

// XOR swizzle of the 16-byte slots of a 128-byte tile row: 16 consecutive rows
// read at one logical slot cover the 64 LDS banks exactly once.
__device__ inline int rt_swz(int row) { return (row >> 1) & 7; }

template <int VM>
__device__ inline void rt_wait_and_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((VM & 15) | 0x70 | ((VM >> 4) << 14));   // vmcnt(VM) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Bytes of the split-weight scratch for a layer (0 if the MFMA router does not apply).
size_t router_split_bytes(int D, int rows) {
    const int nblk = (rows + 31) / 32;
    return (size_t)3 * nblk * 32 * D * 2;
}

// Split kernel: float32 weight rows (router rows, then the W_c rows) -> three
// bf16 pieces, written tile by tile in exactly the byte order of an LDS weight
// tile (piece, row, swizzled 16-byte slot), so that the router kernel can copy
// a tile into LDS with plain contiguous loads.  Rows past the last are zero.
__global__ __launch_bounds__(256) void k_router_split(RouterArgs a, int nblk) {
    typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
    const int D = a.d.D, N = a.d.N, rows = N + 2 * a.d.n_const;
    const int ROWS = nblk * 32, PIECE = ROWS * kRtRow;
    const int per_row = D / 4;                               // float4 per row
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= ROWS * per_row) return;
    const int r = idx / per_row, k4 = idx % per_row;         // row, float4 number
    f32x4 w = {0.f, 0.f, 0.f, 0.f};
    if (r < rows) {
        const float *src = r < N ? a.W_g + (size_t)r * D : a.W_c + (size_t)(r - N) * D;
        w = *reinterpret_cast<const f32x4 *>(src + k4 * 4);
    }
    bf16x4 hi, mid, lo;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const bf16_t h = (bf16_t)w[q];
        const float r1 = w[q] - (float)h;
        const bf16_t m = (bf16_t)r1;
        hi[q] = h;
        mid[q] = m;
        lo[q] = (bf16_t)(r1 - (float)m);
    }
    const int kt = k4 / 16, wq = k4 % 16;                    // K tile, float4 within the tile
    char *p = static_cast<char *>(a.wsplit) + (size_t)kt * 3 * PIECE + r * kRtRow +
              ((((wq >> 1) ^ rt_swz(r)) << 4) | ((wq & 1) << 3));
    *reinterpret_cast<bf16x4 *>(p) = hi;
    *reinterpret_cast<bf16x4 *>(p + PIECE) = mid;
    *reinterpret_cast<bf16x4 *>(p + 2 * PIECE) = lo;
}

template <int NBLK>   // 32-row blocks of weight rows
__global__ __launch_bounds__(kRtThreads, 1) void k_router_mfma(RouterArgs a) {
    constexpr int ROWS = NBLK * 32;
    constexpr int PIECE = ROWS * kRtRow;                  // one bf16 piece of the weight tile
    constexpr int WBYTES = 3 * PIECE;                     // 12 KB per row block
    constexpr int LPT = (kRtXBytes + WBYTES + kRtThreads * 16 - 1) / (kRtThreads * 16);   // loads per thread, tile
    constexpr int STAGE = LPT * kRtThreads * 16;          // x tile, weight tile, padding
    constexpr int NS = (160 * 1024) / STAGE < 4 ? (160 * 1024) / STAGE : 4;
    constexpr int DSTR = ROWS + 1;                        // floats per token in `dots`
    constexpr int E_BYTES = (2 * kRtTok * DSTR + kRtTok * (kMaxExperts + 1) +
                             kMaxExperts * kMaxExperts + kMaxExperts) * 4;
    constexpr int LDS_BYTES = NS * STAGE > E_BYTES ? NS * STAGE : E_BYTES;
    static_assert(NS >= 3 && LDS_BYTES <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];

    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int l32 = lane % 32, lh = lane / 32;
    const int tb = wave % 4, kh = wave / 4;               // token block, K-step parity
    const int D = a.d.D, N = a.d.N, K = a.d.k, nc = a.d.n_const, T = a.d.T;
    const int rows = N + 2 * nc;
    const int t0 = blockIdx.x * kRtTok;
    const int KT = D / kRtBK;

    // ---- loads that write LDS themselves: every thread issues LPT per tile ----
    // chunk c = tid + 512 i.  c < 1024: x tile, row c / 8, slot c % 8 holds
    // global chunk slot ^ swz(row).  Then the weight tile, a plain copy of the
    // pre-split buffer; chunks past its end re-read its start (padding, unused).
    const char *src[LPT];
    int step[LPT];                                        // bytes from one K tile to the next
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int c = tid + kRtThreads * i;
        if (c < kRtXBytes / 16) {
            const int row = c / 8;
            int tok = t0 + row;
            tok = tok < T ? tok : T - 1;
            src[i] = static_cast<const char *>(a.x) + ((size_t)tok * D + (((c % 8) ^ rt_swz(row)) << 3)) * 2;
            step[i] = kRtBK * 2;
        } else {
            int wc = c - kRtXBytes / 16;
            wc = wc < WBYTES / 16 ? wc : wc - WBYTES / 16;
            src[i] = static_cast<const char *>(a.wsplit) + wc * 16;
            step[i] = WBYTES;
        }
    }
    const int wave_off = __builtin_amdgcn_readfirstlane(wave) * 1024;
    auto issue = [&](int kt, char *__restrict__ stage) {
#pragma unroll
        for (int i = 0; i < LPT; ++i)
            __builtin_amdgcn_global_load_lds((rt_gptr_t)(src[i] + (size_t)kt * step[i]),
                                             (rt_lptr_t)(stage + wave_off + i * kRtThreads * 16), 16, 0, 0);
    };

    f32x16 acc_hi[NBLK], acc_lo[NBLK];
#pragma unroll
    for (int b = 0; b < NBLK; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_hi[b][v] = acc_lo[b][v] = 0.f;

    // MFMA operand offsets of this wave's two K steps (2 kh, 2 kh + 1) of a tile
    int rd_off[2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
        rd_off[s] = l32 * kRtRow + (((2 * (2 * kh + s) + lh) ^ rt_swz(l32)) << 4);

    // One tile: refill the stage that was read last, run the MFMAs of this one.
    auto tile = [&](const char *__restrict__ cur, char *__restrict__ dst, int kt_issue, auto issue_c) {
        if constexpr (decltype(issue_c)::value) issue(kt_issue, dst);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const bf16x8 xf = *reinterpret_cast<const bf16x8 *>(cur + tb * 32 * kRtRow + rd_off[s]);
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const char *p = cur + kRtXBytes + b * 32 * kRtRow + rd_off[s];
                const bf16x8 whi = *reinterpret_cast<const bf16x8 *>(p);
                const bf16x8 wmid = *reinterpret_cast<const bf16x8 *>(p + PIECE);
                const bf16x8 wlo = *reinterpret_cast<const bf16x8 *>(p + 2 * PIECE);
                acc_hi[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(whi, xf, acc_hi[b], 0, 0, 0);
                acc_lo[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wmid, xf, acc_lo[b], 0, 0, 0);
                acc_lo[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wlo, xf, acc_lo[b], 0, 0, 0);
            }
        }
    };

    // Ring of NS stages, tile kt in stage kt % NS, NS - 1 tiles in flight.
    // Needs KT >= NS - 1 (the launcher checks).
#pragma unroll
    for (int p = 0; p < NS - 1; ++p) issue(p, lds + p * STAGE);
    rt_wait_and_barrier<(NS - 2) * LPT>();                   // tile 0 landed
    int s_cur = 0, s_dst = NS - 1;
    auto rotate = [&]() {
        s_dst = s_cur;
        s_cur = s_cur + 1 == NS ? 0 : s_cur + 1;
    };
    typedef std::true_type yes_t;
    typedef std::false_type no_t;
    for (int kt = 0; kt < KT - (NS - 1); ++kt) {
        tile(lds + s_cur * STAGE, lds + s_dst * STAGE, kt + NS - 1, yes_t{});
        rt_wait_and_barrier<(NS - 2) * LPT>();               // tile kt+1 landed, tile kt read by all
        rotate();
    }
#pragma unroll
    for (int t = 0; t < NS - 1; ++t) {                       // the last NS-1 tiles: nothing to issue
        tile(lds + s_cur * STAGE, lds + s_dst * STAGE, 0, no_t{});
        rt_wait_and_barrier<0>();
        rotate();
    }

    // ---- epilogue -------------------------------------------------------------
    // (the loop ended with a barrier: the stages are dead)
    float *dots = reinterpret_cast<float *>(lds);               // [kRtTok][DSTR]  K-step parity 0
    float *dots1 = dots + kRtTok * DSTR;                        // [kRtTok][DSTR]  K-step parity 1
    float *prevs = dots1 + kRtTok * DSTR;                       // [kRtTok][N + 1]
    float *wres = prevs + kRtTok * (kMaxExperts + 1);           // [N][N]
    float *sbias = wres + kMaxExperts * kMaxExperts;            // [N]
    // acc[b][v]: weight row b*32 + 8*(v/4) + 4*lh + v%4, token tb*32 + l32
    {
        float *dst = kh == 0 ? dots : dots1;
#pragma unroll
        for (int b = 0; b < NBLK; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                dst[(tb * 32 + l32) * DSTR + b * 32 + 8 * (v / 4) + 4 * lh + (v % 4)] =
                    acc_hi[b][v] + acc_lo[b][v];
    }
    const int n_tok = min(kRtTok, T - t0);
    if (a.prev_gate) {
        for (int c = tid; c < n_tok * N; c += kRtThreads)
            prevs[(c / N) * (N + 1) + c % N] = a.prev_gate[(size_t)t0 * N + c];
        for (int c = tid; c < N * N; c += kRtThreads) wres[c] = a.W_res[c];
    }
    for (int c = tid; c < N; c += kRtThreads) sbias[c] = a.bias ? a.bias[c] : 0.f;
    __syncthreads();

    // logits, all threads: element c -> (token c / rows, row c % rows)
    for (int c = tid; c < n_tok * rows; c += kRtThreads) {
        const int tt = c / rows, i = c % rows;
        float L = dots[tt * DSTR + i] + dots1[tt * DSTR + i];
        if (i < N) {
            if (a.prev_gate) {
                const float *pr = prevs + tt * (N + 1);
                const float *wr = wres + i * N;
                float r0 = 0.f, r1 = 0.f;
                int m = 0;
                for (; m + 1 < N; m += 2) {
                    r0 = fmaf(wr[m], pr[m], r0);
                    r1 = fmaf(wr[m + 1], pr[m + 1], r1);
                }
                if (m < N) r0 = fmaf(wr[m], pr[m], r0);
                L += r0 + r1;
            }
            L += sbias[i];
        }
        dots[tt * DSTR + i] = L;
    }
    __syncthreads();

    if (tid < n_tok) {
        const float *Lr = dots + tid * DSTR;
        float mx = -INFINITY;
        for (int i = 0; i < N; ++i) mx = fmaxf(mx, Lr[i]);
        float sum = 0.f;
        for (int i = 0; i < N; ++i) sum += __expf(Lr[i] - mx);
        const float inv = 1.f / sum;
        unsigned long long taken = 0ull;
        const size_t t = (size_t)(t0 + tid);
        for (int s = 0; s < K; ++s) {
            float bv = -INFINITY;
            int bi = 0;
            bool have = false;
            for (int i = 0; i < N; ++i) {
                const float v = Lr[i];
                if (!((taken >> i) & 1ull) && (!have || v > bv)) {
                    bv = v;
                    bi = i;
                    have = true;
                }
            }
            taken |= 1ull << bi;
            a.topk_idx[t * K + s] = bi;
            a.topk_w[t * K + s] = __expf(bv - mx) * inv;
        }
        for (int j = 0; j < nc; ++j)
            a.alpha1[t * nc + j] = 1.f / (1.f + expf(Lr[N + 2 * j + 1] - Lr[N + 2 * j]));
    }
    // out_gate block [n_tok, N] is contiguous in memory: coalesced copy from LDS
    for (int c = tid; c < n_tok * N; c += kRtThreads)
        a.out_gate[(size_t)t0 * N + c] = dots[(c / N) * DSTR + c % N];
}

bool router_mfma_supported(const Dims &d) {
    // two 32-row blocks of weight rows at most; at least 3 K tiles to fill the ring
    return d.D % kRtBK == 0 && d.D >= 3 * kRtBK && d.N + 2 * d.n_const <= 64;
}

hipError_t launch_router_mfma(const RouterArgs &a, hipStream_t s) {
    if (a.d.T == 0) return hipSuccess;
    const int rows = a.d.N + 2 * a.d.n_const;
    const int nblk = (rows + 31) / 32;
    const int n4 = nblk * 32 * (a.d.D / 4);
    hipLaunchKernelGGL(k_router_split, dim3((n4 + 255) / 256), dim3(256), 0, s, a, nblk);
    dim3 grid((a.d.T + kRtTok - 1) / kRtTok), block(kRtThreads);
    if (nblk == 1)
        hipLaunchKernelGGL(k_router_mfma<1>, grid, block, 0, s, a);
    else
        hipLaunchKernelGGL(k_router_mfma<2>, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace moepp
