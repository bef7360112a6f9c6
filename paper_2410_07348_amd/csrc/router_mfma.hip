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
// The kernel is a skinny GEMM [TOK tokens x K] x [K x (N + 2 n_const)] per
// workgroup of TOK / 16 waves (TOK = 128, or 64 when there are few tokens).
// x and weight tiles of 64 K-elements are loaded with row-contiguous 16-byte
// chunks (every wave-wide load covers whole 128-byte lines) into REGISTERS, PF
// tiles ahead, and stored from there into a double-buffered LDS tile (the
// compiler tracks these ordinary loads exactly, so nothing is waited for
// early).  The weights are read as float32 straight from W and W_c (only the
// real rows: N + 2 n_const of the 32 or 64 the matrix core multiplies) and split
// into their three pieces on the way into LDS: a few VALU operations per
// thread and tile, no prepared copy and no extra pass over them; every
// workgroup reads all of them once, from L2.  That second stream is not free
// (a microbenchmark of the two streams alone: 42 us for x at this workload,
// 42 / 49 / 56 us with 0.5 / 1 / 1.5 bytes of weights per byte of x), which is
// why the weights travel as 4-byte floats (0.375 bytes per byte of x at
// N + 2 n_const = 24, 128 tokens) and not as three bf16 pieces (0.75).  x is
// loaded with the non-temporal hint: it is read once.  Workgroup b starts at
// K tile b % KT and wraps around, so that the workgroups, which walk K in
// lockstep over rows a power of two apart, do not all ask the same memory
// channels at the same time.  Wave w owns tokens 32 (w % (TOK/32)) .. +31 and
// the K steps of parity w / (TOK/32) of every tile; the two halves are added
// at the end.
// Epilogue: gating residual and bias with all threads, then four threads per
// token (each owns the experts i = q mod 4, shuffles combine them) do softmax
// and Top-K on the float32 logits (ties to the lower index, slots in
// descending order).  The workgroup also counts its tokens' selections per
// expert: its TOK * k slots are one chunk of the permutation that follows, which
// then needs no histogram pass of its own.
#include "common.h"
#include "router_device.h"

namespace moepp {

constexpr int kRtBK = 64;                  // K elements per stage
constexpr int kRtRow = kRtBK * 2;          // bytes per tile row

// XOR swizzle of the 16-byte slots of a 128-byte tile row: 16 consecutive rows
// read at one logical slot cover the 64 LDS banks exactly once.
__device__ inline int rt_swz(int row) { return (row >> 1) & 7; }

// NBLK: 32-row blocks of weight rows; PF: tiles prefetched in registers;
// TOK: tokens per workgroup (4 threads per token); WPE: waves per SIMD the
// register budget is sized for (several small workgroups share a CU, so that
// one can compute while another waits at its barrier).
template <int NBLK, int PF, int TOK, int WPE>
__global__ __launch_bounds__(4 * TOK, WPE) void k_router_mfma(RouterArgs a) {
    constexpr int kRtTok = TOK, kRtThreads = 4 * TOK, TB = TOK / 32;
    constexpr int kRtXBytes = kRtTok * kRtRow;            // x part of a stage
    constexpr int ROWS = NBLK * 32;
    constexpr int PIECE = ROWS * kRtRow;                  // one bf16 piece of the weight tile
    constexpr int WBYTES = 3 * PIECE;                     // 12 KB per row block
    constexpr int WCH = ROWS * (kRtBK / 4);               // 16-byte chunks (4 floats) of a float32 weight tile
    constexpr int WL = (WCH + kRtThreads - 1) / kRtThreads;   // weight chunks per thread and tile
    constexpr int STAGE = kRtXBytes + WBYTES;
    constexpr int DSTR = ROWS + 1;                        // floats per token in `dots`
    constexpr int E_BYTES = (2 * kRtTok * DSTR + kRtTok * (kMaxExperts + 1) +
                             kMaxExperts * kMaxExperts + 2 * kMaxExperts) * 4;
    constexpr int LDS_BYTES = 2 * STAGE > E_BYTES ? 2 * STAGE : E_BYTES;
    static_assert(LDS_BYTES <= 160 * 1024 && PF % 2 == 0, "LDS / PF");
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];

    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int l32 = lane % 32, lh = lane / 32;
    const int tb = wave % TB, kh = wave / TB;             // token block, K-step parity
    const int D = a.d.D, N = a.d.N, nc = a.d.n_const, T = a.d.T;
    const int rows = N + 2 * nc;
    const int t0 = blockIdx.x * kRtTok;
    const int KT = D / kRtBK;                             // a multiple of PF (the launcher checks)

    // ---- tile loads ------------------------------------------------------------
    // x chunk c = tid + threads i (i = 0, 1): tile row c / 8, LDS slot c % 8 holds
    // global chunk slot ^ swz(row), so the LDS position of chunk c is simply 16 c.
    const char *px[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid + kRtThreads * i, row = c / 8;
        int tok = t0 + row;
        tok = tok < T ? tok : T - 1;
        px[i] = static_cast<const char *>(a.x) + ((size_t)tok * D + (((c % 8) ^ rt_swz(row)) << 3)) * 2;
    }
    // Weight chunk c = tid + threads i: row c / 16, floats 4 (c % 16) .. + 3 of the
    // tile's 64 columns, read as float32 from W (router rows) or W_c (the rows after
    // them) and split into three bf16 pieces on the way into LDS; rows past the
    // last are never loaded (their LDS rows are zeroed once, below).
    const float *pw[WL];
    int w_lds[WL];                                         // LDS offset of the chunk's hi piece; -1: no chunk
#pragma unroll
    for (int i = 0; i < WL; ++i) {
        const int c = tid + kRtThreads * i, r = c / 16, kq = c % 16;
        const bool act = r < rows;
        pw[i] = (!act ? a.W_g : r < N ? a.W_g + (size_t)r * D : a.W_c + (size_t)(r - N) * D) + kq * 4;
        w_lds[i] = act ? r * kRtRow + ((((kq >> 1) ^ rt_swz(r)) << 4) | ((kq & 1) << 3)) : -1;
    }
    bf16x8 xr[PF][2];
    f32x4 wr[PF][WL];
    // Workgroups walk K in lockstep, and rows of x are a power of two apart, so
    // without a rotation every workgroup would ask the same few memory channels
    // for its 128-byte pieces at the same time.  Workgroup b starts at K tile
    // b % KT and wraps around (a dot product does not care about the order).
    const int rot = blockIdx.x % KT;
    auto load_regs = [&](int kt, bf16x8 *xq, f32x4 *wq) {
        kt = kt < KT ? kt : KT - 1;                       // past the end: harmless reload of the last tile
        kt += rot;
        kt = kt < KT ? kt : kt - KT;
#pragma unroll
        for (int i = 0; i < 2; ++i)      // x is read once: streamed past the caches' retention
            xq[i] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8 *>(px[i] + (size_t)kt * (kRtBK * 2)));
#pragma unroll
        for (int i = 0; i < WL; ++i)
            if (w_lds[i] >= 0) wq[i] = *reinterpret_cast<const f32x4 *>(pw[i] + (size_t)kt * kRtBK);
    };
    typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
    auto store_regs = [&](char *stage, const bf16x8 *xq, const f32x4 *wq) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            *reinterpret_cast<bf16x8 *>(stage + (tid + kRtThreads * i) * 16) = xq[i];
#pragma unroll
        for (int i = 0; i < WL; ++i)
            if (w_lds[i] >= 0) {
                // w = hi + mid + lo exactly: 3 x 8 significand bits cover float32's 24
                bf16x4 hi, mid, lo;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bf16_t h = (bf16_t)wq[i][q];
                    const float r1 = wq[i][q] - (float)h;
                    const bf16_t m = (bf16_t)r1;
                    hi[q] = h;
                    mid[q] = m;
                    lo[q] = (bf16_t)(r1 - (float)m);
                }
                char *p = stage + kRtXBytes + w_lds[i];
                *reinterpret_cast<bf16x4 *>(p) = hi;
                *reinterpret_cast<bf16x4 *>(p + PIECE) = mid;
                *reinterpret_cast<bf16x4 *>(p + 2 * PIECE) = lo;
            }
    };
    // weight rows past the last one: zero in both stages, never written again
    for (int c = tid; c < 2 * 3 * (ROWS - rows) * (kRtRow / 16); c += kRtThreads) {
        const int st = c / (3 * (ROWS - rows) * (kRtRow / 16)), q = c % (3 * (ROWS - rows) * (kRtRow / 16));
        const int pc = q / ((ROWS - rows) * (kRtRow / 16)), o = q % ((ROWS - rows) * (kRtRow / 16));
        *reinterpret_cast<f32x4 *>(lds + st * STAGE + kRtXBytes + pc * PIECE + rows * kRtRow + o * 16) =
            f32x4{0.f, 0.f, 0.f, 0.f};
    }

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
    auto mfma_tile = [&](const char *cur) {
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

    // Tile j waits in register slot j % PF and is computed from LDS stage j % 2.
    // (Refilling slots in groups of consecutive K tiles, to hand DRAM longer
    // contiguous runs, was measured and is slower than one tile per period.)
#pragma unroll
    for (int p = 0; p < PF; ++p) load_regs(p, xr[p], wr[p]);
    store_regs(lds, xr[0], wr[0]);
    load_regs(PF, xr[0], wr[0]);
    // The epilogue's own operands (this block's previous-layer logits, W_g of the
    // gating residual, the bias) are asked for now and wait in registers: loaded
    // after the loop, their latency would sit on every workgroup's critical path.
    const int n_tok = min(kRtTok, T - t0);
    constexpr int PGN = ROWS / 4;                                      // >= N / 4
    constexpr int WRN = (ROWS * ROWS + kRtThreads - 1) / kRtThreads;   // >= N N / threads
    float pg[PGN], wg[WRN], bs = 0.f;
#pragma unroll
    for (int i = 0; i < PGN; ++i) {
        const int c = tid + kRtThreads * i;
        pg[i] = a.prev_gate && c < n_tok * N ? a.prev_gate[(size_t)t0 * N + c] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < WRN; ++i) {
        const int c = tid + kRtThreads * i;
        wg[i] = a.prev_gate && c < N * N ? a.W_res[c] : 0.f;
    }
    if (a.bias && tid < N) bs = a.bias[tid];
    lds_barrier();
    for (int kt0 = 0; kt0 < KT; kt0 += PF) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            const int kt = kt0 + s, q = (s + 1) % PF;     // q: slot of tile kt+1
            // tile kt+1: registers -> the stage that tile kt-1 was read from (every
            // wave passed the barrier after those reads), then refill the slot
            store_regs(lds + ((s + 1) & 1) * STAGE, xr[q], wr[q]);
            load_regs(kt + 1 + PF, xr[q], wr[q]);
            mfma_tile(lds + (s & 1) * STAGE);
            lds_barrier();                // tile kt+1 visible, tile kt read by all; loads stay in flight
        }
    }

    // ---- epilogue -------------------------------------------------------------
    // (the loop ended with a barrier: the stages are dead)
    float *dots = reinterpret_cast<float *>(lds);               // [kRtTok][DSTR]  K-step parity 0
    float *dots1 = dots + kRtTok * DSTR;                        // [kRtTok][DSTR]  K-step parity 1
    float *prevs = dots1 + kRtTok * DSTR;                       // [kRtTok][N + 1]
    float *wres = prevs + kRtTok * (kMaxExperts + 1);           // [N][N]
    float *sbias = wres + kMaxExperts * kMaxExperts;            // [N]
    int *s_hist = reinterpret_cast<int *>(sbias + kMaxExperts); // [N] selections per expert
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
    if (a.prev_gate) {
#pragma unroll
        for (int i = 0; i < PGN; ++i) {
            const int c = tid + kRtThreads * i;
            if (c < n_tok * N) prevs[(c / N) * (N + 1) + c % N] = pg[i];
        }
#pragma unroll
        for (int i = 0; i < WRN; ++i) {
            const int c = tid + kRtThreads * i;
            if (c < N * N) wres[c] = wg[i];
        }
    }
    if (tid < N) {                 // N <= 64 < threads
        sbias[tid] = bs;
        s_hist[tid] = 0;
    }
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

    // Softmax, Top-K, a1: threads 4 tok .. 4 tok + 3 share token tok (every thread
    // runs this, so the shuffles are whole; tokens past the end compute on a copy of
    // the last token and store nothing)
    {
        const int tok = tid >> 2;
        // (prevs is free again: the probabilities of the load-balance statistics go there)
        router_token_quad(a, (size_t)(t0 + tok), tok < n_tok, tid & 3, dots + tok * DSTR,
                          a.chunk_hist ? s_hist : nullptr, nullptr,
                          a.bal_partial ? prevs + tok * (N + 1) : nullptr);
    }
    // out_gate block [n_tok, N] is contiguous in memory: coalesced copy from LDS
    for (int c = tid; c < n_tok * N; c += kRtThreads)
        a.out_gate[(size_t)t0 * N + c] = dots[(c / N) * DSTR + c % N];
    if (a.chunk_hist || a.bal_partial) __syncthreads();
    if (a.chunk_hist)
        for (int c = tid; c < N; c += kRtThreads) a.chunk_hist[(size_t)blockIdx.x * N + c] = s_hist[c];
    if (a.bal_partial && tid < 4 * N) {
        // sum of Softmax(G(x))_e over the workgroup's tokens (P_e of Eq.7 is the mean over all
        // tokens): threads 4 e .. 4 e + 3 add a quarter of the tokens each, in token order, and
        // the four sums are added as (0 + 1) + (2 + 3): the same on every run
        const int e = tid >> 2, part = tid & 3;
        double sum = 0.0;
        for (int tt = part * (kRtTok / 4); tt < (part + 1) * (kRtTok / 4); ++tt)
            sum += (double)prevs[tt * (N + 1) + e];
        sum += __shfl_xor(sum, 1, kWave);
        sum += __shfl_xor(sum, 2, kWave);
        if (part == 0) a.bal_partial[(size_t)blockIdx.x * kMaxExperts + e] = sum;
    }
}

bool router_mfma_supported(const Dims &d) {
    // two 32-row blocks of weight rows at most; an even number of 64-wide K tiles
    return d.D % (2 * kRtBK) == 0 && d.N + 2 * d.n_const <= 64;
}

// Tokens per workgroup of the kernel launch_router_mfma picks for these sizes
// (also the tokens per chunk of the histogram it leaves for the permutation).
int router_mfma_block_tokens(const Dims &d) {
    const int rows = d.N + 2 * d.n_const;
    const int KT = d.D / kRtBK;
    // 128-token workgroups read the weight tiles half as often; 64-token ones
    // fill the chip sooner when there are few tokens
    return rows <= 32 && KT % 8 == 0 && d.T >= 24576 ? 128 : 64;
}

hipError_t launch_router_mfma(const RouterArgs &a, hipStream_t s) {
    if (a.d.T == 0) return hipSuccess;
    const int rows = a.d.N + 2 * a.d.n_const;
    const int nblk = (rows + 31) / 32;
    const int KT = a.d.D / kRtBK;
    const int tok = router_mfma_block_tokens(a.d);
    const dim3 grid((a.d.T + tok - 1) / tok);
    if (nblk == 1) {
        if (tok == 128)
            hipLaunchKernelGGL((k_router_mfma<1, 4, 128, 2>), grid, dim3(512), 0, s, a);
        else if (KT % 4 == 0)
            hipLaunchKernelGGL((k_router_mfma<1, 4, 64, 3>), grid, dim3(256), 0, s, a);
        else
            hipLaunchKernelGGL((k_router_mfma<1, 2, 64, 3>), grid, dim3(256), 0, s, a);
    } else {
        hipLaunchKernelGGL((k_router_mfma<2, 2, 64, 2>), grid, dim3(256), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace moepp
