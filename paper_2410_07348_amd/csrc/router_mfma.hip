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
// One workgroup = 4 waves x 32 tokens.  The weight rows (router rows, then
// the W_c rows) are staged through LDS in chunks of 256 K-elements, split on
// the fly; each wave reads its x fragments straight from global memory into
// MFMA operand registers, one chunk ahead.  The reduction index inside a
// 64-element group is permuted (the same way for x and for the weights, which
// leaves the dot product unchanged) so that the two lanes that share a token
// read 128 contiguous bytes.  Epilogue: one thread per token adds the gating
// residual and bias, then softmax and Top-K on the float32 logits (ties to
// the lower index, slots in descending order).
#include "common.h"

namespace moepp {

constexpr int kRtWaves = 4;
constexpr int kRtTok = 32 * kRtWaves;      // tokens per workgroup
constexpr int kRtKC = 256;                 // K elements per LDS chunk
constexpr int kRtRowBytes = kRtKC * 2;     // one weight row of one piece in LDS

template <int NBLK>   // 32-row blocks of weight rows
__global__ __launch_bounds__(kRtWaves *kWave, 1) void k_router_mfma(RouterArgs a) {
    constexpr int ROWS = NBLK * 32;
    constexpr int PIECE = ROWS * kRtRowBytes;             // bytes of one bf16 piece
    constexpr int DSTR = ROWS + 1;                        // floats per token in `dots`
    constexpr int W_BYTES = 3 * PIECE;
    constexpr int E_BYTES = (kRtTok * DSTR + kRtTok * (kMaxExperts + 1) +
                             kMaxExperts * kMaxExperts + kMaxExperts) * 4;
    constexpr int LDS_BYTES = W_BYTES > E_BYTES ? W_BYTES : E_BYTES;
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];

    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int l32 = lane % 32, lh = lane / 32;
    const int D = a.d.D, N = a.d.N, K = a.d.k, nc = a.d.n_const, T = a.d.T;
    const int rows = N + 2 * nc;
    const int t0 = blockIdx.x * kRtTok;

    // ---- x fragments: lane (token l32, half lh) ------------------------------
    int tok = t0 + wave * 32 + l32;
    tok = tok < T ? tok : T - 1;
    const bf16_t *xp = static_cast<const bf16_t *>(a.x) + (size_t)tok * D + lh * 32;
    // step s = 4*g + ss of a chunk covers elements g*64 + lh*32 + ss*8 .. +7
    bf16x8 xa[16], xb[16];
    auto load_x = [&](bf16x8 *dst, int chunk) {
#pragma unroll
        for (int s = 0; s < 16; ++s)
            dst[s] = *reinterpret_cast<const bf16x8 *>(xp + chunk * kRtKC + (s / 4) * 64 + (s % 4) * 8);
    };

    // ---- weight staging: thread -> (row, float4 index) -----------------------
    // 64 float4 per row and chunk; thread handles rows tid/64 + 4*it
    const int kq = tid % 64;
    f32x4 wreg[ROWS / 4];
    auto load_w = [&](int chunk) {
#pragma unroll
        for (int it = 0; it < ROWS / 4; ++it) {
            const int r = tid / 64 + 4 * it;
            const int rc = r < rows ? r : 0;        // rows past the last one read row 0, zeroed below
            const float *wr = rc < N ? a.W_g + (size_t)rc * D : a.W_c + (size_t)(rc - N) * D;
            f32x4 v = *reinterpret_cast<const f32x4 *>(wr + chunk * kRtKC + kq * 4);
            const float keep = r < rows ? 1.f : 0.f;
            wreg[it] = v * keep;
        }
    };
    auto store_w = [&]() {
        typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int it = 0; it < ROWS / 4; ++it) {
            const int r = tid / 64 + 4 * it;
            bf16x4 hi, mid, lo;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float w = wreg[it][q];
                const bf16_t h = (bf16_t)w;
                const float r1 = w - (float)h;
                const bf16_t m = (bf16_t)r1;
                const float r2 = r1 - (float)m;
                hi[q] = h;
                mid[q] = m;
                lo[q] = (bf16_t)r2;
            }
            // 16-byte slot (kq / 2) of the row, XOR-swizzled by row so that the
            // 32 rows read by one MFMA operand load spread over the banks
            const int off = r * kRtRowBytes + ((((kq >> 1) ^ (r & 15)) << 4) | ((kq & 1) << 3));
            *reinterpret_cast<bf16x4 *>(lds + off) = hi;
            *reinterpret_cast<bf16x4 *>(lds + PIECE + off) = mid;
            *reinterpret_cast<bf16x4 *>(lds + 2 * PIECE + off) = lo;
        }
    };

    f32x16 acc_hi[NBLK], acc_lo[NBLK];
#pragma unroll
    for (int b = 0; b < NBLK; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_hi[b][v] = acc_lo[b][v] = 0.f;

    const int n_chunks = D / kRtKC;
    // One chunk: publish its weights in LDS, start the loads of the next chunk,
    // then run the MFMAs on the x fragments that were loaded one chunk ago.
    auto phase = [&](int c, bf16x8 *cur, bf16x8 *nxt) {
        lds_barrier();                 // everyone is done reading the previous chunk
        store_w();
        lds_barrier();
        if (c + 1 < n_chunks) {
            load_w(c + 1);
            load_x(nxt, c + 1);
        }
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            // weight fragment: row l32 of block b, 16-byte slot (s/4)*8 + lh*4 + s%4
            const int slot = (s / 4) * 8 + lh * 4 + (s % 4);
#pragma unroll
            for (int b = 0; b < NBLK; ++b) {
                const int r = b * 32 + l32;
                const char *p = lds + r * kRtRowBytes + ((slot ^ (r & 15)) << 4);
                const bf16x8 whi = *reinterpret_cast<const bf16x8 *>(p);
                const bf16x8 wmid = *reinterpret_cast<const bf16x8 *>(p + PIECE);
                const bf16x8 wlo = *reinterpret_cast<const bf16x8 *>(p + 2 * PIECE);
                acc_hi[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(whi, cur[s], acc_hi[b], 0, 0, 0);
                acc_lo[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wmid, cur[s], acc_lo[b], 0, 0, 0);
                acc_lo[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wlo, cur[s], acc_lo[b], 0, 0, 0);
            }
        }
    };
    load_w(0);
    load_x(xa, 0);
    for (int c = 0; c < n_chunks; c += 2) {
        phase(c, xa, xb);
        if (c + 1 < n_chunks) phase(c + 1, xb, xa);
    }
    lds_barrier();                     // weights in LDS are dead from here on

    // ---- epilogue -------------------------------------------------------------
    float *dots = reinterpret_cast<float *>(lds);               // [kRtTok][DSTR]
    float *prevs = dots + kRtTok * DSTR;                        // [kRtTok][N + 1]
    float *wres = prevs + kRtTok * (kMaxExperts + 1);           // [N][N]
    float *sbias = wres + kMaxExperts * kMaxExperts;            // [N]
    // acc[b][v]: weight row b*32 + 8*(v/4) + 4*lh + v%4, token wave*32 + l32
#pragma unroll
    for (int b = 0; b < NBLK; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            dots[(wave * 32 + l32) * DSTR + b * 32 + 8 * (v / 4) + 4 * lh + (v % 4)] =
                acc_hi[b][v] + acc_lo[b][v];
    const int n_tok = min(kRtTok, T - t0);
    if (a.prev_gate) {
        for (int c = tid; c < n_tok * N; c += kRtWaves * kWave)
            prevs[(c / N) * (N + 1) + c % N] = a.prev_gate[(size_t)t0 * N + c];
        for (int c = tid; c < N * N; c += kRtWaves * kWave) wres[c] = a.W_res[c];
    }
    for (int c = tid; c < N; c += kRtWaves * kWave) sbias[c] = a.bias ? a.bias[c] : 0.f;
    lds_barrier();

    if (tid < n_tok) {
        float *Lr = dots + tid * DSTR;
        const float *pr = prevs + tid * (N + 1);
        float mx = -INFINITY;
        for (int i = 0; i < N; ++i) {
            float L = Lr[i];
            if (a.prev_gate) {
                float r = 0.f;
                for (int m = 0; m < N; ++m) r = fmaf(wres[i * N + m], pr[m], r);
                L += r;
            }
            L += sbias[i];
            Lr[i] = L;
            mx = fmaxf(mx, L);
        }
        float sum = 0.f;
        for (int i = 0; i < N; ++i) sum += expf(Lr[i] - mx);
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
            a.topk_w[t * K + s] = expf(bv - mx) * inv;
        }
        for (int j = 0; j < nc; ++j)
            a.alpha1[t * nc + j] = 1.f / (1.f + expf(Lr[N + 2 * j + 1] - Lr[N + 2 * j]));
    }
    lds_barrier();
    // out_gate block [n_tok, N] is contiguous in memory: coalesced copy from LDS
    for (int c = tid; c < n_tok * N; c += kRtWaves * kWave)
        a.out_gate[(size_t)t0 * N + c] = dots[(c / N) * DSTR + c % N];
}

bool router_mfma_supported(const Dims &d) {
    return d.D % kRtKC == 0 && d.N + 2 * d.n_const <= 96;
}

hipError_t launch_router_mfma(const RouterArgs &a, hipStream_t s) {
    if (a.d.T == 0) return hipSuccess;
    const int rows = a.d.N + 2 * a.d.n_const;
    dim3 grid((a.d.T + kRtTok - 1) / kRtTok), block(kRtWaves * kWave);
    if (rows <= 32)
        hipLaunchKernelGGL(k_router_mfma<1>, grid, block, 0, s, a);
    else if (rows <= 64)
        hipLaunchKernelGGL(k_router_mfma<2>, grid, block, 0, s, a);
    else
        hipLaunchKernelGGL(k_router_mfma<3>, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace moepp
