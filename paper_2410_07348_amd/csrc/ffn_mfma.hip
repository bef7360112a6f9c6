// Grouped SwiGLU FFN on the bf16 matrix cores (gfx950, v_mfma_f32_32x32x16_bf16).
//
// For every FFN expert e and the rows r of its group (paper Eq.2: the FFN
// experts of the layer; group sizes are ragged, they follow the routing):
//   GEMM1: h[r,f]    = silu(W1_e[f,:] . x_r) * (W3_e[f,:] . x_r),  x_r = x[src_of[r] / k]
//   GEMM2: yffn[r,d] = W2_e[d,:] . h[r,:]
// Both are C[m,n] = sum_k A[m,k] B[n,k] with A and B K-major, fp32 accumulation.
//
// Work decomposition: one workgroup per (M tile of one expert, N tile).  The
// M tiles are enumerated on the device from the group offsets (no host sync):
// expert e owns ceil(count_e / BM) tiles; surplus workgroups exit at once.
// A rows of GEMM1 are gathered straight from x through src_of (no permuted
// copy of x is ever written).  A and B tiles of 64 K-elements are staged in
// LDS (double buffered, 16-byte chunks XOR-swizzled by row so that the MFMA
// operand reads do not pile on one bank group); each wave owns a TM x TN
// sub-tile as 32x32 MFMA blocks.  The weight fragment is fed as the first MFMA
// operand, so a lane ends up with four consecutive output columns of one row
// and the epilogue can pack them into one 8-byte LDS write; the output tile is
// then written to memory with 16-byte row-contiguous stores.
//
// GEMM1 reads the packed [2F, D] matrix in which W1 and W3 rows alternate in
// blocks of 32: 32x32 blocks with even index hold silu's argument, the next
// block its multiplier for the same 32 columns f, in the same registers of the
// same lane, so SwiGLU is applied in registers.
#include "common.h"

namespace moepp {

struct GemmArgs {
    const bf16_t *A;         // GEMM1: x [T, lda]; GEMM2: h [R, lda]
    const bf16_t *B;         // [n_ffn][Nb][K]
    bf16_t *C;               // [R, ldc]
    const int32_t *offsets;  // [n_ffn + 1]
    const int32_t *src_of;   // GEMM1 only
    int lda, ldc;
    int K;                   // reduction length (multiple of 64)
    int Nb;                  // rows of B per expert (2F or D)
    int Nc;                  // columns of C (F or D)
    int n_ffn, topk;
    int n_ntiles;
};

constexpr int BK = 64;                 // K elements per LDS tile (128 bytes per row)
constexpr int kRowBytes = BK * 2;

__device__ inline float fast_silu(float z) { return z * __frcp_rn(1.f + __expf(-z)); }

template <int BM, int BN, int WM, int WN, bool SWIGLU>
__global__ __launch_bounds__(WM *WN *kWave, 1) void k_grouped_gemm(GemmArgs a) {
    constexpr int NT = WM * WN * kWave;
    constexpr int TM = BM / WM, TN = BN / WN;     // wave tile
    constexpr int MB = TM / 32, NB = TN / 32;     // 32x32 blocks per wave
    constexpr int CA = BM * 8 / NT, CB = BN * 8 / NT;   // 16-byte chunks per thread
    constexpr int STAGE = (BM + BN) * kRowBytes;
    constexpr int OUT_W = SWIGLU ? BN / 2 : BN;   // output tile width (elements)
    constexpr int OUT_STRIDE = OUT_W * 2 + 16;    // bytes, padded
    constexpr int OUT_BYTES = BM * OUT_STRIDE;
    constexpr int LDS_BYTES = 2 * STAGE > OUT_BYTES ? 2 * STAGE : OUT_BYTES;
    static_assert(TM % 32 == 0 && TN % 64 == 0, "wave tile");
    static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0 && (NT / 8) % 8 == 0, "chunks");
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid % kWave;
    const int wave = tid / kWave;
    const int wm = wave / WN, wn = wave % WN;

    // ---- which tile --------------------------------------------------------
    const int nt = blockIdx.x % a.n_ntiles;
    const int mt = blockIdx.x / a.n_ntiles;
    int e = 0, row0 = 0, row_end = 0;
    {
        int acc_t = 0;
        bool found = false;
        for (e = 0; e < a.n_ffn; ++e) {
            const int b = a.offsets[e], en = a.offsets[e + 1];
            const int nte = (en - b + BM - 1) / BM;
            if (mt < acc_t + nte) {
                row0 = b + (mt - acc_t) * BM;
                row_end = en;
                found = true;
                break;
            }
            acc_t += nte;
        }
        if (!found) return;
    }
    const int n0 = nt * BN;

    // ---- global -> register -> LDS staging ----------------------------------
    const int kc = tid % 8;              // 16-byte chunk within the 128-byte tile row
    const int r_thr = tid / 8;           // tile row of this thread's first chunk
    const bf16_t *pa[CA];
    const bf16_t *pb[CB];
#pragma unroll
    for (int i = 0; i < CA; ++i) {
        int r = row0 + r_thr + i * (NT / 8);
        r = r < row_end ? r : row_end - 1;
        const int src = SWIGLU ? a.src_of[r] / a.topk : r;
        pa[i] = a.A + (size_t)src * a.lda + kc * 8;
    }
    const bf16_t *Be = a.B + (size_t)e * a.Nb * a.K;
#pragma unroll
    for (int i = 0; i < CB; ++i) {
        int n = n0 + r_thr + i * (NT / 8);
        n = n < a.Nb ? n : a.Nb - 1;
        pb[i] = Be + (size_t)n * a.K + kc * 8;
    }
    const int st_off = r_thr * kRowBytes + ((kc ^ (r_thr & 7)) << 4);

    bf16x8 ra[CA], rb[CB];
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int i = 0; i < CA; ++i) ra[i] = *reinterpret_cast<const bf16x8 *>(pa[i] + kt * BK);
#pragma unroll
        for (int i = 0; i < CB; ++i) rb[i] = *reinterpret_cast<const bf16x8 *>(pb[i] + kt * BK);
    };
    auto store_tile = [&](int stage) {
        char *sa = lds + stage * STAGE;
        char *sb = sa + BM * kRowBytes;
#pragma unroll
        for (int i = 0; i < CA; ++i)
            *reinterpret_cast<bf16x8 *>(sa + st_off + i * (NT / 8) * kRowBytes) = ra[i];
#pragma unroll
        for (int i = 0; i < CB; ++i)
            *reinterpret_cast<bf16x8 *>(sb + st_off + i * (NT / 8) * kRowBytes) = rb[i];
    };

    // ---- MFMA operand addressing --------------------------------------------
    // lane l reads row (l % 32) of a 32-row block, K half (l / 32) of each 16-wide step
    const int l32 = lane % 32, lh = lane / 32;
    int rd_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) rd_off[ks] = l32 * kRowBytes + (((2 * ks + lh) ^ (l32 & 7)) << 4);
    const int a_base = (wm * TM) * kRowBytes;
    const int b_base = BM * kRowBytes + (wn * TN) * kRowBytes;

    f32x16 acc[NB][MB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.f;

    const int KT = a.K / BK;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more) load_tile(kt + 1);
        const char *s = lds + (kt & 1) * STAGE;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 fa[MB], fb[NB];
#pragma unroll
            for (int i = 0; i < MB; ++i)
                fa[i] = *reinterpret_cast<const bf16x8 *>(s + a_base + i * 32 * kRowBytes + rd_off[ks]);
#pragma unroll
            for (int j = 0; j < NB; ++j)
                fb[j] = *reinterpret_cast<const bf16x8 *>(s + b_base + j * 32 * kRowBytes + rd_off[ks]);
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int i = 0; i < MB; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[j][i], 0, 0, 0);
        }
        if (more) store_tile((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: registers -> LDS tile -> 16-byte row-contiguous stores ----
    // acc[j][i][v]: output row m = wm*TM + i*32 + l32,
    //               B row n = wn*TN + j*32 + 8*(v/4) + 4*lh + v%4
    // (the last loop iteration ended with a barrier: all waves are done reading)
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        const int m = wm * TM + i * 32 + l32;
        char *orow = lds + m * OUT_STRIDE;
        if constexpr (SWIGLU) {
#pragma unroll
            for (int j = 0; j < NB; j += 2) {
                const int c0 = (wn * TN + j * 32) / 2 + 4 * lh;   // 32 columns per block pair
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
                    bf16x4 o;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        o[q] = (bf16_t)(fast_silu(acc[j][i][4 * g + q]) * acc[j + 1][i][4 * g + q]);
                    *reinterpret_cast<bf16x4 *>(orow + (c0 + 8 * g) * 2) = o;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int c0 = wn * TN + j * 32 + 4 * lh;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
                    bf16x4 o;
#pragma unroll
                    for (int q = 0; q < 4; ++q) o[q] = (bf16_t)acc[j][i][4 * g + q];
                    *reinterpret_cast<bf16x4 *>(orow + (c0 + 8 * g) * 2) = o;
                }
            }
        }
    }
    __syncthreads();
    constexpr int CPR = OUT_W / 8;                 // 16-byte chunks per output row
    const int c_col0 = SWIGLU ? n0 / 2 : n0;
    for (int c = tid; c < BM * CPR; c += NT) {
        const int m = c / CPR, cc = c % CPR;
        const int row = row0 + m, col = c_col0 + cc * 8;
        if (row < row_end && col < a.Nc)
            *reinterpret_cast<bf16x8 *>(a.C + (size_t)row * a.ldc + col) =
                *reinterpret_cast<const bf16x8 *>(lds + m * OUT_STRIDE + cc * 16);
    }
}

bool ffn_mfma_supported(const Dims &d) { return d.D % BK == 0 && d.F % BK == 0; }

template <int BM, int BN, int WM, int WN>
static hipError_t launch_cfg(const FfnArgs &f, int which, hipStream_t s) {
    GemmArgs a;
    a.offsets = f.offsets;
    a.src_of = f.src_of;
    a.n_ffn = f.d.n_ffn;
    a.topk = f.d.k;
    if (which == 0) {
        a.A = (const bf16_t *)f.x;
        a.lda = f.d.D;
        a.B = (const bf16_t *)f.w13;
        a.K = f.d.D;
        a.Nb = 2 * f.d.F;
        a.C = (bf16_t *)f.h;
        a.ldc = f.d.F;
        a.Nc = f.d.F;
    } else {
        a.A = (const bf16_t *)f.h;
        a.lda = f.d.F;
        a.B = (const bf16_t *)f.w2;
        a.K = f.d.F;
        a.Nb = f.d.D;
        a.C = (bf16_t *)f.yffn;
        a.ldc = f.d.D;
        a.Nc = f.d.D;
    }
    a.n_ntiles = (a.Nb + BN - 1) / BN;
    const long long rows = (long long)f.d.T * f.d.k;
    const long long max_mtiles = (rows + BM - 1) / BM + f.d.n_ffn;   // upper bound of sum ceil(count_e/BM)
    const long long blocks = max_mtiles * a.n_ntiles;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks), block(WM * WN * kWave);
    if (which == 0)
        hipLaunchKernelGGL((k_grouped_gemm<BM, BN, WM, WN, true>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((k_grouped_gemm<BM, BN, WM, WN, false>), grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_ffn_mfma(const FfnArgs &f, int which, hipStream_t s) {
    if (f.d.T == 0 || f.d.n_ffn == 0) return hipSuccess;
    return launch_cfg<256, 256, 2, 4>(f, which, s);
}

}  // namespace moepp
