// Grouped SwiGLU FFN for calls with a handful of rows per expert (decoding,
// small batches): the FFN experts of the layer (paper Eq.2) reduce to streaming
// every selected expert's weights past at most a few 16-row blocks of tokens.
//
//   GEMM1: h[r,f]    = silu(W1_e[f,:] . x_r) * (W3_e[f,:] . x_r),  x_r = x[src_of[r] / k]
//   GEMM2: yffn[r,d] = W2_e[d,:] . h[r,:]
//
// The kernel is bound by the weight stream (2.2 GB at the T = 64 workload
// against a few MB of activations), so it is built around that stream:
//  * an expert without rows is never touched: zero-computation slots and
//    unselected experts remove whole weight reads here (paper Sec. 3.4);
//  * work unit = (expert, block of 16 of its rows, panel of 256 packed weight
//    rows); the units of all experts form one list in that order, every four
//    neighbouring workgroups take a consecutive piece of it and each of the four
//    works on one of the panel's four groups of 64 rows, so a workgroup stays with
//    one expert (and one set of token operands) as long as it can, and what the
//    four read at about the same time is consecutive memory;
//  * the eight waves of a workgroup split the reduction over K: wave w owns K
//    steps [S w, S (w + 1)) of 32 and keeps its slice of the (at most 16) token
//    rows in registers as MFMA operands for as long as the row block stays the
//    same; per step it multiplies four 16-row weight fragments with them
//    (v_mfma_f32_16x16x32_bf16, 16 token rows is all the matrix core needs);
//  * the packed weight layout (panels of 256 rows, slabs of 32 columns) makes a
//    16-row x 32-column fragment 1 KB of consecutive memory and the four
//    fragments of a group 4 KB: every load is a whole-line, wave-wide load, 16 KB
//    per wave in flight (a ring of four steps that runs on across unit
//    boundaries, so the stream does not stop while the partial sums of a
//    unit meet), with the non-temporal hint: every weight is read once;
//  * the eight partial sums of a unit meet in LDS (two buffers, one barrier per
//    unit) and are added in wave order by all threads (the same on every
//    run), which apply SwiGLU and store.
// Rows past the end of a row block are clamped on load and masked on store.
#include "common.h"

#include <type_traits>

namespace moepp {

struct DecodeArgs {
    const bf16_t *A;         // GEMM1: x [T, ld] row-major; GEMM2: h, K-slab-major over h_rows rows
    const bf16_t *B;         // [n_ffn] matrices [Nb, K] in panels of K slabs (panel_row)
    bf16_t *C;               // GEMM1: h, K-slab-major over h_rows rows; GEMM2: yffn [R, ld] row-major
    const int32_t *offsets;  // [n_ffn + 1]
    const int32_t *src_of;   // GEMM1 only
    int ld, h_rows, K, Nb, n_ffn, topk;
};

constexpr int kDecWaves = 8;
constexpr int kDecThreads = kDecWaves * kWave;
constexpr int kDecRing = 4;                    // K steps of weights in flight per wave
constexpr int kDecMaxSteps = 24;               // K steps per wave at most: K <= 8 * 24 * 32 = 6144

__device__ inline float decode_silu(float z) {
    return z * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * z));
}

// S: K steps per wave (K = 256 S).  A unit takes S4 = S rounded up to a multiple
// of the ring depth positions of the stream; the positions S .. S4 - 1 are empty
// (no load, no MFMA), which keeps the ring slot of every step a compile-time
// constant across unit boundaries.  The loop over the units of one row block is
// free of branches around loads, so the compiler's wait counts stay exact
// (after a join of paths with different loads in flight it waits for all of them).
template <bool SWIGLU, int S>
__global__ __launch_bounds__(kDecThreads, 1) void k_ffn_decode(DecodeArgs a) {
    constexpr int S4 = (S + kDecRing - 1) / kDecRing * kDecRing;
    static_assert(S >= 1 && S4 <= kDecMaxSteps, "steps per wave");
    __shared__ __attribute__((aligned(16))) float part[2][kDecWaves][4][kWave][4];   // 64 KB
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int l16 = lane % 16, lq = lane / 16;
    const int ppe = (a.Nb + kPanel - 1) / kPanel;  // panels of 256 packed weight rows per expert
    // Four neighbouring workgroups share a list of (expert, row block, panel) and each takes one
    // of the panel's four groups of 64 rows: what they read at about the same time is the 16 KB
    // of consecutive memory of one K slab of the panel, not four pieces from four places.
    const int sub = blockIdx.x % 4, quad = blockIdx.x / 4, n_quads = gridDim.x / 4;

    // ---- the unit list: lane q looks after expert q --------------------------
    const int eq = lane < a.n_ffn ? lane : a.n_ffn;
    const int o_lo = a.offsets[eq];
    const int o_hi = a.offsets[eq < a.n_ffn ? eq + 1 : eq];
    const int units_q = ((o_hi - o_lo + 15) / 16) * ppe;      // 0 for an expert without rows
    int incl = units_q;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
    const int u0 = (int)((long long)total * quad / n_quads);
    const int u1 = (int)((long long)total * (quad + 1) / n_quads);
    if (u0 >= u1) return;

    // unit u -> expert, first row of its row block, rows in it, weight-row group, panel
    // (nrows = 0: the panel has no group for this workgroup; a valid one is computed, nothing stored)
    struct Unit {
        int e, row0, nrows, g, panel;
    };
    auto locate = [&](int u) {
        const unsigned long long past = __ballot(incl > u);
        Unit r;
        r.e = __builtin_ctzll(past);
        const int local = u - __builtin_amdgcn_readlane(incl - units_q, r.e);
        const int lo = __builtin_amdgcn_readlane(o_lo, r.e), hi = __builtin_amdgcn_readlane(o_hi, r.e);
        const int rb = local / ppe;                            // row blocks outermost: the token operands stay
        r.panel = local - rb * ppe;
        r.g = r.panel * 4 + sub;
        r.row0 = lo + 16 * rb;
        r.nrows = hi - r.row0 < 16 ? hi - r.row0 : 16;
        if (r.g * 64 >= a.Nb) {                                // a last panel with fewer than four groups
            r.g = a.Nb / 64 - 1;
            r.nrows = 0;
        }
        return r;
    };

    // ---- weight fragments: a ring of kDecRing steps -----------------------------
    // fragment (unit, step s, block b): 16 rows x 32 columns = 1 KB; lane l holds row l % 16,
    // columns 8 (l / 16) .. + 7
    bf16x8 wf[kDecRing][4];
    auto weight_ptr = [&](const Unit &un, int s) -> const char * {
        const int n0 = un.g * 64, p = n0 / kPanel;
        const int prow = a.Nb - p * kPanel < kPanel ? a.Nb - p * kPanel : kPanel;   // rows of the panel
        const size_t off = (size_t)un.e * a.Nb * a.K + (size_t)p * kPanel * a.K +
                           (size_t)(wave * S + s) * prow * kSlab + (size_t)(n0 - p * kPanel) * kSlab;
        return reinterpret_cast<const char *>(a.B + off) + l16 * 64 + lq * 16;
    };
    auto load_weights = [&](const Unit &un, int s, bf16x8 *dst) {
        const char *p = weight_ptr(un, s);
#pragma unroll
        for (int b = 0; b < 4; ++b)
            dst[b] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8 *>(p + b * 1024));
    };

    // ---- token operands of this wave's K slice -----------------------------------
    bf16x8 af[S];
    auto load_tokens = [&](const Unit &un) {
        int row = un.row0 + l16;
        const int last = un.row0 + (un.nrows > 0 ? un.nrows - 1 : 0);
        row = row < last ? row : last;
        const char *p;
        size_t step;
        if constexpr (SWIGLU) {
            const int tok = a.src_of[row] / a.topk;
            p = reinterpret_cast<const char *>(a.A + (size_t)tok * a.ld + (size_t)wave * S * 32) + lq * 16;
            step = 64;
        } else {
            p = reinterpret_cast<const char *>(a.A + (size_t)wave * S * a.h_rows * kSlab + (size_t)row * kSlab) + lq * 16;
            step = (size_t)a.h_rows * kSlab * 2;
        }
#pragma unroll
        for (int s = 0; s < S; ++s) af[s] = *reinterpret_cast<const bf16x8 *>(p + s * step);
    };

    f32x4 acc[4];
    auto clear_acc = [&]() {
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    };

    // ---- a finished unit: partial sums -> LDS -> all threads add, finish, store -----
    auto finish_unit = [&](const Unit &un, int buf) {
#pragma unroll
        for (int b = 0; b < 4; ++b) *reinterpret_cast<f32x4 *>(part[buf][wave][b][lane]) = acc[b];
        lds_barrier();         // orders LDS only: the weight loads of the next unit stay in flight
        // thread -> (block, lane of the accumulator layout, half of its four values)
        const int b = tid / 128, pl = (tid % 128) / 2, vh = tid % 2;
        const int m = pl % 16, n = 4 * (pl / 16) + 2 * vh;     // token row of the block, weight row of the 16
        const int row = un.row0 + m;
        typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
        if constexpr (SWIGLU) {
            // blocks 0, 1: rows of W1; blocks 2, 3: the same columns f of W3
            if (b < 2) {
                float z0 = 0.f, z1 = 0.f, g0 = 0.f, g1 = 0.f;
#pragma unroll
                for (int w = 0; w < kDecWaves; ++w) {          // wave order: the same on every run
                    z0 += part[buf][w][b][pl][2 * vh];
                    z1 += part[buf][w][b][pl][2 * vh + 1];
                    g0 += part[buf][w][b + 2][pl][2 * vh];
                    g1 += part[buf][w][b + 2][pl][2 * vh + 1];
                }
                if (m < un.nrows) {
                    bf16x2 o;
                    o[0] = (bf16_t)(decode_silu(z0) * g0);
                    o[1] = (bf16_t)(decode_silu(z1) * g1);
                    // column f = 32 g + 16 b + n of h, which is slab g
                    *reinterpret_cast<bf16x2 *>(a.C + (size_t)un.g * a.h_rows * kSlab + (size_t)row * kSlab + 16 * b + n) = o;
                }
            }
        } else {
            float y0 = 0.f, y1 = 0.f;
#pragma unroll
            for (int w = 0; w < kDecWaves; ++w) {
                y0 += part[buf][w][b][pl][2 * vh];
                y1 += part[buf][w][b][pl][2 * vh + 1];
            }
            if (m < un.nrows) {
                bf16x2 o;
                o[0] = (bf16_t)y0;
                o[1] = (bf16_t)y1;
                *reinterpret_cast<bf16x2 *>(a.C + (size_t)row * a.ld + 64 * un.g + 16 * b + n) = o;
            }
        }
    };

    // ---- the stream: unit after unit, S4 positions each --------------------------
    // While position s of a unit is multiplied, position s + kDecRing of the stream
    // is loaded into the ring slot that s just left: of this unit, or of the next
    // one (past the last unit of the workgroup: the last unit again, never used).
    int buf = 0;
    int u = u0;
    while (u < u1) {
        Unit cur = locate(u);
        const int seg_end = min(u1, u + (ppe - cur.panel));    // units that share cur's token operands
        load_tokens(cur);
#pragma unroll
        for (int r = 0; r < kDecRing; ++r)
            if (r < S) load_weights(cur, r, wf[r]);
        for (; u < seg_end; ++u) {
            const Unit nxt = locate(u + 1 < u1 ? u + 1 : u1 - 1);
            clear_acc();
#pragma unroll
            for (int s = 0; s < S4; ++s) {
                if constexpr (true) {
                    if (s < S) {
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[s % kDecRing][b], af[s], acc[b], 0, 0, 0);
                    }
                    const int pos = s + kDecRing;              // compile-time after unrolling
                    if (pos < S4) {
                        if (pos < S) load_weights(cur, pos, wf[s % kDecRing]);
                    } else if (pos - S4 < S) {
                        load_weights(nxt, pos - S4, wf[s % kDecRing]);
                    }
                }
                // (left alone, the compiler moves a load down to its first use, a ring later)
                __builtin_amdgcn_sched_barrier(0);
            }
            finish_unit(cur, buf);
            buf ^= 1;
            cur = nxt;
        }
        // (the next row block's first weights were loaded with another block's or with
        // this unit's addresses: the segment loop above reloads them; rare)
    }
}

// launch k_ffn_decode<., S> for the run-time S
template <int SMAX>
static hipError_t dispatch_steps(int S, int which, int n_cu, const DecodeArgs &a, hipStream_t s) {
    if constexpr (SMAX < 1) {
        return hipErrorInvalidValue;
    } else {
        if (S != SMAX) return dispatch_steps<SMAX - 1>(S, which, n_cu, a, s);
        if (which == 0)
            hipLaunchKernelGGL((k_ffn_decode<true, SMAX>), dim3(n_cu), dim3(kDecThreads), 0, s, a);
        else
            hipLaunchKernelGGL((k_ffn_decode<false, SMAX>), dim3(n_cu), dim3(kDecThreads), 0, s, a);
        return hipGetLastError();
    }
}

bool ffn_decode_supported(const Dims &d) {
    const long long slots = (long long)d.T * d.k;
    return d.n_ffn > 0 && d.n_ffn <= kWave && slots <= 16ll * d.n_ffn && d.D % 256 == 0 && d.F % 256 == 0 &&
           d.D <= kDecMaxSteps * 256 && d.F <= kDecMaxSteps * 256;
}

hipError_t launch_ffn_decode(const FfnArgs &f, int which, hipStream_t s) {
    if (f.d.T == 0 || f.d.n_ffn == 0) return hipSuccess;
    DecodeArgs a;
    a.offsets = f.offsets;
    a.src_of = f.src_of;
    a.n_ffn = f.d.n_ffn;
    a.topk = f.d.k;
    a.h_rows = f.h_rows;
    a.ld = f.d.D;
    if (which == 0) {
        a.A = (const bf16_t *)f.x;
        a.B = (const bf16_t *)f.w13;
        a.C = (bf16_t *)f.h;
        a.K = f.d.D;
        a.Nb = 2 * f.d.F;
    } else {
        a.A = (const bf16_t *)f.h;
        a.B = (const bf16_t *)f.w2;
        a.C = (bf16_t *)f.yffn;
        a.K = f.d.F;
        a.Nb = f.d.D;
    }
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 4)
            v = 256;
        n_cu = v / 4 * 4;             // workgroups come in fours (one panel each)
    }
    // one workgroup per CU; a workgroup without units returns at once
    const int S = a.K / (32 * kDecWaves);
    return dispatch_steps<kDecMaxSteps>(S, which, n_cu, a, s);
}

}  // namespace moepp
