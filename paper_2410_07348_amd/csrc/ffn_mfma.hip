// Grouped SwiGLU FFN on the bf16 matrix cores (gfx950, v_mfma_f32_16x16x32_bf16 by
// default, v_mfma_f32_32x32x16_bf16 as an option).
//
// For every FFN expert e and the rows r of its group (paper Eq.2: the FFN
// experts of the layer; group sizes are ragged, they follow the routing):
//   GEMM1: h[r,f]    = silu(W1_e[f,:] . x_r) * (W3_e[f,:] . x_r),  x_r = x[src_of[r] / k]
//   GEMM2: yffn[r,d] = W2_e[d,:] . h[r,:]
// Both are C[m,n] = sum_k A[m,k] B[n,k] with A and B K-major, fp32 accumulation.
//
// Work decomposition: output tiles of BM x BN (256 x 256 by default; M tiles
// never cross an expert).  The tiles are enumerated on the device from the
// group offsets (no host sync): expert e owns ceil(count_e / BM) M tiles; the
// numbering walks patches of 8 x 4 tiles and deals the patches to the eight
// XCDs round-robin, so that the tiles that run together on one XCD share their
// A and B panels in that XCD's L2.  In the default (persistent) geometry one
// workgroup per CU walks the tile list with stride gridDim; it looks up and
// gathers the rows of its next tile while the current one computes and issues
// that tile's first K stages before the epilogue of the current one.  When
// the whole problem is only a few rounds of tiles, a last round that fills at
// most half of the workgroups is left to a second launch of the same kernel
// with tiles of half the height (twice as many workgroups busy for about half
// as long).
// A rows of GEMM1 are gathered straight from x through src_of (no permuted
// copy of x is ever written).  K tiles of 32 elements travel from memory
// straight into a ring of LDS stages (global_load_lds, 16-byte chunks
// XOR-swizzled by row so that the MFMA operand reads do not pile on one bank
// group); a few dedicated loader waves issue them, one memory instruction after
// each MFMA, and every wave owns a (BM/WM) x (BN/WN) sub-tile of MFMA blocks.
// The weight fragment is fed as the first MFMA operand, so a lane ends up with
// four consecutive output columns of one row and the epilogue can pack them
// into one 8-byte LDS write; the output tile is then written to memory with
// 16-byte row-contiguous stores.  The weights are read from a packed copy in
// panels of 256 rows x K slabs (one K tile of a panel is contiguous); GEMM1
// writes h in K-slab-major order so that GEMM2's A tiles are contiguous too.
//
// GEMM1 reads the packed [2F, D] matrix in which W1 and W3 rows alternate in
// blocks of 32: 32x32 blocks with even index hold silu's argument, the next
// block its multiplier for the same 32 columns f, in the same registers of the
// same lane, so SwiGLU is applied in registers.
#include "common.h"

#include <type_traits>

namespace moepp {

struct GemmArgs {
    const bf16_t *A;         // GEMM1: x [T, ld] row-major; GEMM2: h, K-slab-major over h_rows rows
    const bf16_t *B;         // [n_ffn] matrices [Nb, K] in panels of K slabs (panel_row)
    bf16_t *C;               // GEMM1: h, K-slab-major over h_rows rows; GEMM2: yffn [R, ld] row-major
    const int32_t *offsets;  // [n_ffn + 1]
    const int32_t *src_of;   // GEMM1 only
    int ld;                  // row length of the row-major operand (x or yffn)
    int h_rows;              // rows of the slab-major h buffer
    int K;                   // reduction length (multiple of 64)
    int Nb;                  // rows of B per expert (2F or D)
    int Nc;                  // columns of C (F or D)
    int n_ffn, topk;
    int n_ntiles;
    int jstride;             // persistent kernel: workgroups per XCD
    int cut_grid;            // > 0: the tiles of a last, at most half-filled round of cut_grid
                             // workgroups are left to the tail kernel (halves of 128 rows)
};

// silu(z) = z / (1 + e^-z) with the hardware exp2 and reciprocal (1 ulp each:
// far inside the rounding of the bf16 result).  A correctly rounded division
// costs ten more instructions per element, a third of the epilogue.
__device__ inline float fast_silu(float z) {
    return z * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * z));
}

typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

// Tile geometry.  BK K-elements per LDS stage; NS stages form a ring, NS - 1
// tiles are in flight (or being computed) at any time.
// LW_ of the WM*WN waves issue the tile loads (0: all of them).
// MI_: edge of the MFMA block, 32 (v_mfma_f32_32x32x16_bf16) or 16 (v_mfma_f32_16x16x32_bf16).
template <int BM_, int BN_, int WM_, int WN_, int BK_, int NS_, int LW_ = 0, bool PERSIST_ = false,
          int MI_ = 32>
struct Geo {
    static constexpr int MI = MI_;
    static constexpr bool PAIR = MI_ == 16;            // GEMM1 issues the A loads of two K tiles together
    static_assert(MI_ == 32 || (MI_ == 16 && BK_ == 32 && NS_ >= 3), "16x16x32 blocks: one MFMA K step per 32-deep stage, ring path");
    static constexpr bool PERSIST = PERSIST_;          // one workgroup per CU runs tile after tile
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = BK_, NS = NS_;
    static constexpr int NT = WM * WN * kWave;         // threads
    static constexpr int LW = LW_ ? LW_ : WM * WN;     // waves that issue the tile loads
    static constexpr int NL = LW * kWave;              // ... and their threads
    static constexpr int RB = BK * 2;                  // bytes per tile row
    static constexpr int CPR = RB / 16;                // 16-byte slots per tile row
    static constexpr int TM = BM / WM, TN = BN / WN;   // wave tile
    static constexpr int MB = TM / 32, NB = TN / 32;   // 32x32 MFMA blocks per wave
    static constexpr int CA = BM * CPR / NL, CB = BN * CPR / NL;   // loads per loading thread and tile
    static constexpr int STAGE = (BM + BN) * RB;
    static constexpr int KS = BK / 16;                 // MFMA K steps per stage
    static constexpr int LPT = CA + CB;                // wave-wide loads per thread and tile
    static constexpr int LPS = LPT / KS;               // tile loads per loading thread and K step
    static_assert(LPT % KS == 0, "tile loads per K step");
    static_assert(TM % 32 == 0 && TN % 64 == 0, "wave tile");
    static_assert((BM * CPR) % NL == 0 && (BN * CPR) % NL == 0 && (NL / CPR) % 16 == 0, "chunks");
    static_assert(BK == 32 || BK == 64, "BK");
    // XOR swizzle of the 16-byte slots of a tile row.  The LDS has 64 banks of
    // 4 bytes (256 bytes) and serves a b128 operand read in four passes of 16
    // lanes; a pass takes lanes {0-3, 12-15, 20-27} or {4-11, 16-19, 28-31} of
    // a half wave (measured: two lanes of one such set that address the same
    // banks cost an extra pass).  The 32x32 operand read (lane l: row l % 32,
    // one slot per half wave) wants any 16 consecutive rows at one logical
    // slot on 16 different bank groups; the 16x16 operand read (lane l: row
    // l % 16, slot l / 16, 64-byte rows) wants that of rows {0-3, 12-15} at
    // one slot together with rows {4-11} at the next, which a swizzle by
    // row / 2 gives and the swizzle by row / 4 does not (two passes per set).
    __device__ static int swz(int row) {
        if constexpr (MI == 16) return (row / 2) % CPR;
        else return (row / (256 / RB)) % CPR;
    }
};

// s_waitcnt vmcnt(VM) lgkmcnt(0), then the workgroup barrier.  The wait is
// the builtin (so the compiler's own counter tracking sees it) and the empty
// asm statements keep every memory access on its side of the barrier; no
// fence builtin is used because it would also wait for the younger
// direct-to-LDS loads, which count as LDS writes.
// Workgroup barrier for plain LDS traffic while direct-to-LDS loads of a later
// tile are in flight: __syncthreads() would wait for those too.
__device__ inline void lds_sync() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int VM>
__device__ inline void wait_and_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((VM & 15) | 0x70 | ((VM >> 4) << 14));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// TAIL: this launch computes what the main launch (tiles of 2 BM rows) left
// over, as half tiles of BM rows; the tiles are numbered as in the main launch.
template <class G, bool SWIGLU, bool TAIL = false>
__global__ __launch_bounds__(G::NT, 1) void k_grouped_gemm(GemmArgs a) {
    constexpr int EBM = TAIL ? 2 * G::BM : G::BM;      // tile height of the numbering
    constexpr int BM = G::BM, BN = G::BN, WN = G::WN, NT = G::NT, NL = G::NL, RB = G::RB, CPR = G::CPR;
    constexpr int TM = G::TM, TN = G::TN, MB = G::MB, NB = G::NB, CA = G::CA, CB = G::CB;
    constexpr int STAGE = G::STAGE, NS = G::NS, BK = G::BK, KS = G::KS;
    // The output tile goes through LDS in EP passes of HB rows (one pass for
    // GEMM1, whose tile is half as wide after SwiGLU).
    constexpr int OUT_W = SWIGLU ? BN / 2 : BN;   // output tile width (elements)
    constexpr int OUT_STRIDE = OUT_W * 2 + 16;    // bytes, padded
    constexpr int EP = SWIGLU || BM < 256 ? 1 : 2;
    constexpr int HB = BM / EP;
    constexpr int OUT_BYTES = HB * OUT_STRIDE;
    static_assert(TM <= HB && HB % TM == 0, "a wave's rows belong to one epilogue pass");
    constexpr int LDS_BYTES = NS * STAGE > OUT_BYTES ? NS * STAGE : OUT_BYTES;
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    // A persistent workgroup (G::PERSIST) runs tile after tile.  The stages
    // the epilogue's LDS patch does not touch, S0 .. NS-1, take the first K
    // tiles of the NEXT output tile while the epilogue of this one runs, so
    // every output tile's ring starts at stage S0.
    constexpr int S0 = G::PERSIST ? (OUT_BYTES + STAGE - 1) / STAGE : 0;
    constexpr int EARLY = G::PERSIST ? NS - S0 : 0;      // K tiles issued before the epilogue
    static_assert(!G::PERSIST || (EARLY >= 1 && EARLY <= NS - 1), "stages free during the epilogue");

    const int tid = threadIdx.x;
    const int lane = tid % kWave;
    const int wave = tid / kWave;
    const int wm = wave / WN, wn = wave % WN;

    // ---- which tiles ---------------------------------------------------------
    // Workgroups are handed to the 8 XCDs round-robin by id, and every XCD has
    // its own L2.  All tiles are put in one linear order in which 32
    // consecutive tiles form a patch of GM m-tiles x GN n-tiles of one expert
    // (they share GM + GN operand panels instead of 64): an XCD's 32 CUs work
    // on one patch at a time out of their L2.  The patches are dealt to the
    // XCDs round-robin, so at any time the 8 XCDs hold 8 neighbouring patches
    // (same rows, next columns): what one XCD fetched from HBM the others
    // find in the memory-side cache.  Tile j of XCD x is run by workgroup
    // x + 8*(j % jstride), jstride = workgroups per XCD (persistent kernel) or
    // by workgroup x + 8*j (one tile per workgroup).  The order is computed
    // here from the group offsets.
    // Assumes the part this library is written for, MI355X in its default (SPX)
    // partition mode: 8 XCDs of 32 CUs, workgroup w dispatched to XCD w % 8.  On
    // another partitioning the tile order is still a valid enumeration (every tile
    // is computed once), only the sharing in L2 it is built for is lost.
    constexpr int GM = 8, GN = 4, NXCD = 8;
    const int Nt = a.n_ntiles;
    // Lane q holds group q: one vector load of the offsets, a wave-wide prefix
    // sum of the tile counts, a ballot to find the group of a tile (a scalar
    // loop over the groups costs a dependent memory round trip per group).
    const int gq = lane < a.n_ffn ? lane : a.n_ffn;
    const int o_lo = a.offsets[gq];
    const int o_hi = a.offsets[gq < a.n_ffn ? gq + 1 : gq];
    const int mt_q = (o_hi - o_lo + EBM - 1) / EBM;            // 0 for lanes past the last group
    int incl = mt_q * Nt;                                       // inclusive prefix sum over lanes
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
    // A last round that fills at most half of the workgroups costs a whole
    // tile time with most of the chip idle: those tiles [cut, total) go to the
    // tail launch, which runs them as twice as many half tiles.
    int cut = total;
    if (a.cut_grid > 0) {
        const int n_left = total % a.cut_grid;
        if (n_left > 0 && 2 * n_left <= a.cut_grid) cut = total - n_left;
    }

    int e = 0, row0 = 0, row_end = 0, nt = 0;                  // the tile being computed
    // tile j of this XCD -> (expert, first row, end of the group, n-tile); false past the end
    auto locate = [&](int j, int &t_e, int &t_row0, int &t_row_end, int &t_nt) -> bool {
        // XCD x takes patch-sized chunks x, x+8, x+16, ... of the order
        int L = ((j / (GM * GN)) * NXCD + blockIdx.x % NXCD) * (GM * GN) + j % (GM * GN);
        int half = 0;
        if constexpr (TAIL) {
            half = L & 1;
            L = cut + (L >> 1);
            if (L >= total) return false;
        } else {
            if (L >= cut) return false;
            // GEMM2 walks the order backwards: it starts with the rows of h that GEMM1
            // wrote last, which are the ones still in the memory-side cache (-0.6 %)
            if constexpr (!SWIGLU) L = cut - 1 - L;
        }
        const unsigned long long past = __ballot(incl > L);     // lanes whose groups end after tile L
        t_e = __builtin_ctzll(past);                            // L < total, so some lane has incl > L
        // (t_e is the same in every lane: these are scalar reads of lane t_e)
        L -= __builtin_amdgcn_readlane(incl - mt_q * Nt, t_e);
        const int b = __builtin_amdgcn_readlane(o_lo, t_e);
        t_row_end = __builtin_amdgcn_readlane(o_hi, t_e);
        const int mt_e = __builtin_amdgcn_readlane(mt_q, t_e);
        // inside the expert: m-groups of GM m-tiles, n-groups of GN n-tiles, m fastest
        const int n_g = (mt_e + GM - 1) / GM;
        int g = L / (GM * Nt);
        g = g < n_g - 1 ? g : n_g - 1;
        const int gm = g < n_g - 1 ? GM : mt_e - GM * (n_g - 1);
        L -= g * GM * Nt;
        const int NG = (Nt + GN - 1) / GN;
        int ng = L / (gm * GN);
        ng = ng < NG - 1 ? ng : NG - 1;
        L -= ng * gm * GN;
        const int mt = g * GM + L % gm;
        t_nt = ng * GN + L / gm;
        // (the second half of a group's last tile may lie past the group's rows: it
        // is computed like any other and stores nothing)
        t_row0 = b + mt * EBM + half * BM;
        return true;
    };

    // ---- global -> LDS, written by the load itself ----------------------------
    // Chunk c = tid + i*NL of a tile (tid < NL: the loading waves): row c/CPR,
    // 16-byte slot c%CPR.  One wave-wide load fills 1 KB of consecutive tile
    // rows: lane l lands at base + 16*l.  Slot s of row r holds global chunk
    // s ^ swz(r) of that row, so each lane fetches the global chunk that
    // belongs in its slot.
    const int slot = tid % CPR;
    const int r_thr = tid / CPR;                 // tile row of this thread's first chunk
    const int kc = slot ^ G::swz(r_thr);         // global chunk within the K tile
    const bf16_t *pa[CA];
    const bf16_t *pb[CB];
    size_t b_kstep = 0;                          // elements of B from one K tile to the next
    static_assert(BN == kPanel, "one tile of B rows is one panel of the packed weights");
    // rows of A (of x through src_of for GEMM1, of h for GEMM2) this thread loads for a tile
    auto gather_rows = [&](int t_row0, int t_row_end, int *src) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            int r = t_row0 + r_thr + i * (NL / CPR);
            r = r < t_row_end ? r : t_row_end - 1;
            src[i] = SWIGLU ? a.src_of[r] / a.topk : r;
        }
    };
    auto set_pointers = [&](int t_e, int t_nt, const int *src) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            // chunk kc of the tile: slab kc/4 of the tile's K range, 16-byte piece kc%4 of the slab row
            pa[i] = SWIGLU ? a.A + (size_t)src[i] * a.ld + kc * 8
                           : a.A + (size_t)(kc / 4) * a.h_rows * kSlab + (size_t)src[i] * kSlab + (kc % 4) * 8;
        }
        const bf16_t *Be = a.B + (size_t)t_e * a.Nb * a.K;
        const int n0 = t_nt * BN;
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            int n = n0 + r_thr + i * (NL / CPR);
            n = n < a.Nb ? n : a.Nb - 1;
            pb[i] = Be + panel_row(n, kc / 4, a.Nb, a.K) + (kc % 4) * 8;
        }
        const int b_rows = a.Nb - n0 < BN ? a.Nb - n0 : BN;     // rows of this tile's panel
        b_kstep = (size_t)(BK / kSlab) * b_rows * kSlab;
    };
    const int wave_off = __builtin_amdgcn_readfirstlane(wave) * 1024;   // this wave's 1 KB of each load group

    const int KT = a.K / BK;
    // elements of A from one K tile to the next
    const size_t a_kstep = SWIGLU ? (size_t)BK : (size_t)(BK / kSlab) * a.h_rows * kSlab;
    // Load q of the LPT = CA + CB wave-wide loads that make up a tile.
    auto issue_one = [&](int q, int kt, char *__restrict__ stage) {
        char *sa = stage + wave_off;
        char *sb = sa + BM * RB;
        if (q < CA)
            __builtin_amdgcn_global_load_lds((gptr_t)(pa[q] + kt * a_kstep),
                                             (lptr_t)(sa + q * (NL / CPR) * RB), 16, 0, 0);
        else
            __builtin_amdgcn_global_load_lds((gptr_t)(pb[q - CA] + kt * b_kstep),
                                             (lptr_t)(sb + (q - CA) * (NL / CPR) * RB), 16, 0, 0);
    };
    auto issue_tile = [&](int kt, char *__restrict__ stage) {
#pragma unroll
        for (int q = 0; q < CA + CB; ++q) issue_one(q, kt, stage);
    };
    // K tiles [first, last) of the current pointers into their ring stages
    // (tile kt: stage (S0 + kt) % NS of the ring at `ring`).  KT >= NS - 1.
    auto issue_range = [&](int first, int last, char *__restrict__ ring) {
#pragma unroll
        for (int p = 0; p < NS - 1; ++p)
            if (p >= first && p < last) issue_tile(p, ring + ((S0 + p) % NS) * STAGE);
    };

    // ---- MFMA operand addressing --------------------------------------------
    // lane l reads row (l % 32) of a 32-row block, K half (l / 32) of each 16-wide step
    const int l32 = lane % 32, lh = lane / 32;
    int rd_off[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        rd_off[ks] = l32 * RB + (((2 * ks + lh) ^ G::swz(l32)) << 4);
    const int a_base = (wm * TM) * RB;
    const int b_base = BM * RB + (wn * TN) * RB;

    // accumulators: 32x32 blocks of 16 registers, or 16x16 blocks of 4
    constexpr int MI = G::MI;
    constexpr int NBX = TN / MI, MBX = TM / MI;
    typedef typename std::conditional<MI == 32, f32x16, f32x4>::type acc_t;
    acc_t acc[NBX][MBX];
    // 16x16x32 blocks: lane l reads row (l % 16) of a 16-row block, 16-byte chunk l / 16 of its 64-byte row
    const int l16 = lane % 16, lq = lane / 16;
    const int rd16 = l16 * RB + ((lq ^ G::swz(l16)) << 4);

    auto read_frags = [&](const char *st, int ks, bf16x8 *fa, bf16x8 *fb) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
            fa[i] = *reinterpret_cast<const bf16x8 *>(st + a_base + i * 32 * RB + rd_off[ks]);
#pragma unroll
        for (int j = 0; j < NB; ++j)
            fb[j] = *reinterpret_cast<const bf16x8 *>(st + b_base + j * 32 * RB + rd_off[ks]);
    };
    auto mfma32 = [&](bf16x8 b, bf16x8 a_, auto &c) {
        if constexpr (MI == 32) c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a_, c, 0, 0, 0);
    };
    auto mfma16 = [&](bf16x8 b, bf16x8 a_, auto &c) {
        if constexpr (MI == 16) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, a_, c, 0, 0, 0);
    };
    auto mfma_step = [&](const bf16x8 *fa, const bf16x8 *fb) {
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int i = 0; i < MB; ++i) mfma32(fb[j], fa[i], acc[j][i]);
    };
    // One K step with its memory operations spread evenly between the MFMAs:
    // first the operand reads of the NEXT step (from `st`, step `ks_rd`, into
    // fa_n/fb_n), then N_LOAD of the loads of tile kt_issue.  A wave issues in
    // order: a burst of reads or loads between two MFMAs leaves the matrix
    // core idle, a single one does not.
    auto mfma_step_mem = [&](const bf16x8 *fa, const bf16x8 *fb, int ks, bool do_read,
                             const char *__restrict__ st, int ks_rd, bf16x8 *fa_n, bf16x8 *fb_n,
                             auto n_load_c, int kt_issue, char *__restrict__ wr) {
        constexpr int N_LOAD = decltype(n_load_c)::value;
        constexpr int N_READ = MB + NB, OPS = N_READ + N_LOAD, SLOTS = MB * NB;
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                mfma32(fb[j], fa[i], acc[j][i]);
                const int idx = j * MB + i;
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int o = 0; o < OPS; ++o) {
                    if (o * SLOTS / OPS != idx) continue;
                    if (o >= N_READ) {
                        issue_one(ks * N_LOAD + o - N_READ, kt_issue, wr);
                    } else if (do_read) {
                        // order of first use by the next step: fb[0], fa[0..], fb[1..]
                        if (o == 0)
                            fb_n[0] = *reinterpret_cast<const bf16x8 *>(st + b_base + rd_off[ks_rd]);
                        else if (o <= MB)
                            fa_n[o - 1] = *reinterpret_cast<const bf16x8 *>(st + a_base + (o - 1) * 32 * RB + rd_off[ks_rd]);
                        else
                            fb_n[o - MB] = *reinterpret_cast<const bf16x8 *>(st + b_base + (o - MB) * 32 * RB + rd_off[ks_rd]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
    };

    constexpr int LPT = G::LPT;

    // ---- the K loop of one output tile ---------------------------------------
    // LOADER: this wave issues tile loads.  With G::LW < WM*WN only the first
    // LW waves do; the others run the same code without them (two copies of
    // everything below, chosen once per wave, each free of branches around
    // the loads).  Expects K tiles 0 .. NS-2 of the tile to be in flight.
    auto main_loop = [&](auto loader_c) {
        constexpr bool LOADER = decltype(loader_c)::value;
        if constexpr (NS >= 3) {
            // Ring of NS stages, tile kt in stage (S0 + kt) % NS.  The workgroup
            // barrier sits before the LAST MFMA step of a tile, not after it:
            // once every wave has issued (and received) all operand reads of
            // tile kt, the stage of tile kt-1 can be refilled and the first
            // operands of tile kt+1 can be read, all while the matrix cores
            // still work on the last step of tile kt.  Operands are double
            // buffered in registers.  The loop body is branch-free (the last
            // NS-1 tiles are peeled off), which keeps the compiler's wait-count
            // tracking exact.  Needs KT >= NS-1.
            static_assert(KS % 2 == 0, "operand double buffering assumes an even number of K steps");
            bf16x8 fa[2][MB], fb[2][NB];
            // One tile.  cur / nxt / wr are three different stages (restrict):
            // the loads that refill wr never make the operand reads wait.  VM =
            // loads of younger tiles that may still be in flight when tile kt+1
            // is needed.
            auto k_tile = [&](const char *__restrict__ cur, const char *__restrict__ nxt,
                              char *__restrict__ wr, int kt_issue, auto vm_c, auto issue_c, auto last_c) {
                constexpr int VM = decltype(vm_c)::value;
                constexpr bool ISSUE = decltype(issue_c)::value, LAST = decltype(last_c)::value;
                typedef std::integral_constant<int, ISSUE && LOADER ? G::LPS : 0> n_load_t;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    if (ks + 1 < KS) {
                        // operands of this step: read during the previous step
                        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0) only
                        __builtin_amdgcn_sched_barrier(0);
                        mfma_step_mem(fa[ks & 1], fb[ks & 1], ks, true, cur, ks + 1, fa[(ks + 1) & 1],
                                      fb[(ks + 1) & 1], n_load_t{}, kt_issue, wr);
                    } else {
                        if constexpr (!LAST) wait_and_barrier<VM>();   // tile kt+1 landed; my reads of tile kt complete
                        else __builtin_amdgcn_s_waitcnt(0xC07F);
                        __builtin_amdgcn_sched_barrier(0);
                        mfma_step_mem(fa[ks & 1], fb[ks & 1], ks, !LAST, nxt, 0, fa[0], fb[0], n_load_t{}, kt_issue, wr);
                    }
                }
            };
            int s_cur = S0, s_nxt = (S0 + 1) % NS, s_wr = (S0 + NS - 1) % NS;
            auto rotate = [&]() {
                s_wr = s_cur;
                s_cur = s_nxt;
                s_nxt = s_nxt + 1 == NS ? 0 : s_nxt + 1;
            };
            typedef std::true_type yes_t;
            typedef std::false_type no_t;
            wait_and_barrier<(NS - 2) * LPT>();     // tile 0 landed
            read_frags(lds + S0 * STAGE, 0, fa[0], fb[0]);
            for (int kt = 0; kt < KT - (NS - 1); ++kt) {
                k_tile(lds + s_cur * STAGE, lds + s_nxt * STAGE, lds + s_wr * STAGE, kt + NS - 1,
                       std::integral_constant<int, (NS - 3) * LPT + (KS - 1) * G::LPS>{}, yes_t{}, no_t{});
                rotate();
            }
            // the last NS-1 tiles: nothing left to issue, fewer loads in flight
            auto tail = [&](auto t_c) {
                constexpr int t = decltype(t_c)::value;
                if constexpr (t < NS - 1) {
                    constexpr int younger = NS - 3 - t > 0 ? NS - 3 - t : 0;
                    k_tile(lds + s_cur * STAGE, lds + s_nxt * STAGE, lds + s_wr * STAGE, 0,
                           std::integral_constant<int, younger * LPT>{}, no_t{},
                           std::integral_constant<bool, t == NS - 2>{});
                    rotate();
                }
            };
            tail(std::integral_constant<int, 0>{});
            tail(std::integral_constant<int, 1>{});
            tail(std::integral_constant<int, 2>{});
            tail(std::integral_constant<int, 3>{});
            static_assert(NS <= 5, "tail unrolling covers NS - 1 <= 4 tiles");
        } else {
            static_assert(G::LW == G::WM * WN && !G::PERSIST, "the two-stage path loads with every wave");
            // Two stages: refill the stage that was computed last with the next
            // tile, then run the MFMAs of this one.  `rd` and `wr` never overlap
            // (restrict), so the operand reads are not made to wait on those loads.
            auto k_tile = [&](const char *__restrict__ rd, char *__restrict__ wr, int kt_issue, bool issue) {
                if (issue) issue_tile(kt_issue, wr);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    bf16x8 fa[MB], fb[NB];
                    read_frags(rd, ks, fa, fb);
                    mfma_step(fa, fb);
                }
            };
            int st_rd = 0, st_wr = NS - 1;      // ring positions: tile kt lives in stage kt % NS
            for (int kt = 0; kt < KT; ++kt) {
                // Tile kt has landed when the loads of the younger tiles are the
                // only ones outstanding.  The wait, the barrier and the compiler
                // fence are one asm block so that nothing else makes this wave wait
                // for the younger loads (a fence builtin would: those loads are LDS
                // writes too).  lgkmcnt(0): this wave's operand reads of the
                // previous tile are complete before any wave refills that stage.
                if (kt + NS - 2 < KT)
                    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((NS - 2) * LPT) : "memory");
                else
                    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
                k_tile(lds + st_rd * STAGE, lds + st_wr * STAGE, kt + NS - 1, kt + NS - 1 < KT);
                st_rd = st_rd + 1 == NS ? 0 : st_rd + 1;
                st_wr = st_wr + 1 == NS ? 0 : st_wr + 1;
            }
        }
    };

    // ---- the same K loop with 16x16x32 MFMA blocks ----------------------------
    // Measured on register operands with random data (the chip is power limited
    // there), v_mfma_f32_16x16x32_bf16 sustains 2130 TFLOP/s where
    // v_mfma_f32_32x32x16_bf16 sustains 1870: a quarter of the accumulator
    // registers move per instruction for half of the flops.  One MFMA covers
    // the whole 32-deep K tile, so the two phases of a tile are the two halves
    // of the wave's rows: phase 0 multiplies A blocks 0 .. MBH-1 with every B
    // block, phase 1 the other MBH.  The barrier sits before phase 1; during
    // phase 0 the A operands of phase 1 are read, during phase 1 the B
    // operands and the first A operands of the next tile (B is double
    // buffered in registers; tiles come in pairs so that the buffer index is a
    // compile-time constant: K % 64 == 0 makes the number of tiles even).
    auto main_loop16 = [&](auto loader_c) {
        constexpr bool LOADER = decltype(loader_c)::value;
        constexpr int NB16 = TN / 16, MBH = TM / 32;          // B blocks; A blocks per phase
        constexpr int SLOTS = NB16 * MBH;                      // MFMAs per phase
        constexpr int L0 = LPT - LPT / 2, L1 = LPT / 2;        // tile loads issued in phase 0 / phase 1
        // PAIR (GEMM1): the A rows are 64-byte pieces of gathered rows of x, the
        // two halves of a 128-byte line belong to consecutive K tiles.  Fetched a
        // whole tile time apart, the line travels from L2 twice (40 B/clk/CU in a
        // microbenchmark of the load path); fetched by consecutive loads, once
        // (55 B/clk/CU).  So the loads of a pair of tiles (T, T+1), T even, go
        // out in this order: during the tile that refills T's stage the CB loads
        // of B(T), during the next one A(T)[0], A(T+1)[0], A(T)[1], A(T+1)[1], ...
        // and then B(T+1).  (A(T) leaves one tile time later than otherwise.)
        constexpr bool PAIR = SWIGLU && G::PAIR;
        constexpr int PL0 = CB - CB / 2, PL1 = CB / 2;                       // even tile: B only
        constexpr int QL0 = (2 * CA + CB) - (2 * CA + CB) / 2, QL1 = (2 * CA + CB) / 2;   // odd tile
        // (at most one memory operation per MFMA in the default geometry; smaller
        // wave tiles put two after some of them)
        static_assert(MBH + L0 <= 2 * SLOTS && NB16 + MBH + L1 <= 2 * SLOTS, "memory operations per MFMA");
        static_assert(!PAIR || (MBH + QL0 <= 2 * SLOTS && NB16 + MBH + QL1 <= 2 * SLOTS), "memory operations per MFMA");
        bf16x8 fa[2][MBH], fb[2][NB16];
        auto read_a = [&](const char *__restrict__ st, int blk) {
            return *reinterpret_cast<const bf16x8 *>(st + a_base + blk * 16 * RB + rd16);
        };
        auto read_b = [&](const char *__restrict__ st, int blk) {
            return *reinterpret_cast<const bf16x8 *>(st + b_base + blk * 16 * RB + rd16);
        };
        // one phase: SLOTS MFMAs, after each at most one read or tile load
        // load n of the loads a tile of parity P issues (for tile kt_issue into
        // stage wr; PAIR, odd tile: also for tile kt_issue - 1 into stage wr_prev)
        auto issue_op = [&](auto par_c, int n, int kt_issue, char *__restrict__ wr, char *__restrict__ wr_prev) {
            constexpr int P = decltype(par_c)::value;
            if constexpr (!PAIR) {
                issue_one(n, kt_issue, wr);
            } else if constexpr (P == 0) {
                issue_one(CA + n, kt_issue, wr);
            } else {
                if (n >= 2 * CA) issue_one(n - CA, kt_issue, wr);
                else if (n % 2 == 0) issue_one(n / 2, kt_issue - 1, wr_prev);
                else issue_one(n / 2, kt_issue, wr);
            }
        };
        auto phase = [&](auto ph_c, auto par_c, auto read_c, auto n_load_c, auto load_base_c,
                         const char *__restrict__ st, int kt_issue, char *__restrict__ wr,
                         char *__restrict__ wr_prev) {
            constexpr int PH = decltype(ph_c)::value, P = decltype(par_c)::value;
            constexpr bool READ = decltype(read_c)::value;
            constexpr int N_LOAD = decltype(n_load_c)::value, LOAD_BASE = decltype(load_base_c)::value;
            constexpr int N_READ = PH == 0 ? MBH : NB16 + MBH;
            constexpr int OPS = N_READ + N_LOAD;
#pragma unroll
            for (int j = 0; j < NB16; ++j)
#pragma unroll
                for (int i = 0; i < MBH; ++i) {
                    mfma16(fb[P][j], fa[PH][i], acc[j][PH * MBH + i]);
                    const int idx = j * MBH + i;
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int o = 0; o < OPS; ++o) {
                        if (o * SLOTS / OPS != idx) continue;
                        if (o >= N_READ) {
                            issue_op(par_c, LOAD_BASE + o - N_READ, kt_issue, wr, wr_prev);
                        } else if (READ) {
                            if (PH == 0) fa[1][o] = read_a(st, MBH + o);          // this tile, phase 1
                            else if (o < NB16) fb[1 - P][o] = read_b(st, o);       // next tile
                            else fa[0][o - NB16] = read_a(st, o - NB16);           // next tile, phase 0
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
        };
        typedef std::true_type yes_t;
        typedef std::false_type no_t;
        // One tile.  cur / nxt / wr are three different stages (restrict).
        auto k_tile = [&](auto par_c, const char *__restrict__ cur, const char *__restrict__ nxt,
                          char *__restrict__ wr, char *__restrict__ wr_prev, int kt_issue, auto vm_c,
                          auto issue_c, auto last_c) {
            constexpr int VM = decltype(vm_c)::value, P = decltype(par_c)::value;
            constexpr bool ISSUE = decltype(issue_c)::value, LAST = decltype(last_c)::value;
            constexpr int N0 = !(ISSUE && LOADER) ? 0 : !PAIR ? L0 : P == 0 ? PL0 : QL0;
            constexpr int N1 = !(ISSUE && LOADER) ? 0 : !PAIR ? L1 : P == 0 ? PL1 : QL1;
            typedef std::integral_constant<int, N0> l0_t;
            typedef std::integral_constant<int, N1> l1_t;
            typedef std::integral_constant<int, 0> base0_t;
            __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): operands read during the previous phase
            __builtin_amdgcn_sched_barrier(0);
            phase(std::integral_constant<int, 0>{}, par_c, yes_t{}, l0_t{}, base0_t{}, cur, kt_issue, wr, wr_prev);
            if constexpr (!LAST) wait_and_barrier<VM>();   // tile kt+1 landed; my reads of tile kt complete
            else __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_sched_barrier(0);
            phase(std::integral_constant<int, 1>{}, par_c, std::integral_constant<bool, !LAST>{}, l1_t{}, l0_t{},
                  nxt, kt_issue, wr, wr_prev);
        };
        // s_wr: the stage the tile being computed refills (tile kt + NS - 1);
        // s_prev: the stage the tile before it refilled
        int s_cur = S0, s_nxt = (S0 + 1) % NS, s_wr = (S0 + NS - 1) % NS, s_prev = (S0 + NS - 2) % NS;
        auto rotate = [&]() {
            s_prev = s_wr;
            s_wr = s_cur;
            s_cur = s_nxt;
            s_nxt = s_nxt + 1 == NS ? 0 : s_nxt + 1;
        };
        wait_and_barrier<(NS - 2) * LPT>();     // tile 0 landed
#pragma unroll
        for (int j = 0; j < NB16; ++j) fb[0][j] = read_b(lds + S0 * STAGE, j);
#pragma unroll
        for (int i = 0; i < MBH; ++i) fa[0][i] = read_a(lds + S0 * STAGE, i);
        // Loads that may still be in flight at a tile's barrier, when the next
        // tile must have landed (loads complete in the order of issue).  In
        // tile order: the tiles after the next one, and this tile's phase 0.
        // PAIR, at even tile T (tile T+1 went out last during tile T-3): the loads
        // of tiles T-2 and T-1 and of this phase 0; at odd tile T+1 (the last load
        // of tile T+2 is A(T+2)[CA-1], issued during T-1 and followed there by
        // A(T+3)[CA-1] and B(T+3)): those 1 + CB, tile T's and this phase 0.  The
        // first tiles of an output tile were issued in tile order, which leaves
        // at least as many younger loads at each of these points.
        constexpr int VM0 = !PAIR ? (NS - 3) * LPT + L0 : CB + (2 * CA + CB) + PL0;
        constexpr int VM1 = !PAIR ? (NS - 3) * LPT + L0 : (1 + CB) + CB + QL0;
        static_assert(NS == 5 && VM0 < 64 && VM1 < 64, "ring of five stages; vmcnt has six bits");
        typedef std::integral_constant<int, 0> par0_t;
        typedef std::integral_constant<int, 1> par1_t;
        // KT is even and NS - 1 = 4 tiles are peeled: the steady tiles come in pairs
        for (int kt = 0; kt < KT - (NS - 1); kt += 2) {
            k_tile(par0_t{}, lds + s_cur * STAGE, lds + s_nxt * STAGE, lds + s_wr * STAGE, lds + s_prev * STAGE,
                   kt + NS - 1, std::integral_constant<int, VM0>{}, yes_t{}, no_t{});
            rotate();
            k_tile(par1_t{}, lds + s_cur * STAGE, lds + s_nxt * STAGE, lds + s_wr * STAGE, lds + s_prev * STAGE,
                   kt + NS, std::integral_constant<int, VM1>{}, yes_t{}, no_t{});
            rotate();
        }
        // the last NS-1 tiles: nothing left to issue, fewer loads in flight
        // (PAIR: tiles KT-2 and KT-1 went out as A, A, ..., B during tile KT-5)
        auto tail = [&](auto t_c) {
            constexpr int t = decltype(t_c)::value;
            constexpr int younger = NS - 3 - t > 0 ? NS - 3 - t : 0;
            constexpr int VMT = !PAIR ? younger * LPT : t == 0 ? CB + (2 * CA + CB) : t == 1 ? 1 + CB : 0;
            k_tile(std::integral_constant<int, t % 2>{}, lds + s_cur * STAGE, lds + s_nxt * STAGE,
                   lds + s_wr * STAGE, lds + s_prev * STAGE, 0, std::integral_constant<int, VMT>{}, no_t{},
                   std::integral_constant<bool, t == NS - 2>{});
            rotate();
        };
        tail(std::integral_constant<int, 0>{});
        tail(std::integral_constant<int, 1>{});
        tail(std::integral_constant<int, 2>{});
        tail(std::integral_constant<int, 3>{});
    };

    // ---- epilogue: registers -> LDS patch -> 16-byte stores --------------------
    // acc[j][i][v]: output row m = wm*TM + i*32 + l32,
    //               B row n = wn*TN + j*32 + 8*(v/4) + 4*lh + v%4
    // The weight fragment is the first MFMA operand, so a lane holds four
    // consecutive output columns of one row (8-byte LDS writes).
    // `early` tiles of the NEXT output tile (pointers already set) are issued
    // first; they land in stages the patch does not touch (the two restrict
    // pointers tell the compiler so: it would otherwise wait for those loads
    // before every LDS access below).
    auto epilogue = [&](char *__restrict__ patch, char *__restrict__ ring, auto early_c) {
        constexpr int N_EARLY = decltype(early_c)::value;
        issue_range(0, N_EARLY, ring);
        typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
        const int n0 = nt * BN;
        const int c_col0 = SWIGLU ? n0 / 2 : n0;
        constexpr int OCPR = OUT_W / 8;                // 16-byte chunks per output row
#pragma unroll
        for (int ep = 0; ep < EP; ++ep) {
            if (ep > 0) lds_sync();                    // the previous pass has left the patch
            if ((wm * TM) / HB == ep) {
                if constexpr (MI == 16) {
                    // 16x16 blocks: acc[j][i][v] is output row wm*TM + i*16 + l16,
                    // B row wn*TN + j*16 + 4*lq + v; B rows come in blocks of 32
                    // rows of W1 then 32 rows of W3 (GEMM1), so 16-row block j
                    // pairs with block j + 2
#pragma unroll
                    for (int i = 0; i < MBX; ++i) {
                        const int m = wm * TM + i * 16 + l16 - ep * HB;
                        char *orow = patch + m * OUT_STRIDE;
                        if constexpr (SWIGLU) {
#pragma unroll
                            for (int jp = 0; jp < NBX / 2; ++jp) {
                                const int jg = (jp / 2) * 4 + jp % 2;             // silu's argument
                                const int c0 = (wn * TN) / 2 + (jp / 2) * 32 + (jp % 2) * 16 + 4 * lq;
                                bf16x4 o;
#pragma unroll
                                for (int q = 0; q < 4; ++q)
                                    o[q] = (bf16_t)(fast_silu(acc[jg][i][q]) * acc[jg + 2][i][q]);
                                *reinterpret_cast<bf16x4 *>(orow + c0 * 2) = o;
                            }
                        } else {
#pragma unroll
                            for (int j = 0; j < NBX; ++j) {
                                const int c0 = wn * TN + j * 16 + 4 * lq;
                                bf16x4 o;
#pragma unroll
                                for (int q = 0; q < 4; ++q) o[q] = (bf16_t)acc[j][i][q];
                                *reinterpret_cast<bf16x4 *>(orow + c0 * 2) = o;
                            }
                        }
                    }
                } else {
#pragma unroll
                for (int i = 0; i < MB; ++i) {
                    const int m = wm * TM + i * 32 + l32 - ep * HB;
                    char *orow = patch + m * OUT_STRIDE;
                    if constexpr (SWIGLU) {
#pragma unroll
                        for (int j = 0; j < NB; j += 2) {
                            const int c0 = (wn * TN + j * 32) / 2 + 4 * lh;   // 32 columns per block pair
#pragma unroll
                            for (int g = 0; g < 4; ++g) {
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
                                bf16x4 o;
#pragma unroll
                                for (int q = 0; q < 4; ++q) o[q] = (bf16_t)acc[j][i][4 * g + q];
                                *reinterpret_cast<bf16x4 *>(orow + (c0 + 8 * g) * 2) = o;
                            }
                        }
                    }
                }
                }
            }
            lds_sync();
            if constexpr (SWIGLU) {
                // h is K-slab-major: the patch is OUT_W/32 slabs of HB rows x 64
                // bytes, each consecutive in memory; consecutive threads take
                // consecutive 16-byte pieces of a slab.
                for (int c = tid; c < HB * OCPR; c += NT) {
                    const int sl = c / (HB * 4), m = (c / 4) % HB, q = c % 4;
                    const int row = row0 + ep * HB + m, col = c_col0 + sl * kSlab + q * 8;
                    if (row < row_end && col < a.Nc)
                        *reinterpret_cast<bf16x8 *>(a.C + (size_t)(col / kSlab) * a.h_rows * kSlab +
                                                    (size_t)row * kSlab + q * 8) =
                            *reinterpret_cast<const bf16x8 *>(patch + m * OUT_STRIDE + (sl * 4 + q) * 16);
                }
            } else {
                for (int c = tid; c < HB * OCPR; c += NT) {
                    const int m = c / OCPR, cc = c % OCPR;
                    const int row = row0 + ep * HB + m, col = c_col0 + cc * 8;
                    if (row < row_end && col < a.Nc)
                        *reinterpret_cast<bf16x8 *>(a.C + (size_t)row * a.ld + col) =
                            *reinterpret_cast<const bf16x8 *>(patch + m * OUT_STRIDE + cc * 16);
                }
            }
        }
    };

    // ---- tile after tile -----------------------------------------------------
    auto run = [&](auto loader_c) {
        constexpr bool LOADER = decltype(loader_c)::value;
        int j = blockIdx.x / NXCD;
        if (!locate(j, e, row0, row_end, nt)) return;
        int src[CA];
        if constexpr (LOADER) {
            gather_rows(row0, row_end, src);
            set_pointers(e, nt, src);
            issue_range(0, NS - 1, lds);
        }
        // the loading waves win instruction arbitration over the others (+1 %, measured)
        if constexpr (G::LW != G::WM * WN) __builtin_amdgcn_s_setprio(LOADER ? 2 : 0);
        for (;;) {
            // The next tile of this workgroup; the rows of x it gathers are
            // fetched now, a whole K loop before they are needed.  When
            // there is no next tile everything below is done once more for
            // the tile just finished (and never used): no branch around a
            // load, so the compiler adds no wait for one.
            int n_e = e, n_row0 = row0, n_row_end = row_end, n_nt = nt;
            bool more = false;
            if constexpr (G::PERSIST) {
                j += a.jstride;
                more = locate(j, n_e, n_row0, n_row_end, n_nt);
                if constexpr (LOADER) gather_rows(n_row0, n_row_end, src);
            }
#pragma unroll
            for (int jj = 0; jj < NBX; ++jj)
#pragma unroll
                for (int i = 0; i < MBX; ++i)
#pragma unroll
                    for (int v = 0; v < (int)(sizeof(acc_t) / sizeof(float)); ++v) acc[jj][i][v] = 0.f;
            if constexpr (MI == 16) main_loop16(loader_c);
            else main_loop(loader_c);
            __syncthreads();                    // all waves done reading the stages
            if constexpr (!G::PERSIST) {
                epilogue(lds, lds, std::integral_constant<int, 0>{});
                return;
            } else {
                // The first K tiles of the next output tile go out before the
                // epilogue, into the stages the epilogue does not use, the
                // others after it.
                if constexpr (LOADER) set_pointers(n_e, n_nt, src);
                epilogue(lds, lds, std::integral_constant<int, LOADER ? EARLY : 0>{});
                if (!more) break;
                lds_sync();                     // the epilogue has left its LDS patch
                if constexpr (LOADER) issue_range(EARLY, NS - 1, lds);
                e = n_e; row0 = n_row0; row_end = n_row_end; nt = n_nt;
            }
        }
        // loads into LDS must not outlive the workgroup
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };
    if constexpr (G::LW == G::WM * WN) {
        run(std::true_type{});
    } else {
        if (__builtin_amdgcn_readfirstlane(wave) < G::LW) run(std::true_type{});
        else run(std::false_type{});
    }
}

bool ffn_mfma_supported(const Dims &d) { return d.D % 64 == 0 && d.F % 64 == 0; }

// TAILG: geometry (half the tile height of G) of a second launch that takes
// over a sparsely filled last round of G's tiles; void: none.
template <class G, class TAILG = void>
static hipError_t launch_cfg(const FfnArgs &f, int which, hipStream_t s) {
    GemmArgs a;
    a.offsets = f.offsets;
    a.src_of = f.src_of;
    a.n_ffn = f.d.n_ffn;
    a.topk = f.d.k;
    a.h_rows = f.h_rows;
    if (which == 0) {
        a.A = (const bf16_t *)f.x;
        a.ld = f.d.D;
        a.B = (const bf16_t *)f.w13;
        a.K = f.d.D;
        a.Nb = 2 * f.d.F;
        a.C = (bf16_t *)f.h;
        a.Nc = f.d.F;
    } else {
        a.A = (const bf16_t *)f.h;
        a.B = (const bf16_t *)f.w2;
        a.K = f.d.F;
        a.Nb = f.d.D;
        a.C = (bf16_t *)f.yffn;
        a.ld = f.d.D;
        a.Nc = f.d.D;
    }
    constexpr int BM = G::BM, BN = G::BN;
    a.n_ntiles = (a.Nb + BN - 1) / BN;
    const long long rows = (long long)f.d.T * f.d.k;
    const long long max_mtiles = (rows + BM - 1) / BM + f.d.n_ffn;   // upper bound of sum ceil(count_e/BM)
    const long long rnd = 8 * 8 * 4;   // whole rounds of one patch (GM x GN tiles) per XCD
    long long blocks = (max_mtiles * a.n_ntiles + rnd - 1) / rnd * rnd;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    if (a.K / G::BK < G::NS - 1) return hipErrorInvalidConfiguration;   // the ring starts with NS-1 K tiles in flight
    a.jstride = 0;
    if (G::PERSIST) {
        // one workgroup per CU (the LDS ring fills a CU), a multiple of 8 so that
        // workgroup w runs on XCD w % 8 and owns tiles w/8, w/8 + jstride, ...
        static int n_cu = 0;
        if (n_cu == 0) {
            int dev = 0, v = 0;
            if (hipGetDevice(&dev) != hipSuccess ||
                hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 8)
                v = 256;
            n_cu = v / 8 * 8;
        }
        if (blocks > n_cu) blocks = n_cu;
        a.jstride = (int)(blocks / 8);
    }
    dim3 grid((unsigned)blocks), block(G::NT);
    a.cut_grid = 0;
    bool tail = false;
    if constexpr (!std::is_void<TAILG>::value) {
        static_assert(G::PERSIST && TAILG::PERSIST && 2 * TAILG::BM == G::BM && TAILG::BN == G::BN &&
                          TAILG::BK == G::BK && TAILG::NS == G::NS,
                      "the tail launch halves the tiles of the main launch");
        // With few rounds a sparsely filled last one is worth a second launch
        // (measured: +6 to +12 % at 3 - 5 rounds, +2 % at 13); with many it
        // costs little, the few busy CUs also clock higher (nothing at 36).
        // The host knows an upper bound of the number of rounds only.
        tail = max_mtiles * a.n_ntiles < 24 * blocks;
        if (tail) a.cut_grid = (int)blocks;
    }
    if (which == 0)
        hipLaunchKernelGGL((k_grouped_gemm<G, true>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((k_grouped_gemm<G, false>), grid, block, 0, s, a);
    if constexpr (!std::is_void<TAILG>::value) if (tail) {
        // same grid and numbering; a workgroup finds at most one half tile, none
        // when the main launch kept its last round
        if (which == 0)
            hipLaunchKernelGGL((k_grouped_gemm<TAILG, true, true>), grid, dim3(TAILG::NT), 0, s, a);
        else
            hipLaunchKernelGGL((k_grouped_gemm<TAILG, false, true>), grid, dim3(TAILG::NT), 0, s, a);
    }
    return hipGetLastError();
}

hipError_t launch_ffn_mfma(const FfnArgs &f, int which, hipStream_t s) {
    if (f.d.T == 0 || f.d.n_ffn == 0) return hipSuccess;
    // Default: 256x256 tile, 8 waves of which the first 4 issue the tile loads,
    // 16x16x32 MFMA blocks, persistent workgroups, 32-deep K stages in a ring
    // of 5 (the whole 160 KB of LDS), which needs at least 4 K tiles; shorter
    // reductions use two 64-deep stages.
    const int K = which == 0 ? f.d.D : f.d.F;
    if (K / 32 < 4)                       // too few K tiles to fill a ring of stages
        return launch_cfg<Geo<256, 256, 2, 4, 64, 2>>(f, which, s);
    // Few rows per expert (decoding, small batches): the GEMMs only stream
    // the weights, so use 128-row tiles: half of the (mostly wasted)
    // matrix work of a 256-row tile per byte of weights, bound by HBM instead.
    if ((long long)f.d.T * f.d.k <= 128ll * f.d.n_ffn)
        return launch_cfg<Geo<128, 256, 1, 4, 32, 5, 0, true>>(f, which, s);
    if (f.no_tail) return launch_cfg<Geo<256, 256, 2, 4, 32, 5, 4, true, 16>>(f, which, s);
    return launch_cfg<Geo<256, 256, 2, 4, 32, 5, 4, true, 16>, Geo<128, 256, 2, 4, 32, 5, 4, true, 16>>(
        f, which, s);
}

}  // namespace moepp
