// Measurement aid: the sustained bf16 MFMA rate of this GPU with no memory
// traffic at all.  MI355X lowers its clock under matrix load, by an amount
// that depends on the operand bits (all-zero operands run at the full clock,
// random operands do not), so the published peak is not reachable by any
// kernel that multiplies real data; this gives the ceiling that is.  It runs
// the instruction the grouped GEMM uses, v_mfma_f32_16x16x32_bf16, which under
// that limit sustains more than v_mfma_f32_32x32x16_bf16 (measured: about
// 2130 against 1870 TFLOP/s with the same operands): a quarter of the
// accumulator registers move per instruction for half of the flops.
#include "common.h"

namespace moepp {

__global__ __launch_bounds__(512, 1) void k_mfma_ceiling(float *out, int iters) {
    // pseudo-random operands in [-1, 1), different in every lane
    unsigned rs = 12345u + (blockIdx.x * 512u + threadIdx.x) * 2654435761u;
    bf16x8 fa[4], fb[2];
    for (int i = 0; i < 4; ++i)
        for (int q = 0; q < 8; ++q) {
            rs = rs * 1664525u + 1013904223u;
            fa[i][q] = (bf16_t)(((rs >> 8) & 0xffff) / 32768.0f - 1.0f);
        }
    for (int i = 0; i < 2; ++i)
        for (int q = 0; q < 8; ++q) {
            rs = rs * 1664525u + 1013904223u;
            fb[i][q] = (bf16_t)(0.02f * (((rs >> 8) & 0xffff) / 32768.0f - 1.0f));
        }
    // 32 independent 16x16 accumulators (128 registers, as in the GEMM kernel)
    f32x4 acc[32];
    for (int i = 0; i < 32; ++i)
        for (int v = 0; v < 4; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int i = 0; i < 32; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[i & 1], fa[i & 3], acc[i], 0, 0, 0);
    float s = 0.f;
    for (int i = 0; i < 32; ++i)
        for (int v = 0; v < 4; ++v) s += acc[i][v];
    out[blockIdx.x * 512 + threadIdx.x] = s;
}

constexpr int kCeilBlocks = 256;   // of 8 waves: 2 waves on each of the 1024 SIMDs

hipError_t launch_mfma_ceiling(float *scratch, int iters, hipStream_t s) {
    hipLaunchKernelGGL(k_mfma_ceiling, dim3(kCeilBlocks), dim3(512), 0, s, scratch, iters);
    return hipGetLastError();
}

double mfma_ceiling_flops(int iters) {
    return (double)kCeilBlocks * 8 * iters * 32 * (2.0 * 16 * 16 * 32);
}
size_t mfma_ceiling_scratch_bytes() { return (size_t)kCeilBlocks * 512 * sizeof(float); }

// ---- what a kernel that only moves data reaches ------------------------------
// mode 0: read `bytes` (each wave whole 1 KB pieces, four in flight per lane);
// mode 1: copy the first half of the buffer over the second.  The published
// 8 TB/s is a pin rate; this is what the memory system delivers to a kernel.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_stream(u32x4_t *buf, size_t n_vec, int mode) {
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    if (mode == 0) {
        for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i + 768 < n_vec; i += stride) {
            const u32x4_t a = __builtin_nontemporal_load(buf + i), b = __builtin_nontemporal_load(buf + i + 256);
            const u32x4_t c = __builtin_nontemporal_load(buf + i + 512), d = __builtin_nontemporal_load(buf + i + 768);
            acc ^= a ^ b ^ c ^ d;
        }
        // never true for the buffers this is run on; keeps the loads alive
        if (acc.x == 0x9e3779b9u && acc.y == 0x7f4a7c15u && acc.z == 0x6a09e667u && acc.w == 0xbb67ae85u)
            buf[threadIdx.x] = acc;
    } else {
        const size_t half = n_vec / 2;
        for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i + 768 < half; i += stride) {
            const u32x4_t a = __builtin_nontemporal_load(buf + i), b = __builtin_nontemporal_load(buf + i + 256);
            const u32x4_t c = __builtin_nontemporal_load(buf + i + 512), d = __builtin_nontemporal_load(buf + i + 768);
            __builtin_nontemporal_store(a, buf + half + i);
            __builtin_nontemporal_store(b, buf + half + i + 256);
            __builtin_nontemporal_store(c, buf + half + i + 512);
            __builtin_nontemporal_store(d, buf + half + i + 768);
        }
    }
}

hipError_t launch_stream(void *buf, size_t bytes, int mode, hipStream_t s) {
    hipLaunchKernelGGL(k_stream, dim3(256 * 16), dim3(256), 0, s, (u32x4_t *)buf, bytes / 16, mode);
    return hipGetLastError();
}

}  // namespace moepp
