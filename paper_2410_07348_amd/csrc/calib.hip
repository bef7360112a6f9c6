// Measurement aid: the sustained bf16 MFMA rate of this GPU with no memory
// traffic at all.  MI355X lowers its clock under matrix load, by an amount
// that depends on the operand bits (all-zero operands run at the full clock,
// random operands do not), so the published peak is not reachable by any
// kernel that multiplies real data; this gives the ceiling that is.
#include "common.h"

namespace moepp {

__global__ __launch_bounds__(256) void k_mfma_ceiling(float *out, int iters) {
    // pseudo-random operands in [-1, 1), different in every lane
    unsigned rs = 12345u + (blockIdx.x * 256u + threadIdx.x) * 2654435761u;
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
    f32x16 acc[2][4];
    for (int j = 0; j < 2; ++j)
        for (int i = 0; i < 4; ++i)
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[j][i], 0, 0, 0);
    float s = 0.f;
    for (int j = 0; j < 2; ++j)
        for (int i = 0; i < 4; ++i)
            for (int v = 0; v < 16; ++v) s += acc[j][i][v];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

constexpr int kCeilBlocks = 512;   // 2 waves on each of the 1024 SIMDs

hipError_t launch_mfma_ceiling(float *scratch, int iters, hipStream_t s) {
    hipLaunchKernelGGL(k_mfma_ceiling, dim3(kCeilBlocks), dim3(256), 0, s, scratch, iters);
    return hipGetLastError();
}

double mfma_ceiling_flops(int iters) {
    return (double)kCeilBlocks * 4 * iters * 8 * (2.0 * 32 * 32 * 16);
}
size_t mfma_ceiling_scratch_bytes() { return (size_t)kCeilBlocks * 256 * sizeof(float); }

}  // namespace moepp
