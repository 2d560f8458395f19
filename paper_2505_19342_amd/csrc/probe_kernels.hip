// Measurement probe: a matrix-core-only loop, the on-box reference the benchmark quotes next to the published
// MFMA peak.  No memory traffic inside the loop, four independent accumulators per wavefront, two wavefronts per
// SIMD, operands with ordinary (non-constant) bit patterns: the chip lowers its clock under matrix load depending
// on how much the operands toggle, so an all-zero probe would overstate what a real kernel can reach.
#include "common.h"

namespace astra {

constexpr int kProbeThreads = 512;

__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(float* __restrict__ out, int iters) {
    const int tid = threadIdx.x;
    bf16x8 a[2], b[2];
    uint32_t hsh = (uint32_t)(blockIdx.x * kProbeThreads + tid) * 2654435761u + 12345u;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            hsh = hsh * 1664525u + 1013904223u;
            a[j][e] = (__bf16)(((int)(hsh >> 20) - 2048) * (1.f / 4096.f));          // values in (-0.5, 0.5)
            hsh = hsh * 1664525u + 1013904223u;
            b[j][e] = (__bf16)(((int)(hsh >> 20) - 2048) * (1.f / 4096.f));
        }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = mfma_32x32x16(a[j & 1], b[j >> 1], acc[j]);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[j][v];
    out[(int64_t)blockIdx.x * kProbeThreads + tid] = s;
}

// out: n_blocks * 512 floats.  Work: n_blocks * 8 wavefronts * iters * 4 MFMAs * 32768 flop.
int launch_mfma_probe(float* out, int n_blocks, int iters, hipStream_t s) {
    if (n_blocks <= 0 || iters <= 0) return ASTRA_ERR_SHAPE;
    mfma_probe_kernel<<<n_blocks, kProbeThreads, 0, s>>>(out, iters);
    return launch_status();
}

}  // namespace astra
