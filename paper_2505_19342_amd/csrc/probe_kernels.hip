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

// The same loop with NV vector-ALU instructions of the same wavefront after every MFMA (fused multiply-adds on eight
// independent registers, or EXP: a base-2 exponential and a multiply each): what a softmax or an address computation
// placed between MFMAs costs.  The program order is pinned so that the compiler cannot bunch them.
template <int NV, bool EXP>
__global__ __launch_bounds__(kProbeThreads) void mfma_valu_probe_kernel(float* __restrict__ out, int iters) {
    const int tid = threadIdx.x;
    bf16x8 a[2], b[2];
    uint32_t hsh = (uint32_t)(blockIdx.x * kProbeThreads + tid) * 2654435761u + 12345u;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            hsh = hsh * 1664525u + 1013904223u;
            a[j][e] = (__bf16)(((int)(hsh >> 20) - 2048) * (1.f / 4096.f));
            hsh = hsh * 1664525u + 1013904223u;
            b[j][e] = (__bf16)(((int)(hsh >> 20) - 2048) * (1.f / 4096.f));
        }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (float)(tid + i) * 1e-3f;
    const float m = 0.999f, c = 1e-4f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[j] = mfma_32x32x16(a[j & 1], b[j >> 1], acc[j]);
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (EXP) x[q % 8] = __builtin_amdgcn_exp2f(-x[q % 8]) * m;       // stays in (0, 1]: the sign is a free operand modifier
                else x[q % 8] = __builtin_fmaf(x[q % 8], m, c);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[j][v];
#pragma unroll
    for (int i = 0; i < 8; ++i) s += x[i];
    out[(int64_t)blockIdx.x * kProbeThreads + tid] = s;
}

int launch_mfma_valu_probe(float* out, int n_blocks, int iters, int valu_per_mfma, int use_exp, hipStream_t s) {
    if (n_blocks <= 0 || iters <= 0) return ASTRA_ERR_SHAPE;
#define ASTRA_PROBE_CASE(NV)                                                                              \
    case NV:                                                                                              \
        if (use_exp) mfma_valu_probe_kernel<NV, true><<<n_blocks, kProbeThreads, 0, s>>>(out, iters);     \
        else mfma_valu_probe_kernel<NV, false><<<n_blocks, kProbeThreads, 0, s>>>(out, iters);            \
        break;
    switch (valu_per_mfma) {
        ASTRA_PROBE_CASE(0)
        ASTRA_PROBE_CASE(2)
        ASTRA_PROBE_CASE(4)
        ASTRA_PROBE_CASE(8)
        ASTRA_PROBE_CASE(16)
        default: return ASTRA_ERR_UNSUPPORTED;
    }
#undef ASTRA_PROBE_CASE
    return launch_status();
}

}  // namespace astra
