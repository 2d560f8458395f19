// The parts of a Transformer block around the attention layer that are not matrix products (paper Sec. 3.1: each
// block normalises, attends with the mixed-precision layer, and runs its position-wise MLP locally): the row-wise
// normalisation of the fp32 residual stream into the layer's element type, and the gating of the fp32 MLP.
// Both are bound by HBM traffic: one read of the row, one write of the result.
#include "common.h"

namespace astra {

constexpr int kNormThreads = 256;
constexpr int kNormCache = 8;        // float4 values a thread keeps in registers: rows up to 256 * 8 * 4 = 8192 wide are read once

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
// sum over the workgroup; every thread gets the result.  `slot` alternates between calls so that a second reduction
// may start before every wavefront has read the first one's partial sums.
__device__ __forceinline__ float block_sum(float v, float (*part)[kNormThreads / kWave], int slot) {
    v = wave_sum(v);
    if (lane_id() == 0) part[slot][threadIdx.x / kWave] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kNormThreads / kWave; ++w) t += part[slot][w];
    return t;
}

template <typename OutT>
__device__ __forceinline__ void store_elem(OutT* o, float v);
template <>
__device__ __forceinline__ void store_elem<float>(float* o, float v) { *o = v; }
template <>
__device__ __forceinline__ void store_elem<uint16_t>(uint16_t* o, float v) { *o = f32_to_bf16_bits(v); }

// One workgroup per row.  kind 0: (x - mean) / sqrt(var + eps) * gain + bias, biased variance, computed as the mean of
// squared deviations (two passes over the registers, no cancellation); kind 1: x / sqrt(mean(x^2) + eps) * gain.
// VEC: D % 4 == 0 and D <= 8192, the row lives in registers; otherwise the row is re-read (from cache) per pass.
template <typename OutT, bool VEC>
__global__ __launch_bounds__(kNormThreads) void norm_kernel(const float* __restrict__ x, int D, int kind, float eps,
                                                            const float* __restrict__ gain, const float* __restrict__ bias,
                                                            OutT* __restrict__ out) {
    __shared__ float part[2][kNormThreads / kWave];
    const int tid = threadIdx.x;
    const float* __restrict__ row = x + (int64_t)blockIdx.x * D;
    OutT* __restrict__ orow = out + (int64_t)blockIdx.x * D;
    const float inv_d = 1.f / (float)D;
    if (VEC) {
        const int n4 = D >> 2;
        f32x4 c[kNormCache];
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < kNormCache; ++j) {
            const int i = tid + j * kNormThreads;
            c[j] = i < n4 ? reinterpret_cast<const f32x4*>(row)[i] : f32x4{0.f, 0.f, 0.f, 0.f};
            s += (c[j].x + c[j].y) + (c[j].z + c[j].w);
        }
        const float mean = kind == 0 ? block_sum(s, part, 0) * inv_d : 0.f;
        float q = 0.f;
#pragma unroll
        for (int j = 0; j < kNormCache; ++j) {
            const int i = tid + j * kNormThreads;
            if (i < n4) {
                const f32x4 d = c[j] - mean;
                q += (d.x * d.x + d.y * d.y) + (d.z * d.z + d.w * d.w);
            }
        }
        const float inv = 1.f / sqrtf(block_sum(q, part, 1) * inv_d + eps);
#pragma unroll
        for (int j = 0; j < kNormCache; ++j) {
            const int i = tid + j * kNormThreads;
            if (i < n4) {
                f32x4 v = (c[j] - mean) * inv;
                if (gain) v *= reinterpret_cast<const f32x4*>(gain)[i];
                if (kind == 0 && bias) v += reinterpret_cast<const f32x4*>(bias)[i];
                if constexpr (sizeof(OutT) == 2) {
                    u32x2 w;
                    w.x = pack_bf16x2(v.x, v.y);
                    w.y = pack_bf16x2(v.z, v.w);
                    reinterpret_cast<u32x2*>(orow)[i] = w;
                } else {
                    reinterpret_cast<f32x4*>(orow)[i] = v;
                }
            }
        }
    } else {
        float s = 0.f;
        for (int i = tid; i < D; i += kNormThreads) s += row[i];
        const float mean = kind == 0 ? block_sum(s, part, 0) * inv_d : 0.f;
        float q = 0.f;
        for (int i = tid; i < D; i += kNormThreads) {
            const float d = row[i] - mean;
            q += d * d;
        }
        const float inv = 1.f / sqrtf(block_sum(q, part, 1) * inv_d + eps);
        for (int i = tid; i < D; i += kNormThreads) {
            float v = (row[i] - mean) * inv;
            if (gain) v *= gain[i];
            if (kind == 0 && bias) v += bias[i];
            store_elem<OutT>(orow + i, v);
        }
    }
}

int launch_norm(int dtype, int kind, const float* x, int64_t T, int D, float eps, const float* gain, const float* bias, void* out,
                hipStream_t s) {
    if (T < 0 || D <= 0 || T > 0x7fffffff || (kind != 0 && kind != 1)) return ASTRA_ERR_SHAPE;
    if (T == 0) return ASTRA_OK;
    const bool vec = D % 4 == 0 && D <= kNormThreads * kNormCache * 4;
    if (dtype == ASTRA_BF16) {
        if (vec) norm_kernel<uint16_t, true><<<(int)T, kNormThreads, 0, s>>>(x, D, kind, eps, gain, bias, (uint16_t*)out);
        else norm_kernel<uint16_t, false><<<(int)T, kNormThreads, 0, s>>>(x, D, kind, eps, gain, bias, (uint16_t*)out);
    } else {
        if (vec) norm_kernel<float, true><<<(int)T, kNormThreads, 0, s>>>(x, D, kind, eps, gain, bias, (float*)out);
        else norm_kernel<float, false><<<(int)T, kNormThreads, 0, s>>>(x, D, kind, eps, gain, bias, (float*)out);
    }
    return launch_status();
}

// fp32 MLP gate: out[t, f] = silu(a[t, f]) * a[t, F + f]  (the bf16 path does this in the epilogue of its first GEMM)
__global__ __launch_bounds__(256) void swiglu_f32_kernel(const float* __restrict__ a, int64_t n, int F, float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t t = i / F;
    const int f = (int)(i - t * F);
    const float g = a[t * 2 * F + f], u = a[t * 2 * F + F + f];
    out[i] = g / (1.f + expf(-g)) * u;
}

int launch_swiglu_f32(const float* a, int64_t T, int F, float* out, hipStream_t s) {
    if (T < 0 || F <= 0) return ASTRA_ERR_SHAPE;
    const int64_t n = T * F;
    if (n == 0) return ASTRA_OK;
    const int64_t blocks = ceil_div(n, 256);
    if (blocks > 0x7fffffff) return ASTRA_ERR_SHAPE;
    swiglu_f32_kernel<<<(int)blocks, 256, 0, s>>>(a, n, F, out);
    return launch_status();
}

}  // namespace astra
