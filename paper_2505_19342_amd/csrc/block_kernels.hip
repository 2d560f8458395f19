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

// ---- optional rotary position embedding (not part of the paper; Su et al., "RoFormer", Eq. 34, interleaved pairs), in
// place on a [rows, n_heads * head_dim] matrix of the element type with row stride ld: pair i of every head's vector at
// position m is turned by m * base^(-2i / head_dim).  Row r has position r + add_lo when r < split and r + add_hi
// otherwise; rows below `skip` have no position and are left alone.  The angle is formed in fp64 and reduced to a
// fraction of a turn before it is rounded (positions reach 10^5, the cosine of an fp32 product would be off by 10^-3);
// the frequencies of a head are computed once per workgroup.  A thread turns PAIRS consecutive pairs of a row.
constexpr int kRopeThreads = 256;

template <typename T, int PAIRS>
__global__ __launch_bounds__(kRopeThreads) void rope_kernel(T* __restrict__ mat, int64_t ld, int rows, int width, int head_dim, int skip,
                                                            int split, int add_lo, int add_hi, float base) {
    extern __shared__ double theta[];                    // [head_dim / 2]
    const int half = head_dim >> 1;
    for (int i = threadIdx.x; i < half; i += kRopeThreads) theta[i] = exp2(-2.0 * (double)i / (double)head_dim * log2((double)base));
    __syncthreads();
    const int per_row = width / (2 * PAIRS);
    const int64_t id = (int64_t)blockIdx.x * kRopeThreads + threadIdx.x;
    if (id >= (int64_t)rows * per_row) return;
    const int r = (int)(id / per_row), c = (int)(id - (int64_t)r * per_row) * 2 * PAIRS;       // first column of this thread
    if (r < skip) return;
    const double m = (double)(r < split ? r + add_lo : r + add_hi);
    T* __restrict__ p = mat + (int64_t)r * ld + c;
    float v[2 * PAIRS];
    if constexpr (sizeof(T) == 2 && PAIRS == 4) {
        const u32x4 w = *reinterpret_cast<const u32x4*>(p);
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = __uint_as_float(ww[e] << 16);
            v[2 * e + 1] = __uint_as_float(ww[e] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 2 * PAIRS; ++e) {
            if constexpr (sizeof(T) == 2) v[e] = bf16_bits_to_f32(p[e]);
            else v[e] = p[e];
        }
    }
    const int i0 = (c % head_dim) >> 1;
#pragma unroll
    for (int e = 0; e < PAIRS; ++e) {
        double turns = m * theta[i0 + e] * 0.15915494309189535;       // angle / 2 pi
        turns -= floor(turns);
        const float a = (float)(turns * 6.283185307179586);
        const float cs = cosf(a), sn = sinf(a);
        const float x0 = v[2 * e], x1 = v[2 * e + 1];
        v[2 * e] = x0 * cs - x1 * sn;
        v[2 * e + 1] = x0 * sn + x1 * cs;
    }
    if constexpr (sizeof(T) == 2 && PAIRS == 4) {
        u32x4 w;
        w.x = pack_bf16x2(v[0], v[1]);
        w.y = pack_bf16x2(v[2], v[3]);
        w.z = pack_bf16x2(v[4], v[5]);
        w.w = pack_bf16x2(v[6], v[7]);
        *reinterpret_cast<u32x4*>(p) = w;
    } else {
#pragma unroll
        for (int e = 0; e < 2 * PAIRS; ++e) store_elem<T>(p + e, v[e]);
    }
}

int launch_rope(int dtype, void* mat, int64_t ld, int rows, int n_heads, int head_dim, int skip, int split, int add_lo, int add_hi,
                float base, hipStream_t s) {
    if (rows <= 0) return ASTRA_OK;
    if (head_dim <= 0 || head_dim % 2 != 0 || !(base > 0.f)) return ASTRA_ERR_SHAPE;
    const int width = n_heads * head_dim;
    const size_t lds = (size_t)(head_dim / 2) * sizeof(double);
    const bool vec = dtype == ASTRA_BF16 && head_dim % 8 == 0 && ld % 8 == 0;
    const int64_t n = (int64_t)rows * (width / (vec ? 8 : 2));
    const int64_t blocks = ceil_div(n, kRopeThreads);
    if (blocks > 0x7fffffff) return ASTRA_ERR_SHAPE;
    if (vec) rope_kernel<uint16_t, 4><<<(int)blocks, kRopeThreads, lds, s>>>((uint16_t*)mat, ld, rows, width, head_dim, skip, split, add_lo, add_hi, base);
    else if (dtype == ASTRA_BF16) rope_kernel<uint16_t, 1><<<(int)blocks, kRopeThreads, lds, s>>>((uint16_t*)mat, ld, rows, width, head_dim, skip, split, add_lo, add_hi, base);
    else rope_kernel<float, 1><<<(int)blocks, kRopeThreads, lds, s>>>((float*)mat, ld, rows, width, head_dim, skip, split, add_lo, add_hi, base);
    return launch_status();
}

}  // namespace astra
