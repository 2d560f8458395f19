// The bf16 tile kernel's instantiations for the Transformer block around the attention layer (paper Sec. 3.1: the
// position-wise MLP runs locally on each device): activation and gated epilogues, the fp32 store that starts its
// accumulation from the residual stream, and the split contraction with its reduction.
#include "gemm_bf16_tile.h"

namespace astra {

// out[m, n] = sum over slices (ascending) of part[s][m, n] + bias[n] + residual[m, n]; N % 4 == 0.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, int n_split, int64_t mn, int N, int ldc,
                                                            const uint16_t* __restrict__ bias, const float* residual, float* out) {
    const int64_t i4 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i4 >= mn) return;
    const int64_t m = i4 / N;
    const int n = (int)(i4 - m * N);
    f32x4 acc = *reinterpret_cast<const f32x4*>(part + i4);
    for (int s = 1; s < n_split; ++s) acc += *reinterpret_cast<const f32x4*>(part + s * mn + i4);
    if (bias) {
        const u32x2 bb = *reinterpret_cast<const u32x2*>(bias + n);
        acc.x += __uint_as_float(bb.x << 16);
        acc.y += __uint_as_float(bb.x & 0xffff0000u);
        acc.z += __uint_as_float(bb.y << 16);
        acc.w += __uint_as_float(bb.y & 0xffff0000u);
    }
    const int64_t at = m * ldc + n;
    if (residual) acc += *reinterpret_cast<const f32x4*>(residual + at);
    *reinterpret_cast<f32x4*>(out + at) = acc;
}

// A wide, short bf16 output (few 256 x 256 tiles) with a long contraction is cut along the contraction so that the
// large tiles fill the chip: the number of slices (1 = no split).
int gemm_split_factor(int dtype, int64_t M, int64_t N, int64_t K) {
    if (dtype != ASTRA_BF16 || N % 4 != 0) return 1;
    const int64_t tiles = ceil_div(M, 256) * ceil_div(N, 256);
    if (tiles >= 128 || tiles == 0) return 1;
    for (int s = 8; s >= 2; --s)
        if (tiles * s <= kCus && tiles * s >= kCus * 3 / 4 && K % (kBK * s) == 0 && K / s >= 2048) return s;
    return 1;
}
size_t gemm_split_workspace_bytes(int dtype, int64_t M, int64_t N, int64_t K) {
    const int s = gemm_split_factor(dtype, M, N, K);
    return s > 1 ? (size_t)s * M * N * sizeof(float) : 0;
}

int launch_split_reduce(const float* part, int n_split, const GemmProblem& p, hipStream_t s) {
    const int64_t mn = (int64_t)p.M * p.N;
    splitk_reduce_kernel<<<(int)ceil_div(mn / 4, 256), 256, 0, s>>>(part, n_split, mn, p.N, p.ldc, (const uint16_t*)p.bias, p.residual,
                                                                     (float*)p.c);
    return launch_status();
}

template <int EPI>
static void launch_epi(bool big, const GemmBatch& batch, int grid, hipStream_t s) {
    if (big) gemm_nt_bf16_kernel<256, 256, 2, 4, false, false, EPI><<<grid, 512, 0, s>>>(batch);
    else if (grid <= kCus && batch.p[0].K % (2 * kBK) == 0) gemm_nt_bf16_kernel<128, 128, 2, 2, false, false, EPI, 2><<<grid, 512, 0, s>>>(batch);
    else gemm_nt_bf16_kernel<128, 128, 4, 2, false, false, EPI><<<grid, 512, 0, s>>>(batch);
}

// 64 x 64 tiles on two contraction groups (launches of a handful of tiles: see launch_gemm_batch); the batch was filled
// for that tile size and every contraction is a multiple of 128
int launch_gemm_mlp_small(int epi, const GemmBatch& batch, int grid, hipStream_t s) {
    if (grid <= 0) return ASTRA_OK;
    switch (epi) {
        case kEpiResidualF32: gemm_nt_bf16_kernel<64, 64, 2, 2, false, false, kEpiResidualF32, 2><<<grid, 512, 0, s>>>(batch); break;
        case kEpiGeluTanh: gemm_nt_bf16_kernel<64, 64, 2, 2, false, false, kEpiGeluTanh, 2><<<grid, 512, 0, s>>>(batch); break;
        case kEpiGeluErf: gemm_nt_bf16_kernel<64, 64, 2, 2, false, false, kEpiGeluErf, 2><<<grid, 512, 0, s>>>(batch); break;
        default: return ASTRA_ERR_UNSUPPORTED;
    }
    return launch_status();
}

// big: 256 x 256 tiles, else 128 x 128 (two contraction groups when the contraction is a multiple of 128), both on 512
// threads; the batch was filled for that tile size.
int launch_gemm_mlp(int epi, bool big, const GemmBatch& batch, int grid, hipStream_t s) {
    if (grid <= 0) return ASTRA_OK;
    switch (epi) {
        case kEpiResidualF32: launch_epi<kEpiResidualF32>(big, batch, grid, s); break;
        case kEpiGeluTanh: launch_epi<kEpiGeluTanh>(big, batch, grid, s); break;
        case kEpiGeluErf: launch_epi<kEpiGeluErf>(big, batch, grid, s); break;
        case kEpiSwiGLU: launch_epi<kEpiSwiGLU>(big, batch, grid, s); break;
        case kEpiSplit:
            if (!big) return ASTRA_ERR_UNSUPPORTED;
            gemm_nt_bf16_kernel<256, 256, 2, 4, false, false, kEpiSplit><<<grid, 512, 0, s>>>(batch);
            break;
        default: return ASTRA_ERR_UNSUPPORTED;
    }
    return launch_status();
}

}  // namespace astra
