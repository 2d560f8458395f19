// Grouped VQ encode (paper Sec. 2, "Vanilla VQ" / "Grouped VQ") for wide groups, compiled with the matrix-core accumulators in the
// accumulation registers (this file is built without the flag that keeps them in ordinary vector registers): a wavefront
// holds 64 accumulator values next to two chunks of 20 operand fragments in flight, which only fit that way.
#include "common.h"
#include "vq_encode_body.h"

namespace astra {

// ------------------------------------------------------------------------------------------------
// Encode, bf16, wide groups (dg a multiple of 64 above 64: few groups, down to the paper's G = 1, where the whole embedding is
// one codeword).  The distance matrix of a group is then a real GEMM over dg, too long a contraction to keep a token's slice
// in registers.  A workgroup of 8 wavefronts owns 32 tokens of one group (the N side of the 32x32x16 MFMA, the same 32 for
// every wavefront); wavefront w owns codewords [1024 p + 128 w, +128) of pass p as four accumulator blocks preloaded with
// ||c||^2, and streams both operands over dg in chunks of 64 STRAIGHT FROM GLOBAL MEMORY INTO REGISTERS: a codeword is
// read by exactly one wavefront of the workgroup, so staging it in LDS would buy nothing, and the 32 token rows are served by
// the first-level cache after the first wavefront.  Inside a chunk the contraction index is assigned so that a lane's four
// MFMA steps read 64 contiguous bytes of its row (k = 32 h + 8 s + e for half-wave h, step s): every 128-byte line is
// fetched once and used whole.  The next half chunk's 10 fragments are in flight while the 8 MFMAs of the current half run.
// The token fragment is -2x (exact in bf16), so the accumulators end as ||c||^2 - 2 x.c; the running argmin is the one of
// the narrow-group kernel (strict '<' in ascending codeword order per lane; half-waves, wavefronts and passes merged by
// (distance, index), lowest index on ties).  The codebook of the group is read once per 32 tokens (from L2).
// ------------------------------------------------------------------------------------------------
constexpr int kWideTokens = 32;
constexpr int kWideThreads = 512;
constexpr int kWideCwPass = 1024;      // codewords per pass of the workgroup: 8 wavefronts x 4 blocks of 32

template <typename CodeT>
__global__ __launch_bounds__(kWideThreads) void vq_encode_bf16_wide_kernel(const uint16_t* __restrict__ x, int64_t ldx, int n_tokens,
                                                                           const uint16_t* __restrict__ codebook,
                                                                           const float* __restrict__ cnorm, CodeT* __restrict__ codes,
                                                                           int G, int K, int dg) {
    __shared__ float m_val[8][kWideTokens];
    __shared__ int m_arg[8][kWideTokens];
    const int g = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i32 = lane & 31, h = lane >> 5;
    const int n_chunks = dg >> 6;

    const int tok = blockIdx.x * kWideTokens + i32;
    const int tok_ld = tok < n_tokens ? tok : n_tokens - 1;
    const char* __restrict__ xrow = (const char*)(x + (int64_t)tok_ld * ldx + (int64_t)g * dg) + 64 * h;
    const uint16_t* __restrict__ cb_g = codebook + (int64_t)g * K * dg;
    const float* __restrict__ cn_g = cnorm + (int64_t)g * K;

    float best = INFINITY;
    int arg = 0;
    for (int cw0 = wave * 128; cw0 < K; cw0 += kWideCwPass) {      // wave-uniform trip count
        const char* __restrict__ crow[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int cw = min(cw0 + 32 * b + i32, K - 1);
            crow[b] = (const char*)(cb_g + (int64_t)cw * dg) + 64 * h;
        }
        // accumulators start at ||c||^2; codewords past K start at +inf and never win.  Loads are clamped, not guarded (a guarded
        // load per value would become a branch each); with K a multiple of 4 a lane's four consecutive rows are one 16-byte load
        f32x16 acc[4];
        if ((K & 3) == 0) {
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int cw = cw0 + 32 * b + 8 * q + 4 * h;
                    const f32x4 cn = *reinterpret_cast<const f32x4*>(cn_g + min(cw, K - 4));
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[b][4 * q + e] = cw < K ? cn[e] : INFINITY;
                }
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int cw = cw0 + 32 * b + acc_row(v, h);
                    const float cn = cn_g[min(cw, K - 1)];
                    acc[b][v] = cw < K ? cn : INFINITY;
                }
        }
        // two register slots of half a chunk each (MFMA steps {0, 1} and {2, 3} of a chunk: the two 32-byte halves of a lane's
        // 64 bytes): while one half is multiplied, the next half is in flight
        u32x4 cf[2][4][2], xf[2][2];
        auto fetch = [&](int slot, int half_idx) {                 // half_idx = 2 * chunk + (0 | 1)
            const int o = (half_idx >> 1) * 128 + (half_idx & 1) * 32;
#pragma unroll
            for (int s_ = 0; s_ < 2; ++s_) xf[slot][s_] = *reinterpret_cast<const u32x4*>(xrow + o + 16 * s_);
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int s_ = 0; s_ < 2; ++s_) cf[slot][b][s_] = *reinterpret_cast<const u32x4*>(crow[b] + o + 16 * s_);
        };
        auto multiply = [&](int slot) {
#pragma unroll
            for (int s_ = 0; s_ < 2; ++s_) {
                const bf16x8 xv = __builtin_bit_cast(bf16x8, xf[slot][s_]);
                bf16x8 xm;
#pragma unroll
                for (int e = 0; e < 8; ++e) xm[e] = (__bf16)(-2.f * (float)xv[e]);
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[b] = mfma_32x32x16(__builtin_bit_cast(bf16x8, cf[slot][b][s_]), xm, acc[b]);
            }
        };
        const int n_half = 2 * n_chunks;                           // even
        fetch(0, 0);
        for (int hi = 0; hi < n_half; hi += 2) {
            fetch(1, hi + 1);
            multiply(0);
            if (hi + 2 < n_half) fetch(0, hi + 2);
            multiply(1);
        }
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float sc = acc[b][v];
                const bool better = sc < best;
                best = better ? sc : best;
                arg = better ? cw0 + 32 * b + acc_row(v, h) : arg;
            }
    }
    // the two half-waves hold the same tokens
    {
        const float ob = __shfl_xor(best, 32);
        const int oa = __shfl_xor(arg, 32);
        if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    }
    if (h == 0) { m_val[wave][i32] = best; m_arg[wave][i32] = arg; }
    __syncthreads();
    if (tid < kWideTokens && tok < n_tokens) {
        float bv = m_val[0][tid];
        int ba = m_arg[0][tid];
#pragma unroll
        for (int w = 1; w < 8; ++w) {
            const float ov = m_val[w][tid];
            const int oa = m_arg[w][tid];
            if (ov < bv || (ov == bv && oa < ba)) { bv = ov; ba = oa; }
        }
        codes[(int64_t)tok * G + g] = (CodeT)ba;
    }
}

bool vq_encode_wide_ok(int K, int dg, int64_t ldx) { return dg > kEncKt && dg % 64 == 0 && ldx % 8 == 0 && K >= 1; }

int launch_vq_encode_wide(const astra_vq_desc& d, const void* x, int64_t ldx, int64_t n_tokens, const void* codebook,
                          const float* cnorm, void* codes, hipStream_t s) {
    const int G = d.n_groups, K = d.codebook_size, dg = d.d_model / G;
    const int64_t n_tb = ceil_div(n_tokens, kWideTokens);
    if (G > 65535 || n_tb > 0x7fffffff) return ASTRA_ERR_SHAPE;
    dim3 grid((unsigned)n_tb, (unsigned)G);
    if (d.code_type == ASTRA_CODE_U8)
        vq_encode_bf16_wide_kernel<uint8_t><<<grid, kWideThreads, 0, s>>>((const uint16_t*)x, ldx, (int)n_tokens, (const uint16_t*)codebook,
                                                                        cnorm, (uint8_t*)codes, G, K, dg);
    else
        vq_encode_bf16_wide_kernel<uint16_t><<<grid, kWideThreads, 0, s>>>((const uint16_t*)x, ldx, (int)n_tokens, (const uint16_t*)codebook,
                                                                         cnorm, (uint16_t*)codes, G, K, dg);
    return launch_status();
}

// The second half of the encode when the distance products were run as matrix products of their own (wide groups inside the
// layer): one wavefront per (token, group) walks the K scores x.c, forms ||c||^2 - 2 x.c in fp32 and keeps the smallest, lowest
// index first (strict '<' in ascending order per lane, lanes merged by (distance, index)).
template <typename CodeT>
__global__ __launch_bounds__(256) void vq_argmin_scores_kernel(const float* __restrict__ scores, const float* __restrict__ cnorm,
                                                               CodeT* __restrict__ codes, int64_t n_rows, int G, int K) {
    const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) / kWave;        // (token, group)
    if (row >= n_rows) return;
    const int lane = lane_id();
    const int g = (int)(row % G);
    const float* __restrict__ sr = scores + row * K;
    const float* __restrict__ cn = cnorm + (int64_t)g * K;
    float best = INFINITY;
    int arg = 0x7fffffff;
    for (int k0 = 4 * lane; k0 < K; k0 += 4 * kWave) {                         // K is a multiple of 4
        const f32x4 sv = *reinterpret_cast<const f32x4*>(sr + k0);
        const f32x4 cv = *reinterpret_cast<const f32x4*>(cn + k0);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float d = fmaf(-2.f, sv[e], cv[e]);
            if (d < best) { best = d; arg = k0 + e; }
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float ob = __shfl_xor(best, off);
        const int oa = __shfl_xor(arg, off);
        if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    }
    if (lane == 0) codes[row] = (CodeT)arg;
}

int launch_vq_argmin_scores(const astra_vq_desc& d, const float* scores, const float* cnorm, int64_t n_tokens, void* codes, hipStream_t s) {
    if (n_tokens == 0) return ASTRA_OK;
    if (d.codebook_size % 4 != 0) return ASTRA_ERR_UNSUPPORTED;
    const int64_t rows = n_tokens * d.n_groups;
    const int64_t blocks = ceil_div(rows, 4);
    if (blocks > 0x7fffffff) return ASTRA_ERR_SHAPE;
    if (d.code_type == ASTRA_CODE_U8)
        vq_argmin_scores_kernel<uint8_t><<<(int)blocks, 256, 0, s>>>(scores, cnorm, (uint8_t*)codes, rows, d.n_groups, d.codebook_size);
    else
        vq_argmin_scores_kernel<uint16_t><<<(int)blocks, 256, 0, s>>>(scores, cnorm, (uint16_t*)codes, rows, d.n_groups, d.codebook_size);
    return launch_status();
}

}  // namespace astra
