// Linear projections C[M,N] = A[M,K] . B[N,K]^T (+ bias) for the attention layer (the projections
// named under Eq. 1 of the paper): Q, K, V of the local rows, K-hat, V-hat of the rows rebuilt from
// codes, and the output projection.  Several problems run in one grouped launch; a problem may take
// its A rows straight from the codebook through the token codes (decode fused into the operand load).
#include "common.h"

namespace astra {

struct GemmBatch {
    int32_t n;
    int32_t tile_begin[kMaxGemmProblems + 1];
    int32_t tiles_n[kMaxGemmProblems];
    GemmProblem p[kMaxGemmProblems];
};

// ------------------------------------------------------------------------------------------------
// bf16, matrix cores.  128x128 output tile per workgroup of 4 wavefronts (2x2, 64x64 each = 2x2
// MFMA 32x32x16 tiles), contraction in steps of 64 staged through double-buffered LDS.  LDS tiles are
// [rows][8 pieces of 8 bf16]; piece p of row r sits at p ^ (r & 7) so that the 16-byte fragment reads
// of 8 consecutive rows cover all banks.
// ------------------------------------------------------------------------------------------------
constexpr int kBM = 128, kBN = 128, kBK = 64;

__device__ __forceinline__ int find_problem(const GemmBatch& b, int tile) {
    int p = 0;
    while (p + 1 < b.n && tile >= b.tile_begin[p + 1]) ++p;
    return p;
}

__global__ __launch_bounds__(256) void gemm_nt_bf16_kernel(const GemmBatch batch) {
    __shared__ uint4 lds_a[2][kBM * kBK / 8];   // 2 x 16 KiB
    __shared__ uint4 lds_b[2][kBN * kBK / 8];   // 2 x 16 KiB

    const int pi = find_problem(batch, blockIdx.x);
    const GemmProblem& P = batch.p[pi];
    const int tile = blockIdx.x - batch.tile_begin[pi];
    const int tn = tile % batch.tiles_n[pi], tm = tile / batch.tiles_n[pi];
    const int m0 = tm * kBM, n0 = tn * kBN;
    const int M = P.M, N = P.N, K = P.K;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int i32 = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    // Global -> register staging: thread handles piece kc of rows r0 + 32*it, it = 0..3, for A and B.
    const int kc = tid & 7, r0 = tid >> 3;
    const uint16_t* __restrict__ A = (const uint16_t*)P.a;
    const uint16_t* __restrict__ B = (const uint16_t*)P.b;
    const bool gather = P.codes != nullptr;
    const uint16_t* __restrict__ CB = (const uint16_t*)P.codebook;

    int arow[4], brow[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int ra = m0 + r0 + 32 * it, rb = n0 + r0 + 32 * it;
        arow[it] = ra < M ? ra : M - 1;
        brow[it] = rb < N ? rb : N - 1;
    }

    uint4 ra[4], rb[4];
    auto load_tile = [&](int k0) {
        const int k = k0 + kc * 8;
        const bool kin = k < K;
        if (!gather) {
#pragma unroll
            for (int it = 0; it < 4; ++it)
                ra[it] = kin ? *reinterpret_cast<const uint4*>(A + (int64_t)arow[it] * P.lda + k) : make_uint4(0, 0, 0, 0);
        } else {
            const int kk = kin ? k : 0;
            const int g = kk / P.dg, j = kk - g * P.dg;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                int code;
                if (P.code_bytes == 1) code = ((const uint8_t*)P.codes)[(int64_t)arow[it] * P.G + g];
                else code = ((const uint16_t*)P.codes)[(int64_t)arow[it] * P.G + g];
                code = code < P.Kc ? code : P.Kc - 1;
                ra[it] = kin ? *reinterpret_cast<const uint4*>(CB + ((int64_t)g * P.Kc + code) * P.dg + j) : make_uint4(0, 0, 0, 0);
            }
        }
#pragma unroll
        for (int it = 0; it < 4; ++it)
            rb[it] = kin ? *reinterpret_cast<const uint4*>(B + (int64_t)brow[it] * K + k) : make_uint4(0, 0, 0, 0);
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int r = r0 + 32 * it;
            lds_a[buf][r * 8 + (kc ^ (r & 7))] = ra[it];
            lds_b[buf][r * 8 + (kc ^ (r & 7))] = rb[it];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int n_kt = (K + kBK - 1) / kBK;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < n_kt; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < n_kt) load_tile((kt + 1) * kBK);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const int r = wm * 64 + a * 32 + i32;
                fa[a] = as_bf16x8(lds_a[buf][r * 8 + ((2 * ks + h) ^ (r & 7))]);
            }
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int r = wn * 64 + b * 32 + i32;
                fb[b] = as_bf16x8(lds_b[buf][r * 8 + ((2 * ks + h) ^ (r & 7))]);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) acc[a][b] = mfma_32x32x16(fa[a], fb[b], acc[a][b]);
        }
        if (kt + 1 < n_kt) store_tile(buf ^ 1);
        __syncthreads();
    }

    // epilogue: bias, round to bf16 (or keep fp32), store.  acc[a][b][v] is C[m, n] with m = row(v, h), n = lane % 32.
    uint16_t* __restrict__ C = (uint16_t*)P.c;
    float* __restrict__ Cf = (float*)P.c;
    const bool c_f32 = P.c_f32 != 0;
    const uint16_t* __restrict__ bias = (const uint16_t*)P.bias;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int n = n0 + wn * 64 + b * 32 + i32;
        if (n >= N) continue;
        const float bv = bias ? bf16_bits_to_f32(bias[n]) : 0.f;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 64 + a * 32 + acc_row(v, h);
                if (m < M) {
                    if (c_f32) Cf[(int64_t)m * P.ldc + n] = acc[a][b][v] + bv;
                    else C[(int64_t)m * P.ldc + n] = f32_to_bf16_bits(acc[a][b][v] + bv);
                }
            }
    }
}

// ------------------------------------------------------------------------------------------------
// fp32, vector ALU: 64x64 output tile, 256 threads x (4x4) outputs, contraction in steps of 16 through
// LDS.  Used for the small fp32 configuration; sums in ascending k with fused multiply-add.
// ------------------------------------------------------------------------------------------------
constexpr int kFM = 64, kFN = 64, kFK = 16;

__global__ __launch_bounds__(256) void gemm_nt_f32_kernel(const GemmBatch batch) {
    __shared__ float sa[kFK][kFM + 4];
    __shared__ float sb[kFK][kFN + 4];

    const int pi = find_problem(batch, blockIdx.x);
    const GemmProblem& P = batch.p[pi];
    const int tile = blockIdx.x - batch.tile_begin[pi];
    const int tn = tile % batch.tiles_n[pi], tm = tile / batch.tiles_n[pi];
    const int m0 = tm * kFM, n0 = tn * kFN;
    const int M = P.M, N = P.N, K = P.K;
    const float* __restrict__ A = (const float*)P.a;
    const float* __restrict__ B = (const float*)P.b;
    const bool gather = P.codes != nullptr;
    const float* __restrict__ CB = (const float*)P.codebook;

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    // staging: thread loads 4 consecutive k of one row: row = tid / 4, k4 = (tid % 4) * 4
    const int lr = tid >> 2, lk = (tid & 3) * 4;
    const int am = m0 + lr < M ? m0 + lr : M - 1;
    const int bn = n0 + lr < N ? n0 + lr : N - 1;

    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += kFK) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = k0 + lk + j;
            float av = 0.f, bv = 0.f;
            if (k < K) {
                if (!gather) {
                    av = A[(int64_t)am * P.lda + k];
                } else {
                    const int g = k / P.dg, jj = k - g * P.dg;
                    int code;
                    if (P.code_bytes == 1) code = ((const uint8_t*)P.codes)[(int64_t)am * P.G + g];
                    else code = ((const uint16_t*)P.codes)[(int64_t)am * P.G + g];
                    code = code < P.Kc ? code : P.Kc - 1;
                    av = CB[((int64_t)g * P.Kc + code) * P.dg + jj];
                }
                bv = B[(int64_t)bn * K + k];
            }
            sa[lk + j][lr] = av;
            sb[lk + j][lr] = bv;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kFK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sa[k][ty * 4 + i]; b[i] = sb[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    float* __restrict__ C = (float*)P.c;
    const float* __restrict__ bias = (const float*)P.bias;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n < N) C[(int64_t)m * P.ldc + n] = acc[i][j] + (bias ? bias[n] : 0.f);
        }
    }
}

int launch_gemm_batch(int dtype, const GemmProblem* problems, int n_problems, hipStream_t s) {
    if (n_problems > kMaxGemmProblems) return ASTRA_ERR_UNSUPPORTED;
    const int bm = dtype == ASTRA_BF16 ? kBM : kFM, bn = dtype == ASTRA_BF16 ? kBN : kFN;
    GemmBatch batch{};
    int total = 0, n = 0;
    for (int i = 0; i < n_problems; ++i) {
        const GemmProblem& p = problems[i];
        if (p.M <= 0 || p.N <= 0) continue;
        if (p.K <= 0) return ASTRA_ERR_SHAPE;
        if (dtype == ASTRA_BF16) {
            // 16-byte operand pieces: rows and gathered slices must start on 8-element boundaries
            if (p.K % 8 != 0 || (!p.codes && p.lda % 8 != 0) || (p.codes && p.dg % 8 != 0)) return ASTRA_ERR_UNSUPPORTED;
        }
        const int64_t tm = ceil_div(p.M, bm), tn = ceil_div(p.N, bn);
        if (tm * tn + total > 0x7fffffff) return ASTRA_ERR_SHAPE;
        batch.p[n] = p;
        batch.tile_begin[n] = total;
        batch.tiles_n[n] = (int)tn;
        total += (int)(tm * tn);
        ++n;
    }
    batch.n = n;
    for (int i = n; i <= kMaxGemmProblems; ++i) batch.tile_begin[i] = total;
    if (total == 0) return ASTRA_OK;
    if (dtype == ASTRA_BF16) gemm_nt_bf16_kernel<<<total, 256, 0, s>>>(batch);
    else gemm_nt_f32_kernel<<<total, 256, 0, s>>>(batch);
    return launch_status();
}

}  // namespace astra
