// Grouped vector quantisation on gfx950: codeword norms, nearest-codeword encode, codebook-gather
// decode (paper Sec. 2 "Vanilla VQ" / "Grouped VQ", Sec. 3.2 "Vector-Quantized Non-Local Tokens").
#include <type_traits>

#include "common.h"
#include "vq_encode_body.h"

namespace astra {

// ------------------------------------------------------------------------------------------------
// ||c||^2 per codeword, fp32.  Sixteen lanes per codeword read its values in consecutive 16-lane strides (coalesced for wide
// groups, where one thread per codeword would walk thousands of values alone); each lane adds its values in ascending
// order with fused multiply-adds, the sixteen partial sums are then added pairwise across lanes: a fixed order.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void vq_cnorm_kernel(const T* __restrict__ codebook, float* __restrict__ cnorm, int64_t n_codewords, int dg) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;
    const int sub = threadIdx.x & 15;
    const int64_t ic = i < n_codewords ? i : n_codewords - 1;         // clamped: every lane takes part in the shuffles
    const T* c = codebook + ic * dg;
    float s = 0.f;
    for (int j = sub; j < dg; j += 16) {
        float v;
        if constexpr (sizeof(T) == 2) v = bf16_bits_to_f32(c[j]); else v = c[j];
        s = fmaf(v, v, s);
    }
    for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (sub == 0 && i < n_codewords) cnorm[i] = s;
}

int launch_vq_prepare(const astra_vq_desc& d, const void* codebook, float* cnorm, hipStream_t s) {
    const int64_t n = (int64_t)d.n_groups * d.codebook_size;
    const int dg = d.d_model / d.n_groups;
    const int64_t blocks = ceil_div(n * 16, 256);
    if (blocks > 0x7fffffff) return ASTRA_ERR_SHAPE;
    if (d.dtype == ASTRA_BF16)
        vq_cnorm_kernel<uint16_t><<<(int)blocks, 256, 0, s>>>((const uint16_t*)codebook, cnorm, n, dg);
    else
        vq_cnorm_kernel<float><<<(int)blocks, 256, 0, s>>>((const float*)codebook, cnorm, n, dg);
    return launch_status();
}

// ------------------------------------------------------------------------------------------------
// Decode: a pure gather.  One CHUNK-byte piece of one (token, group) row per thread and pass, kDecUnroll passes per
// thread a whole grid apart: consecutive threads write consecutive addresses of x_hat; the lanes of one group row read
// the same code (a broadcast) and consecutive pieces of one codeword.  The passes' code reads, codeword reads and stores
// are issued as three batches, so that every thread has kDecUnroll independent chains in flight (the step is bound by
// memory latency times bytes in flight, not by arithmetic); piece -> (token, group, offset) uses multiply-high divisions.
// ------------------------------------------------------------------------------------------------
constexpr int kDecUnroll = 4;

template <typename ChunkT, typename CodeT>
__global__ __launch_bounds__(256) void vq_decode_kernel(const CodeT* __restrict__ codes, const ChunkT* __restrict__ codebook,
                                                        ChunkT* __restrict__ x_hat, uint32_t n_chunks, uint32_t chunks_per_token,
                                                        uint32_t chunks_per_group, uint32_t magic_token, uint32_t magic_group, int G, int K) {
    const uint32_t stride = gridDim.x * 256u;
    const uint32_t first = blockIdx.x * 256u + threadIdx.x;
    uint32_t idx[kDecUnroll], src[kDecUnroll];
    int code[kDecUnroll];
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
        idx[u] = first + (uint32_t)u * stride;
        const uint32_t i = idx[u] < n_chunks ? idx[u] : n_chunks - 1;       // clamped, not guarded: the store below is the only guard
        const uint32_t t = __umulhi(i, magic_token);
        const uint32_t c = i - t * chunks_per_token;
        const uint32_t g = __umulhi(c, magic_group);
        src[u] = g * (uint32_t)K * chunks_per_group + (c - g * chunks_per_group);
        code[u] = (int)codes[(uint64_t)t * (uint32_t)G + g];
    }
    ChunkT v[kDecUnroll];
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
        const int cd = code[u] < K ? code[u] : K - 1;
        v[u] = codebook[(uint64_t)src[u] + (uint64_t)cd * chunks_per_group];
    }
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u)
        if (idx[u] < n_chunks) x_hat[idx[u]] = v[u];
}

// one thread per piece, 64-bit indices: shapes beyond 2^31 pieces
template <typename ChunkT, typename CodeT>
__global__ void vq_decode_big_kernel(const CodeT* __restrict__ codes, const ChunkT* __restrict__ codebook,
                                     ChunkT* __restrict__ x_hat, int64_t n_chunks, int chunks_per_token,
                                     int chunks_per_group, int G, int K) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_chunks) return;
    const int64_t t = idx / chunks_per_token;
    const int c = (int)(idx - t * chunks_per_token);
    const int g = c / chunks_per_group;
    const int r = c - g * chunks_per_group;
    int code = (int)codes[t * G + g];
    code = code < K ? code : K - 1;
    x_hat[idx] = codebook[((int64_t)g * K + code) * chunks_per_group + r];
}

// floor(n / d) == umulhi(n, magic) with magic = floor(2^32 / d) + 1 for every n <= n_max as long as
// n_max * (magic * d - 2^32) < 2^32 (the estimate's excess stays below 1 / d; for a power of two magic = 2^32 / d is exact);
// false when that cannot be guaranteed or d < 2
// (the caller then runs the kernel with 64-bit divisions)
static bool magic_div(uint32_t d, uint64_t n_max, uint32_t* magic) {
    if (d < 2) return false;
    if ((((uint64_t)1 << 32) % d) == 0) {           // a power of two: 2^32 / d is exact for every 32-bit n
        *magic = (uint32_t)(((uint64_t)1 << 32) / d);
        return true;
    }
    const uint64_t m = ((uint64_t)1 << 32) / d + 1;
    // error of the estimate: n * (m * d - 2^32) / (2^32 * d) must stay below 1 / d  <=>  n * (m * d - 2^32) < 2^32
    const uint64_t e = m * d - ((uint64_t)1 << 32);
    if (m > 0xffffffffull || n_max * e >= ((uint64_t)1 << 32)) return false;
    *magic = (uint32_t)m;
    return true;
}

template <typename ChunkT>
static int decode_dispatch(const astra_vq_desc& d, const void* codes, int64_t n_tokens, const void* codebook,
                           void* x_hat, hipStream_t s) {
    const int eb = elem_bytes(d.dtype);
    const int dg = d.d_model / d.n_groups;
    const int cpg = dg * eb / (int)sizeof(ChunkT);
    const int cpt = cpg * d.n_groups;
    const int64_t n_chunks = n_tokens * cpt;
    const int threads = 256;
    uint32_t magic_t = 0, magic_g = 0;
    const int64_t cb_chunks = (int64_t)d.n_groups * d.codebook_size * cpg;
    if (n_chunks < ((int64_t)1 << 31) && cb_chunks < ((int64_t)1 << 32) && magic_div((uint32_t)cpt, (uint64_t)n_chunks, &magic_t) &&
        magic_div((uint32_t)cpg, (uint64_t)cpt, &magic_g)) {
        const int64_t blocks = ceil_div(n_chunks, threads * kDecUnroll);
        if (d.code_type == ASTRA_CODE_U8)
            vq_decode_kernel<ChunkT, uint8_t><<<(int)blocks, threads, 0, s>>>(
                (const uint8_t*)codes, (const ChunkT*)codebook, (ChunkT*)x_hat, (uint32_t)n_chunks, (uint32_t)cpt, (uint32_t)cpg, magic_t,
                magic_g, d.n_groups, d.codebook_size);
        else
            vq_decode_kernel<ChunkT, uint16_t><<<(int)blocks, threads, 0, s>>>(
                (const uint16_t*)codes, (const ChunkT*)codebook, (ChunkT*)x_hat, (uint32_t)n_chunks, (uint32_t)cpt, (uint32_t)cpg, magic_t,
                magic_g, d.n_groups, d.codebook_size);
        return launch_status();
    }
    const int64_t blocks = ceil_div(n_chunks, threads);
    if (blocks > 0x7fffffff) return ASTRA_ERR_SHAPE;
    if (d.code_type == ASTRA_CODE_U8)
        vq_decode_big_kernel<ChunkT, uint8_t><<<(int)blocks, threads, 0, s>>>(
            (const uint8_t*)codes, (const ChunkT*)codebook, (ChunkT*)x_hat, n_chunks, cpt, cpg, d.n_groups, d.codebook_size);
    else
        vq_decode_big_kernel<ChunkT, uint16_t><<<(int)blocks, threads, 0, s>>>(
            (const uint16_t*)codes, (const ChunkT*)codebook, (ChunkT*)x_hat, n_chunks, cpt, cpg, d.n_groups, d.codebook_size);
    return launch_status();
}

int launch_vq_decode(const astra_vq_desc& d, const void* codes, int64_t n_tokens, const void* codebook,
                     void* x_hat, hipStream_t s) {
    if (n_tokens == 0) return ASTRA_OK;
    const int row_bytes = d.d_model / d.n_groups * elem_bytes(d.dtype);
    if (row_bytes % 16 == 0) return decode_dispatch<uint4>(d, codes, n_tokens, codebook, x_hat, s);
    if (row_bytes % 8 == 0) return decode_dispatch<uint2>(d, codes, n_tokens, codebook, x_hat, s);
    if (row_bytes % 4 == 0) return decode_dispatch<uint32_t>(d, codes, n_tokens, codebook, x_hat, s);
    return decode_dispatch<uint16_t>(d, codes, n_tokens, codebook, x_hat, s);
}

// ------------------------------------------------------------------------------------------------
// Rows -> the transposed layout the bf16 attention kernel reads its values in: dst [C, ldv] with the token index
// permuted inside blocks of 16 (offsets 0-3, 8-11, 4-7, 12-15: bits 2 and 3 of the offset swapped), columns beyond
// T zero.  The rows are either a dense matrix src [T, ld_src] or, for values that arrive as codes (the variant that
// quantises K and V after projection), looked up in the codebook on the way (GATHER; dg a multiple of 8).
// One workgroup moves 64 tokens x 64 channels through LDS: 16-byte pieces in, 16-byte pieces (8 tokens of one
// channel) out, 8 consecutive threads writing 128 contiguous bytes.
// ------------------------------------------------------------------------------------------------
constexpr int kVtStride = 72;      // halfwords per LDS row: 16-byte aligned, and 8 rows of one column fall into 8 different banks

template <bool GATHER, typename CodeT>
__global__ __launch_bounds__(256) void vt_pack_kernel(const uint16_t* __restrict__ src, int64_t ld_src, const CodeT* __restrict__ codes,
                                                      const uint16_t* __restrict__ codebook, int T, int G, int K, int dg,
                                                      uint16_t* __restrict__ dst, int ldv) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * kVtStride];
    const int t0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int piece = tid + 256 * it;
        const int tl = piece >> 3, pc = piece & 7;
        const int t = t0 + tl, c = c0 + 8 * pc;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (t < T) {
            if (GATHER) {
                const int g = c / dg, j = c - g * dg;
                int code = (int)codes[(int64_t)t * G + g];
                code = code < K ? code : K - 1;
                v = *reinterpret_cast<const u32x4*>(codebook + ((int64_t)g * K + code) * dg + j);
            } else {
                v = *reinterpret_cast<const u32x4*>(src + (int64_t)t * ld_src + c);
            }
        }
        *reinterpret_cast<u32x4*>(&tile[tl * kVtStride + 8 * pc]) = v;
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int q = tid & 7;                      // which run of 8 positions of the 64 tokens
        const int c = (tid >> 3) + 32 * it;
        const int blk = q >> 1, half = q & 1;
        uint16_t e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int p = 8 * half + i;
            const int o = (((p >> 2) & 1) << 3) | ((p >> 3) << 2) | (p & 3);
            e[i] = tile[(16 * blk + o) * kVtStride + c];
        }
        u32x4 w;
        w.x = e[0] | ((uint32_t)e[1] << 16);
        w.y = e[2] | ((uint32_t)e[3] << 16);
        w.z = e[4] | ((uint32_t)e[5] << 16);
        w.w = e[6] | ((uint32_t)e[7] << 16);
        *reinterpret_cast<u32x4*>(dst + (int64_t)(c0 + c) * ldv + t0 + 8 * q) = w;
    }
}

// src != nullptr: plain rows; else codes + codebook (d describes the codebook; d.d_model = C).
int launch_vt_pack(const astra_vq_desc& d, const void* src, int64_t ld_src, const void* codes, const void* codebook, int T, int C,
                   void* dst, int ldv, hipStream_t s) {
    if (d.dtype != ASTRA_BF16 || C % 64 != 0 || ldv % 64 != 0 || ldv < T || T < 0) return ASTRA_ERR_UNSUPPORTED;
    if (ldv == 0) return ASTRA_OK;
    const dim3 grid(ldv / 64, C / 64);
    uint16_t* out = (uint16_t*)dst;
    if (src) {
        if (ld_src % 8 != 0) return ASTRA_ERR_UNSUPPORTED;
        vt_pack_kernel<false, uint8_t><<<grid, 256, 0, s>>>((const uint16_t*)src, ld_src, nullptr, nullptr, T, 0, 0, 0, out, ldv);
        return launch_status();
    }
    const int dg = d.d_model / d.n_groups;
    if (dg % 8 != 0 || d.d_model != C) return ASTRA_ERR_UNSUPPORTED;
    if (d.code_type == ASTRA_CODE_U16)
        vt_pack_kernel<true, uint16_t><<<grid, 256, 0, s>>>(nullptr, 0, (const uint16_t*)codes, (const uint16_t*)codebook, T, d.n_groups,
                                                            d.codebook_size, dg, out, ldv);
    else
        vt_pack_kernel<true, uint8_t><<<grid, 256, 0, s>>>(nullptr, 0, (const uint8_t*)codes, (const uint16_t*)codebook, T, d.n_groups,
                                                           d.codebook_size, dg, out, ldv);
    return launch_status();
}

// ------------------------------------------------------------------------------------------------
// The three gathers of the layer that quantises K and V after projection, as one launch (each is a few microseconds of
// work behind a launch's fixed cost): K-hat rows looked up from the peers' key codes (row-major), V-hat looked up from
// their value codes and the local V rows, both into the transposed layout of vt_pack_kernel.  A workgroup moves 64
// tokens x 64 channels; blockIdx.x walks the tiles of the three jobs one after the other.
// ------------------------------------------------------------------------------------------------
struct KvPackJob {
    const void* codes_k;      // [T_n, G]
    const void* codes_v;
    const uint16_t* cb_k;     // [G, K, dg]
    const uint16_t* cb_v;
    const uint16_t* v_loc;    // [T_q, C] row-major
    uint16_t* k_hat;          // [T_n, C] row-major
    uint16_t* v_hat_t;        // [C, ldv_hat]
    uint16_t* v_loc_t;        // [C, ldv_loc]
    int32_t T_n, T_q, C, G, K, dg, ldv_hat, ldv_loc;
    int32_t tiles_khat, tiles_vhat;     // tiles of the first two jobs
};

template <typename CodeT>
__global__ __launch_bounds__(256) void kv_pack_kernel(const KvPackJob j) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * kVtStride];
    const int tid = threadIdx.x;
    const int cblocks = j.C / 64;
    int b = blockIdx.x;
    int kind = 0;                                       // 0: K-hat rows, 1: V-hat transposed, 2: local V transposed
    if (b >= j.tiles_khat) { b -= j.tiles_khat; kind = 1; }
    if (kind == 1 && b >= j.tiles_vhat) { b -= j.tiles_vhat; kind = 2; }
    const int t0 = (b / cblocks) * 64, c0 = (b % cblocks) * 64;
    const int T = kind == 2 ? j.T_q : j.T_n;
    const CodeT* __restrict__ codes = (const CodeT*)(kind == 0 ? j.codes_k : j.codes_v);
    const uint16_t* __restrict__ cb = kind == 0 ? j.cb_k : j.cb_v;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int piece = tid + 256 * it;
        const int tl = piece >> 3, pc = piece & 7;
        const int t = t0 + tl, c = c0 + 8 * pc;
        const int tc = t < T ? t : T - 1;               // clamped: the load is never guarded
        const uint16_t* from;
        if (kind == 2) {
            from = j.v_loc + (int64_t)tc * j.C + c;
        } else {
            const int g = c / j.dg, jj = c - g * j.dg;
            int code = (int)codes[(int64_t)tc * j.G + g];
            code = code < j.K ? code : j.K - 1;
            from = cb + ((int64_t)g * j.K + code) * j.dg + jj;
        }
        u32x4 v = *reinterpret_cast<const u32x4*>(from);
        if (t >= T) v = u32x4{0u, 0u, 0u, 0u};
        if (kind == 0) {
            if (t < T) *reinterpret_cast<u32x4*>(j.k_hat + (int64_t)t * j.C + c) = v;
        } else {
            *reinterpret_cast<u32x4*>(&tile[tl * kVtStride + 8 * pc]) = v;
        }
    }
    if (kind == 0) return;                              // the same for the whole workgroup
    __syncthreads();
    uint16_t* __restrict__ dst = kind == 1 ? j.v_hat_t : j.v_loc_t;
    const int ldv = kind == 1 ? j.ldv_hat : j.ldv_loc;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int q = tid & 7;                      // which run of 8 positions of the 64 tokens
        const int c = (tid >> 3) + 32 * it;
        const int blk = q >> 1, half = q & 1;
        uint16_t e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int p = 8 * half + i;
            const int o = (((p >> 2) & 1) << 3) | ((p >> 3) << 2) | (p & 3);
            e[i] = tile[(16 * blk + o) * kVtStride + c];
        }
        u32x4 w;
        w.x = e[0] | ((uint32_t)e[1] << 16);
        w.y = e[2] | ((uint32_t)e[3] << 16);
        w.z = e[4] | ((uint32_t)e[5] << 16);
        w.w = e[6] | ((uint32_t)e[7] << 16);
        *reinterpret_cast<u32x4*>(dst + (int64_t)(c0 + c) * ldv + t0 + 8 * q) = w;
    }
}

// bf16 only; C = H_kv * dh a multiple of 64, dg a multiple of 8, ldv_* multiples of 64 >= the token counts.  T_n or T_q may be 0.
int launch_kv_pack(const astra_vq_desc& d, const void* codes_k, const void* codes_v, const void* cb_k, const void* cb_v, const void* v_loc,
                   int T_n, int T_q, int C, void* k_hat, void* v_hat_t, int ldv_hat, void* v_loc_t, int ldv_loc, hipStream_t s) {
    const int dg = d.d_model / d.n_groups;
    if (d.dtype != ASTRA_BF16 || d.d_model != C || C % 64 != 0 || dg % 8 != 0 || ldv_hat % 64 != 0 || ldv_loc % 64 != 0 || ldv_hat < T_n ||
        ldv_loc < T_q || T_n < 0 || T_q < 0)
        return ASTRA_ERR_UNSUPPORTED;
    KvPackJob j{};
    j.codes_k = codes_k; j.codes_v = codes_v; j.cb_k = (const uint16_t*)cb_k; j.cb_v = (const uint16_t*)cb_v; j.v_loc = (const uint16_t*)v_loc;
    j.k_hat = (uint16_t*)k_hat; j.v_hat_t = (uint16_t*)v_hat_t; j.v_loc_t = (uint16_t*)v_loc_t;
    j.T_n = T_n; j.T_q = T_q; j.C = C; j.G = d.n_groups; j.K = d.codebook_size; j.dg = dg; j.ldv_hat = ldv_hat; j.ldv_loc = ldv_loc;
    const int64_t cblocks = C / 64;
    const int64_t t_khat = ceil_div(T_n, 64) * cblocks, t_vhat = T_n > 0 ? (int64_t)(ldv_hat / 64) * cblocks : 0;
    const int64_t t_vloc = T_q > 0 ? (int64_t)(ldv_loc / 64) * cblocks : 0;
    const int64_t total = t_khat + t_vhat + t_vloc;
    if (total > 0x7fffffff) return ASTRA_ERR_SHAPE;
    if (total == 0) return ASTRA_OK;
    j.tiles_khat = (int)t_khat; j.tiles_vhat = (int)t_vhat;
    if (d.code_type == ASTRA_CODE_U16) kv_pack_kernel<uint16_t><<<(int)total, 256, 0, s>>>(j);
    else kv_pack_kernel<uint8_t><<<(int)total, 256, 0, s>>>(j);
    return launch_status();
}

// ------------------------------------------------------------------------------------------------
// Projections of the peers' tokens from pre-projected codebooks.  A rebuilt row is a concatenation of codewords, so its
// projection is a sum of per-group products that do not depend on the token (paper Sec. 3.2: X-hat is rebuilt from the
// indices and projected with the same W_k, W_v as the local rows):
//     (X-hat W)[t, :] = sum_g C_g[codes[t, g], :] . W[g*dg:(g+1)*dg, :] = sum_g P[g, codes[t, g], :],
// with P [G, K, N] fp32 computed once per (codebook, weights) by astra_vq_project_codebook.  out[t, n] = bias[n] +
// sum_g P[g, codes[t, g], n], groups added in ascending order in fp32 and rounded once to the element type.  It reads
// G * N * 4 bytes per token and matrix where the product costs 2 * D * N flops: it pays for one or two groups.
// A workgroup owns 64 tokens x 64 channels (a thread: 8 channels of a token, twice).  TRANSPOSED (bf16): the tile goes
// through LDS into the [N, ld] layout with permuted token positions that the attention kernel reads V in (vt_pack_kernel).
// ------------------------------------------------------------------------------------------------
template <typename CodeT, typename ElemT, bool TRANSPOSED>
__global__ __launch_bounds__(256) void preproj_gather_kernel(const CodeT* __restrict__ codes, const float* __restrict__ P,
                                                             const ElemT* __restrict__ bias, int T, int G, int K, int N,
                                                             ElemT* __restrict__ dst, int ld) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[TRANSPOSED ? 64 * kVtStride : 8];
    const int t0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int piece = tid + 256 * it;
        const int tl = piece >> 3, pc = piece & 7;
        const int t = t0 + tl, c = c0 + 8 * pc;
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        const bool live = t < T && c < N;
        if (live) {
            if (bias) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if constexpr (sizeof(ElemT) == 2) acc[i] = bf16_bits_to_f32(((const uint16_t*)bias)[c + i]);
                    else acc[i] = ((const float*)bias)[c + i];
                }
            }
            for (int g = 0; g < G; ++g) {
                int code = (int)codes[(int64_t)t * G + g];
                code = code < K ? code : K - 1;
                const float* __restrict__ row = P + ((int64_t)g * K + code) * N + c;
                const f32x4 lo = *reinterpret_cast<const f32x4*>(row), hi = *reinterpret_cast<const f32x4*>(row + 4);
                acc[0] += lo.x; acc[1] += lo.y; acc[2] += lo.z; acc[3] += lo.w;
                acc[4] += hi.x; acc[5] += hi.y; acc[6] += hi.z; acc[7] += hi.w;
            }
        }
        if constexpr (sizeof(ElemT) == 2) {
            u32x4 v;
            v.x = pack_bf16x2(acc[0], acc[1]);
            v.y = pack_bf16x2(acc[2], acc[3]);
            v.z = pack_bf16x2(acc[4], acc[5]);
            v.w = pack_bf16x2(acc[6], acc[7]);
            if constexpr (TRANSPOSED) *reinterpret_cast<u32x4*>(&tile[tl * kVtStride + 8 * pc]) = v;      // zeros beyond T
            else if (live) *reinterpret_cast<u32x4*>((uint16_t*)dst + (int64_t)t * ld + c) = v;
        } else if (live) {
            float* o = (float*)dst + (int64_t)t * ld + c;
            *reinterpret_cast<f32x4*>(o) = f32x4{acc[0], acc[1], acc[2], acc[3]};
            *reinterpret_cast<f32x4*>(o + 4) = f32x4{acc[4], acc[5], acc[6], acc[7]};
        }
    }
    if constexpr (TRANSPOSED) {
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int q = tid & 7;                      // which run of 8 positions of the 64 tokens
            const int c = (tid >> 3) + 32 * it;
            const int blk = q >> 1, half = q & 1;
            uint16_t e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int p = 8 * half + i;
                const int o = (((p >> 2) & 1) << 3) | ((p >> 3) << 2) | (p & 3);
                e[i] = tile[(16 * blk + o) * kVtStride + c];
            }
            u32x4 w;
            w.x = e[0] | ((uint32_t)e[1] << 16);
            w.y = e[2] | ((uint32_t)e[3] << 16);
            w.z = e[4] | ((uint32_t)e[5] << 16);
            w.w = e[6] | ((uint32_t)e[7] << 16);
            *reinterpret_cast<u32x4*>((uint16_t*)dst + (int64_t)(c0 + c) * ld + t0 + 8 * q) = w;
        }
    }
}

// out [T, ld] row-major in the element type, or (transposed, bf16 only) [N, ld] with ld the padded token count.
int launch_preproj_gather(int dtype, int code_type, const void* codes, const float* P, const void* bias, int T, int G, int K, int N,
                          void* dst, int ld, bool transposed, hipStream_t s) {
    if (T < 0 || G <= 0 || K <= 0 || N <= 0 || N % 8 != 0) return ASTRA_ERR_UNSUPPORTED;
    if (transposed && (dtype != ASTRA_BF16 || N % 64 != 0 || ld % 64 != 0 || ld < T)) return ASTRA_ERR_UNSUPPORTED;
    if (!transposed && ld < N) return ASTRA_ERR_SHAPE;
    const int64_t bt = transposed ? ld / 64 : ceil_div(T, 64);
    if (bt == 0) return ASTRA_OK;
    if (bt > 0x7fffffff || ceil_div(N, 64) > 65535) return ASTRA_ERR_SHAPE;
    const dim3 grid((unsigned)bt, (unsigned)ceil_div(N, 64));
    const bool c16 = code_type == ASTRA_CODE_U16;
#define ASTRA_GATHER(CT, ET, TR) preproj_gather_kernel<CT, ET, TR><<<grid, 256, 0, s>>>((const CT*)codes, P, (const ET*)bias, T, G, K, N, (ET*)dst, ld)
    if (dtype == ASTRA_BF16) {
        if (transposed) { if (c16) ASTRA_GATHER(uint16_t, uint16_t, true); else ASTRA_GATHER(uint8_t, uint16_t, true); }
        else { if (c16) ASTRA_GATHER(uint16_t, uint16_t, false); else ASTRA_GATHER(uint8_t, uint16_t, false); }
    } else {
        if (c16) ASTRA_GATHER(uint16_t, float, false); else ASTRA_GATHER(uint8_t, float, false);
    }
#undef ASTRA_GATHER
    return launch_status();
}

// ------------------------------------------------------------------------------------------------
// Encode, fp32: one wavefront per (token, group).  Lanes stride over the codewords and evaluate the
// definition sum_j (x_j - c_j)^2 directly; the wavefront then reduces (distance, index)
// lexicographically so that the lowest index wins a tie.
// ------------------------------------------------------------------------------------------------
template <typename CodeT>
__global__ __launch_bounds__(256) void vq_encode_f32_kernel(const float* __restrict__ x, int64_t ldx, int64_t n_tokens,
                                                            const float* __restrict__ codebook, CodeT* __restrict__ codes,
                                                            int G, int K, int dg) {
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    if (wave >= n_tokens * G) return;
    const int64_t t = wave / G;
    const int g = (int)(wave - t * G);
    const int lane = lane_id();
    const float* z = x + t * ldx + (int64_t)g * dg;
    float best = INFINITY;
    int arg = 0x7fffffff;
    // four elements per load where the slices allow it; the additions keep their order
    const bool vec4 = dg % 4 == 0 && ldx % 4 == 0 && ((uintptr_t)x | (uintptr_t)codebook) % 16 == 0;
    for (int k = lane; k < K; k += kWave) {
        const float* e = codebook + ((int64_t)g * K + k) * dg;
        float dist = 0.f;
        int j = 0;
        if (vec4)
            // 32 values at a time: the eight codeword loads are issued together, then consumed in ascending order
            for (; j + 32 <= dg; j += 32) {
                f32x4 ev[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) ev[u] = *reinterpret_cast<const f32x4*>(e + j + 4 * u);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const f32x4 zv = *reinterpret_cast<const f32x4*>(z + j + 4 * u);
                    const f32x4 df = ev[u] - zv;
                    dist = fmaf(df.x, df.x, dist);
                    dist = fmaf(df.y, df.y, dist);
                    dist = fmaf(df.z, df.z, dist);
                    dist = fmaf(df.w, df.w, dist);
                }
            }
        if (vec4)
            for (; j + 4 <= dg; j += 4) {
                const f32x4 ev = *reinterpret_cast<const f32x4*>(e + j);
                const f32x4 zv = *reinterpret_cast<const f32x4*>(z + j);
                const f32x4 df = ev - zv;
                dist = fmaf(df.x, df.x, dist);
                dist = fmaf(df.y, df.y, dist);
                dist = fmaf(df.z, df.z, dist);
                dist = fmaf(df.w, df.w, dist);
            }
        for (; j < dg; ++j) {
            const float diff = e[j] - z[j];
            dist = fmaf(diff, diff, dist);
        }
        if (dist < best) { best = dist; arg = k; }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float ob = __shfl_xor(best, off);
        const int oa = __shfl_xor(arg, off);
        if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    }
    if (lane == 0) codes[t * G + g] = (CodeT)arg;
}

// ------------------------------------------------------------------------------------------------
// Encode, bf16: matrix-core distance tile with a fused argmax.
//
// Minimising ||x - c||^2 over c is maximising x.c - ||c||^2/2 (||x||^2 is common to all codewords).
// A workgroup of 4 wavefronts owns 128 tokens of one group; wavefront w owns 32 of them as the N side
// of a 32x32x16 MFMA, codewords are the M side.  The accumulator is preloaded with -||c||^2/2, so after
// the contraction over the group's dg values it holds the score itself, and because a lane's 16
// accumulator values all belong to one token the running (best, index) pair lives in two registers
// per lane.  The two half-waves that share a token are merged once at the end.
// The codebook streams through LDS in tiles of 128 codewords x 64 values (XOR-swizzled 16-byte
// pieces); a token's slice stays in registers when dg <= 64, otherwise it is re-read per tile.
// ------------------------------------------------------------------------------------------------
constexpr int kEncTokens = 128;   // tokens per workgroup

// 8 consecutive bf16 of a row slice of length dg starting at element k; zero beyond dg.  Loads are never guarded
// (a guarded load compiles to a branch with a wait of its own): addresses are clamped into the slice and the
// values beyond it replaced afterwards.
__device__ __forceinline__ uint4 load_slice_chunk(const uint16_t* __restrict__ row, int k, int dg, bool vec_ok) {
    uint4 r;
    if (vec_ok) {
        r = *reinterpret_cast<const uint4*>(row + (k < dg ? k : dg - 8));
        if (k >= dg) r = make_uint4(0, 0, 0, 0);
    } else {
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t v = row[k + j < dg ? k + j : dg - 1];
            e[j] = k + j < dg ? v : 0u;
        }
        r.x = e[0] | (e[1] << 16);
        r.y = e[2] | (e[3] << 16);
        r.z = e[4] | (e[5] << 16);
        r.w = e[6] | (e[7] << 16);
    }
    return r;
}

// DW: slices of an even length that is no multiple of 8, at most 64 values (e.g. D = 768 in 64 groups of 12).  A tile
// of 128 codewords is then a contiguous run of 64 * dg 32-bit words: each thread fetches words tid, tid + 256, ...
// (coalesced) and writes each into the padded LDS layout at a position worked out once; the padding is zeroed once.
template <typename CodeT, bool DW>
__global__ __launch_bounds__(256) void vq_encode_bf16_kernel(const uint16_t* __restrict__ x, int64_t ldx, int n_tokens,
                                                             const uint16_t* __restrict__ codebook,
                                                             const float* __restrict__ cnorm, CodeT* __restrict__ codes,
                                                             int G, int K, int dg) {
    __shared__ uint4 cb_lds[kEncCw * kEncKt / 8];     // 16 KiB: [128 codewords][8 pieces of 8 bf16], swizzled
    __shared__ __align__(16) float cn_lds[kEncCw];

    const int g = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int i32 = lane & 31, h = lane >> 5;
    const bool vec_ok = (dg % 8) == 0;
    const int n_kt = (dg + kEncKt - 1) / kEncKt;

    // this lane's token (N side): clamp ragged tail for loads
    const int tok = blockIdx.x * kEncTokens + wave * 32 + i32;
    const int tok_ld = tok < n_tokens ? tok : n_tokens - 1;
    const uint16_t* xrow = x + (int64_t)tok_ld * ldx + (int64_t)g * dg;
    const uint16_t* cb_g = codebook + (int64_t)g * K * dg;
    const float* cn_g = cnorm + (int64_t)g * K;

    bf16x8 xfrag[4];
    if (n_kt == 1) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            xfrag[ks] = as_bf16x8(make_uint4(0, 0, 0, 0));
            if (16 * ks < dg) xfrag[ks] = as_bf16x8(load_slice_chunk(xrow, 16 * ks + 8 * h, dg, vec_ok));
        }
    }

    float best = -INFINITY;
    int arg = 0;

    // The pieces of the tile after the current one are fetched into registers while the current one is multiplied (the
    // loads are not 16-byte aligned in general, so they cannot go to LDS directly): (codeword tile, contraction tile)
    // pairs in walking order.
    constexpr int kDwMax = 16;                          // 64 * dg words per tile over 256 threads, dg <= 64
    uint4 stage[4];
    uint32_t stage_dw[DW ? kDwMax : 1];
    int dw_lds[DW ? kDwMax : 1];                        // byte position in cb_lds of word tid + 256 * n of a tile; -1: none
    float stage_cn = 0.f;
    const int tile_dw = 64 * dg;                        // DW: words per full tile
    const uint32_t* cb_dw = reinterpret_cast<const uint32_t*>(cb_g);
    const int last_dw = (K * dg >> 1) - 1;
    if (DW) {
        for (int c = tid; c < kEncCw * kEncKt / 8; c += 256) cb_lds[c] = make_uint4(0, 0, 0, 0);
        const float inv_dg = 1.0f / (float)dg;
#pragma unroll
        for (int n = 0; n < kDwMax; ++n) {
            const int e = 2 * (tid + 256 * n);          // first of the word's two values, counted from the tile's start
            const int cw = (int)(((float)e + 0.5f) * inv_dg);      // exact: e < 8192, dg <= 64
            const int k = e - cw * dg;
            dw_lds[n] = e < 2 * tile_dw ? (cw * 8 + ((k >> 3) ^ (cw & 7))) * 16 + (k & 7) * 2 : -1;
        }
    }
    auto fetch = [&](int cw0, int kt) {
        if (DW) {
            const int first = cw0 * (dg >> 1);
#pragma unroll
            for (int n = 0; n < kDwMax; ++n)
                if (256 * n < tile_dw) {                // the same for every thread
                    const int w = first + tid + 256 * n;
                    stage_dw[n] = cb_dw[w < last_dw ? w : last_dw];
                }
        } else {
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int c = tid + 256 * it;
                const int cw = c >> 3, kc = c & 7;
                const int cwg = cw0 + cw < K ? cw0 + cw : K - 1;
                stage[it] = load_slice_chunk(cb_g + (int64_t)cwg * dg, kt * kEncKt + kc * 8, dg, vec_ok);
            }
        }
        if (kt == 0 && tid < kEncCw) {
            const int cwg = cw0 + tid;
            stage_cn = cwg < K ? -0.5f * cn_g[cwg] : -INFINITY;
        }
    };
    fetch(0, 0);
    for (int cw0 = 0; cw0 < K; cw0 += kEncCw) {
        f32x16 acc[4];
        for (int kt = 0; kt < n_kt; ++kt) {
            __syncthreads();      // previous tile fully consumed (DW, first pass: the zero fill is complete)
            // the staged tile goes to LDS
            if (DW) {
#pragma unroll
                for (int n = 0; n < kDwMax; ++n)
                    if (256 * n < tile_dw && dw_lds[n] >= 0)
                        *reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(cb_lds) + dw_lds[n]) = stage_dw[n];
            } else {
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int c = tid + 256 * it;
                    const int cw = c >> 3, kc = c & 7;
                    cb_lds[cw * 8 + (kc ^ (cw & 7))] = stage[it];
                }
            }
            if (kt == 0 && tid < kEncCw) cn_lds[tid] = stage_cn;
            if (n_kt > 1) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    xfrag[ks] = as_bf16x8(load_slice_chunk(xrow, kt * kEncKt + 16 * ks + 8 * h, dg, vec_ok));
            }
            __syncthreads();
            // next pair on its way
            if (kt + 1 < n_kt) fetch(cw0, kt + 1);
            else if (cw0 + kEncCw < K) fetch(cw0 + kEncCw, 0);
            if (kt == 0) {
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 c4 = *reinterpret_cast<const float4*>(&cn_lds[mb * 32 + 8 * q + 4 * h]);
                        acc[mb][4 * q + 0] = c4.x; acc[mb][4 * q + 1] = c4.y;
                        acc[mb][4 * q + 2] = c4.z; acc[mb][4 * q + 3] = c4.w;
                    }
            }
            const int k_left = dg - kt * kEncKt;
            const int n_ks = k_left >= kEncKt ? 4 : (k_left + 15) / 16;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks < n_ks) {
#pragma unroll
                    for (int mb = 0; mb < 4; ++mb) {
                        const int row = mb * 32 + i32;
                        const bf16x8 a = as_bf16x8(cb_lds[row * 8 + ((2 * ks + h) ^ (row & 7))]);
                        acc[mb] = mfma_32x32x16(a, xfrag[ks], acc[mb]);
                    }
                }
            }
        }
        // fused argmax: ascending codeword order inside the lane, strict '>' keeps the lowest index
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float s = acc[mb][v];
                const int cw = cw0 + mb * 32 + acc_row(v, h);
                if (s > best) { best = s; arg = cw; }
            }
    }
    // merge the two half-waves that hold the same token
    const float ob = __shfl_xor(best, 32);
    const int oa = __shfl_xor(arg, 32);
    if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    if (h == 0 && tok < n_tokens) codes[(int64_t)tok * G + g] = (CodeT)arg;
}

// ------------------------------------------------------------------------------------------------
// Encode, bf16, fast path (vq_encode_body.h) as a kernel of its own: one workgroup of 256 threads per
// (group, block of 128 tokens).  Workgroup ids are remapped so that all token blocks of a group run on the
// same XCD and find the group's codebook in that XCD's L2.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void vq_encode_bf16_fast_kernel(const EncodeJob job) {
    __shared__ u32x4 cb_lds[kEncBufs * kEncCbSlots];    // 4 x 16 KiB: [128 codewords][8 pieces of 8 bf16], swizzled
    __shared__ f32x4 cn_lds[kEncBufs * kEncCnSlots];    // 4 x 512 B
    // contiguous runs of workgroups per XCD; consecutive virtual ids share the group
    const int total = gridDim.x;
    const int q = total / 8, rr = total % 8, xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int vid = xcd < rr ? xcd * (q + 1) + slot : rr * (q + 1) + (xcd - rr) * q + slot;
    if (vq_encode_fast_needs_zero(job.dg)) {
        vq_encode_fast_zero_lds<256>(cb_lds);
        __syncthreads();                               // zero fill done before any transfer lands
    }
    vq_encode_fast_body<256>(job, vid / job.n_tb, vid % job.n_tb, cb_lds, cn_lds);
}

int launch_vq_encode(const astra_vq_desc& d, const void* x, int64_t ldx, int64_t n_tokens, const void* codebook,
                     const float* cnorm, void* codes, hipStream_t s) {
    if (n_tokens == 0) return ASTRA_OK;
    const int G = d.n_groups, K = d.codebook_size, dg = d.d_model / G;
    if (n_tokens > 0x7fffffff / 2) return ASTRA_ERR_SHAPE;
    if (d.dtype == ASTRA_BF16) {
        if (d.d_model % 8 != 0 && dg % 8 == 0) return ASTRA_ERR_UNSUPPORTED;   // 16-byte slices need aligned rows
        const int64_t n_tb = ceil_div(n_tokens, kEncTokens);
        // fast path: whole 16-byte pieces, one contraction tile, norms readable as aligned groups of 4
        if (vq_encode_fast_ok(K, dg) && n_tb * G <= 0x7fffffff) {
            const int total = (int)(n_tb * G);
            EncodeJob job{};
            job.x = x; job.codebook = codebook; job.cnorm = cnorm; job.codes = codes; job.ldx = ldx;
            job.n_tokens = (int)n_tokens; job.G = G; job.K = K; job.dg = dg;
            job.code_bytes = d.code_type == ASTRA_CODE_U8 ? 1 : 2;
            job.n_tb = (int)n_tb; job.n_wgs = total;
            vq_encode_bf16_fast_kernel<<<total, 256, 0, s>>>(job);
            return launch_status();
        }
        if (G > 65535) return ASTRA_ERR_SHAPE;
        if (vq_encode_wide_ok(K, dg, ldx)) return launch_vq_encode_wide(d, x, ldx, n_tokens, codebook, cnorm, codes, s);
        dim3 grid((unsigned)n_tb, (unsigned)G);
        // even slices of at most 64 values that are not whole 16-byte pieces: tiles fetched as 32-bit words
        const bool dw = dg % 2 == 0 && dg % 8 != 0 && dg <= 64 && (int64_t)K * dg < 0x7fffffff &&
                        reinterpret_cast<uintptr_t>(codebook) % 4 == 0;
        const uint16_t* xb = (const uint16_t*)x;
        const uint16_t* cb = (const uint16_t*)codebook;
        if (d.code_type == ASTRA_CODE_U8) {
            if (dw) vq_encode_bf16_kernel<uint8_t, true><<<grid, 256, 0, s>>>(xb, ldx, (int)n_tokens, cb, cnorm, (uint8_t*)codes, G, K, dg);
            else vq_encode_bf16_kernel<uint8_t, false><<<grid, 256, 0, s>>>(xb, ldx, (int)n_tokens, cb, cnorm, (uint8_t*)codes, G, K, dg);
        } else {
            if (dw) vq_encode_bf16_kernel<uint16_t, true><<<grid, 256, 0, s>>>(xb, ldx, (int)n_tokens, cb, cnorm, (uint16_t*)codes, G, K, dg);
            else vq_encode_bf16_kernel<uint16_t, false><<<grid, 256, 0, s>>>(xb, ldx, (int)n_tokens, cb, cnorm, (uint16_t*)codes, G, K, dg);
        }
    } else {
        const int64_t waves = n_tokens * G;
        const int64_t blocks = ceil_div(waves, 4);
        if (blocks > 0x7fffffff) return ASTRA_ERR_SHAPE;
        if (d.code_type == ASTRA_CODE_U8)
            vq_encode_f32_kernel<uint8_t><<<(int)blocks, 256, 0, s>>>((const float*)x, ldx, n_tokens, (const float*)codebook,
                                                                      (uint8_t*)codes, G, K, dg);
        else
            vq_encode_f32_kernel<uint16_t><<<(int)blocks, 256, 0, s>>>((const float*)x, ldx, n_tokens, (const float*)codebook,
                                                                       (uint16_t*)codes, G, K, dg);
    }
    return launch_status();
}

}  // namespace astra
