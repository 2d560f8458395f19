// Grouped vector quantisation on gfx950: codeword norms, nearest-codeword encode, codebook-gather
// decode (paper Sec. 2 "Vanilla VQ" / "Grouped VQ", Sec. 3.2 "Vector-Quantized Non-Local Tokens").
#include <type_traits>

#include "common.h"

namespace astra {

// ------------------------------------------------------------------------------------------------
// ||c||^2 per codeword, fp32.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void vq_cnorm_kernel(const T* __restrict__ codebook, float* __restrict__ cnorm, int64_t n_codewords, int dg) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_codewords) return;
    const T* c = codebook + i * dg;
    float s = 0.f;
    for (int j = 0; j < dg; ++j) {
        float v;
        if constexpr (sizeof(T) == 2) v = bf16_bits_to_f32(c[j]); else v = c[j];
        s = fmaf(v, v, s);
    }
    cnorm[i] = s;
}

int launch_vq_prepare(const astra_vq_desc& d, const void* codebook, float* cnorm, hipStream_t s) {
    const int64_t n = (int64_t)d.n_groups * d.codebook_size;
    const int dg = d.d_model / d.n_groups;
    const int threads = 256;
    const int blocks = (int)ceil_div(n, threads);
    if (d.dtype == ASTRA_BF16)
        vq_cnorm_kernel<uint16_t><<<blocks, threads, 0, s>>>((const uint16_t*)codebook, cnorm, n, dg);
    else
        vq_cnorm_kernel<float><<<blocks, threads, 0, s>>>((const float*)codebook, cnorm, n, dg);
    return launch_status();
}

// ------------------------------------------------------------------------------------------------
// Decode: a pure gather.  One thread copies one CHUNK-byte piece of one (token, group) row.
// Consecutive threads write consecutive addresses of x_hat; the lanes of one group row read the same
// code (a broadcast) and consecutive pieces of one codeword.
// ------------------------------------------------------------------------------------------------
template <typename ChunkT, typename CodeT>
__global__ void vq_decode_kernel(const CodeT* __restrict__ codes, const ChunkT* __restrict__ codebook,
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

template <typename ChunkT>
static int decode_dispatch(const astra_vq_desc& d, const void* codes, int64_t n_tokens, const void* codebook,
                           void* x_hat, hipStream_t s) {
    const int eb = elem_bytes(d.dtype);
    const int dg = d.d_model / d.n_groups;
    const int cpg = dg * eb / (int)sizeof(ChunkT);
    const int cpt = cpg * d.n_groups;
    const int64_t n_chunks = n_tokens * cpt;
    const int threads = 256;
    const int64_t blocks = ceil_div(n_chunks, threads);
    if (blocks > 0x7fffffff) return ASTRA_ERR_SHAPE;
    if (d.code_type == ASTRA_CODE_U8)
        vq_decode_kernel<ChunkT, uint8_t><<<(int)blocks, threads, 0, s>>>(
            (const uint8_t*)codes, (const ChunkT*)codebook, (ChunkT*)x_hat, n_chunks, cpt, cpg, d.n_groups, d.codebook_size);
    else
        vq_decode_kernel<ChunkT, uint16_t><<<(int)blocks, threads, 0, s>>>(
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
    for (int k = lane; k < K; k += kWave) {
        const float* e = codebook + ((int64_t)g * K + k) * dg;
        float dist = 0.f;
        for (int j = 0; j < dg; ++j) {
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
constexpr int kEncCw = 128;       // codewords per LDS tile
constexpr int kEncKt = 64;        // contraction values per LDS tile

// 8 consecutive bf16 of a row slice of length dg starting at element k; zero beyond dg.
__device__ __forceinline__ uint4 load_slice_chunk(const uint16_t* __restrict__ row, int k, int dg, bool vec_ok) {
    uint4 r = make_uint4(0, 0, 0, 0);
    if (vec_ok) {
        if (k < dg) r = *reinterpret_cast<const uint4*>(row + k);
    } else {
        uint16_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = (k + j < dg) ? row[k + j] : (uint16_t)0;
        r.x = e[0] | ((uint32_t)e[1] << 16);
        r.y = e[2] | ((uint32_t)e[3] << 16);
        r.z = e[4] | ((uint32_t)e[5] << 16);
        r.w = e[6] | ((uint32_t)e[7] << 16);
    }
    return r;
}

template <typename CodeT>
__global__ __launch_bounds__(256) void vq_encode_bf16_kernel(const uint16_t* __restrict__ x, int64_t ldx, int n_tokens,
                                                             const uint16_t* __restrict__ codebook,
                                                             const float* __restrict__ cnorm, CodeT* __restrict__ codes,
                                                             int G, int K, int dg) {
    __shared__ uint4 cb_lds[kEncCw * kEncKt / 8];     // 16 KiB: [128 codewords][8 pieces of 8 bf16], swizzled
    __shared__ float cn_lds[kEncCw];

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
        for (int ks = 0; ks < 4; ++ks) xfrag[ks] = as_bf16x8(load_slice_chunk(xrow, 16 * ks + 8 * h, dg, vec_ok));
    }

    float best = -INFINITY;
    int arg = 0;

    for (int cw0 = 0; cw0 < K; cw0 += kEncCw) {
        f32x16 acc[4];
        for (int kt = 0; kt < n_kt; ++kt) {
            __syncthreads();      // previous tile fully consumed
            // stage codebook tile: 1024 pieces, 4 per thread
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int c = tid + 256 * it;
                const int cw = c >> 3, kc = c & 7;
                const int cwg = cw0 + cw < K ? cw0 + cw : K - 1;
                const uint4 v = load_slice_chunk(cb_g + (int64_t)cwg * dg, kt * kEncKt + kc * 8, dg, vec_ok);
                cb_lds[cw * 8 + (kc ^ (cw & 7))] = v;
            }
            if (kt == 0 && tid < kEncCw) {
                const int cwg = cw0 + tid;
                cn_lds[tid] = cwg < K ? -0.5f * cn_g[cwg] : -INFINITY;
            }
            if (n_kt > 1) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    xfrag[ks] = as_bf16x8(load_slice_chunk(xrow, kt * kEncKt + 16 * ks + 8 * h, dg, vec_ok));
            }
            __syncthreads();
            if (kt == 0) {
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[mb][v] = cn_lds[mb * 32 + acc_row(v, h)];
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
// Encode, bf16, fast path for groups of at most 64 values (dg a multiple of 8): same MFMA tile and
// fused argmin as above, restructured for throughput.
//   - The score is kept as a distance, ||c||^2 - 2 x.c: the token fragments are loaded once, negated and
//     doubled (exact in bf16), and the accumulator is preloaded with ||c||^2 straight from LDS, so no
//     vector-ALU work is spent on forming the score; the argmin costs a compare and two selects per value.
//   - Codebook tiles (128 codewords) and their norms go from global memory straight into double-buffered
//     LDS, one tile ahead of the one being multiplied.  Pieces beyond dg are never transferred: those LDS
//     slots are zeroed once and meet zero token values.
//   - Workgroup ids are remapped so that all token blocks of a group run on the same XCD and find the
//     group's codebook in that XCD's L2.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int enc_swz(int r) { return (r >> 1) & 7; }

constexpr int kEncBufs = 4;       // LDS tile buffers of the fast path: transfers run three tiles ahead

template <typename CodeT>
__global__ __launch_bounds__(256) void vq_encode_bf16_fast_kernel(const uint16_t* __restrict__ x, int64_t ldx, int n_tokens,
                                                                  const uint16_t* __restrict__ codebook,
                                                                  const float* __restrict__ cnorm, CodeT* __restrict__ codes,
                                                                  int G, int K, int dg, int n_tb) {
    __shared__ u32x4 cb_lds[kEncBufs][kEncCw * 8];      // 4 x 16 KiB: [128 codewords][8 pieces of 8 bf16], swizzled
    __shared__ f32x4 cn_lds[kEncBufs][kEncCw / 4];      // 4 x 512 B

    // contiguous runs of workgroups per XCD; consecutive virtual ids share the group
    const int total = gridDim.x;
    const int q = total / 8, rr = total % 8, xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int vid = xcd < rr ? xcd * (q + 1) + slot : rr * (q + 1) + (xcd - rr) * q + slot;
    const int g = vid / n_tb, tb = vid % n_tb;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i32 = lane & 31, h = lane >> 5;
    const int n_pieces = dg >> 3;                       // valid 16-byte pieces per codeword
    const int n_ks = (dg + 15) >> 4;                    // contraction steps of 16

    // zero the tile buffers once (slots of pieces >= n_pieces stay zero for good)
    for (int i = tid; i < kEncBufs * kEncCw * 8; i += 256) (&cb_lds[0][0])[i] = u32x4{0u, 0u, 0u, 0u};

    // this lane's token (N side), as -2x so that the MFMA accumulates ||c||^2 - 2 x.c
    const int tok = tb * kEncTokens + wave * 32 + i32;
    const int tok_ld = tok < n_tokens ? tok : n_tokens - 1;
    const uint16_t* xrow = x + (int64_t)tok_ld * ldx + (int64_t)g * dg;
    bf16x8 xfrag[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int k = 16 * ks + 8 * h;
        u32x4 raw = u32x4{0u, 0u, 0u, 0u};
        if (k < dg) raw = *reinterpret_cast<const u32x4*>(xrow + k);
        const bf16x8 xv = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
        for (int e = 0; e < 8; ++e) xfrag[ks][e] = (__bf16)(-2.f * (float)xv[e]);
    }
    __syncthreads();                                   // zero fill done before any transfer lands

    const char* __restrict__ cb_g = (const char*)(codebook + (int64_t)g * K * dg);
    const char* __restrict__ cn_g = (const char*)(cnorm + (int64_t)g * K);
    const uint32_t row_b = (uint32_t)dg * 2u;
    const int n_tiles = (K + kEncCw - 1) / kEncCw;
    // Transfer geometry: slot c = tid + 256*it is (codeword c/8, physical piece c%8) and receives logical
    // piece (c%8) ^ swz(c/8); swz has period 16 codewords and 32 codewords separate two `it`.  Every
    // wavefront issues exactly kEncDma transfers per tile (4 codebook passes + its quarter of the norms),
    // so "tile t has landed" is a fixed vmcnt threshold.
    constexpr int kEncDma = 5;
    const int cw_l = tid >> 3;
    const int piece = (tid & 7) ^ enc_swz(cw_l);
    const bool piece_ok = piece < n_pieces;
    auto issue_tile = [&](int t) {
        const int buf = t % kEncBufs;
        const int cw0 = t * kEncCw;
        const uint32_t base = lds_byte_addr(&cb_lds[buf][0]);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int cw = min(cw0 + cw_l + 32 * it, K - 1);
            if (piece_ok)
                dma_global_to_lds_16(cb_g, (uint32_t)cw * row_b + (uint32_t)piece * 16u, base + (uint32_t)(64 * (wave + 4 * it)) * 16u);
        }
        if (lane < 8) {                                 // 128 norms = 4 wavefronts x 8 lanes x 16 bytes
            const int cwn = min(cw0 + 32 * wave + 4 * lane, K - 4);
            dma_global_to_lds_16(cn_g, (uint32_t)cwn * 4u, lds_byte_addr(&cn_lds[buf][0]) + (uint32_t)wave * 128u);
        }
    };

    // Running argmin of this lane.  The winner is remembered as (tile, slot) with slot = mb*16 + v, a
    // small compile-time constant per accumulator value, so the loop spends exactly a compare and two
    // selects per score; slots ascend with the codeword index inside a lane and strict '<' keeps the
    // lowest index.
    float best = INFINITY;
    int arg_slot = 0, arg_tile = 0;
    auto process_tile = [&](int t, auto ragged_tag) {
        constexpr bool kRagged = decltype(ragged_tag)::value;
        const int buf = t % kEncBufs;
        const int cw0 = t * kEncCw;
        f32x16 acc[4];
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const f32x4 cn = cn_lds[buf][mb * 8 + 2 * vq + h];     // rows 32*mb + 8*vq + 4*h .. +3
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[mb][4 * vq + e] = cn[e];
            }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < n_ks) {
#pragma unroll
                for (int mb = 0; mb < 4; ++mb) {
                    const int row = mb * 32 + i32;
                    const bf16x8 a = __builtin_bit_cast(bf16x8, cb_lds[buf][row * 8 + ((2 * ks + h) ^ enc_swz(row))]);
                    acc[mb] = mfma_32x32x16(a, xfrag[ks], acc[mb]);
                }
            }
        }
        const float best_in = best;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float sc = acc[mb][v];
                if (kRagged && cw0 + mb * 32 + acc_row(v, h) >= K) sc = INFINITY;   // codewords past K: last tile only
                const bool better = sc < best;
                best = better ? sc : best;
                arg_slot = better ? (mb * 16 + v) : arg_slot;
            }
        arg_tile = best < best_in ? t : arg_tile;
    };

#pragma unroll
    for (int t = 0; t < kEncBufs - 1; ++t)
        if (t < n_tiles) issue_tile(t);
    const int n_full = K / kEncCw;                      // tiles without codewords past K
    for (int t = 0; t < n_tiles; ++t) {
        // tile t has landed once at most the transfers of the (up to two) younger tiles are outstanding
        if (t + 2 < n_tiles) wait_vmem<2 * kEncDma>();
        else if (t + 1 < n_tiles) wait_vmem<kEncDma>();
        else wait_vmem<0>();
        __syncthreads();        // everyone's share of tile t is visible; everyone is done with tile t-1
        if (t + kEncBufs - 1 < n_tiles) issue_tile(t + kEncBufs - 1);     // into the buffer tile t-1 used
        if (t < n_full) process_tile(t, std::false_type{});
        else process_tile(t, std::true_type{});
    }
    // (tile, slot) -> codeword index
    int arg = arg_tile * kEncCw + (arg_slot >> 4) * 32 + acc_row(arg_slot & 15, h);
    // merge the two half-waves that hold the same token
    const float ob = __shfl_xor(best, 32);
    const int oa = __shfl_xor(arg, 32);
    if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    if (h == 0 && tok < n_tokens) codes[(int64_t)tok * G + g] = (CodeT)arg;
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
        if (dg <= kEncKt && dg % 8 == 0 && K % 4 == 0 && n_tb * G <= 0x7fffffff && (int64_t)K * dg * 2 < ((int64_t)1 << 31)) {
            const int total = (int)(n_tb * G);
            if (d.code_type == ASTRA_CODE_U8)
                vq_encode_bf16_fast_kernel<uint8_t><<<total, 256, 0, s>>>((const uint16_t*)x, ldx, (int)n_tokens, (const uint16_t*)codebook,
                                                                          cnorm, (uint8_t*)codes, G, K, dg, (int)n_tb);
            else
                vq_encode_bf16_fast_kernel<uint16_t><<<total, 256, 0, s>>>((const uint16_t*)x, ldx, (int)n_tokens, (const uint16_t*)codebook,
                                                                           cnorm, (uint16_t*)codes, G, K, dg, (int)n_tb);
            return launch_status();
        }
        dim3 grid((unsigned)n_tb, (unsigned)G);
        if (G > 65535) return ASTRA_ERR_SHAPE;
        if (d.code_type == ASTRA_CODE_U8)
            vq_encode_bf16_kernel<uint8_t><<<grid, 256, 0, s>>>((const uint16_t*)x, ldx, (int)n_tokens, (const uint16_t*)codebook,
                                                                cnorm, (uint8_t*)codes, G, K, dg);
        else
            vq_encode_bf16_kernel<uint16_t><<<grid, 256, 0, s>>>((const uint16_t*)x, ldx, (int)n_tokens, (const uint16_t*)codebook,
                                                                 cnorm, (uint16_t*)codes, G, K, dg);
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
