// Fast bf16 encode (paper Sec. 2 "Grouped VQ": nearest codeword per group, lowest index on ties), as a device
// function over caller-provided LDS, so that it can run as a kernel of its own and as extra workgroups of the
// projection launch.
#pragma once
#include <type_traits>

#include "common.h"

namespace astra {

constexpr int kEncCw = 128;       // codewords per LDS tile
constexpr int kEncKt = 64;        // contraction values per LDS tile
constexpr int kEncBufs = 4;       // LDS tile buffers of the fast path: transfers run three tiles ahead
constexpr int kEncCbSlots = kEncCw * 8;          // 16-byte slots of one codebook tile (16 KiB)
constexpr int kEncCnSlots = kEncCw / 4;          // 16-byte slots of one tile of norms (512 B)

__device__ __forceinline__ int enc_swz(int r) { return (r >> 1) & 7; }

// What the encode needs, as plain values (also travels inside the projection launch's argument block).
struct EncodeJob {
    const void* x;            // [n_tokens, ldx] bf16
    const void* codebook;     // [G, K, dg] bf16
    const float* cnorm;       // [G, K]
    void* codes;              // [n_tokens, G] uint8 / uint16
    int64_t ldx;
    int32_t n_tokens, G, K, dg;
    int32_t code_bytes;       // 1 or 2
    int32_t n_tb;             // token blocks per group (of THREADS/2 tokens)
    int32_t n_wgs;            // workgroups that share the items (fused launch only)
};

// ------------------------------------------------------------------------------------------------
// Groups of at most 64 values (dg a multiple of 8).  A workgroup of THREADS threads owns THREADS/2 tokens
// of one group (32 per wavefront, on the N side of the 32x32x16 MFMA) and walks the group's codebook in
// tiles of 128 codewords (M side).
//   - The score is kept as a distance, ||c||^2 - 2 x.c: the token fragments are loaded once, negated and
//     doubled (exact in bf16), and the accumulator is preloaded with ||c||^2 straight from LDS, so no
//     vector-ALU work is spent on forming the score; the argmin costs a compare and two selects per value.
//   - Codebook tiles and their norms go from global memory straight into a ring of four LDS buffers,
//     three tiles ahead of the one being multiplied.  Pieces beyond dg are never transferred; the one such
//     slot a contraction step can read (dg an odd multiple of 8) is zeroed once by the caller
//     (vq_encode_fast_zero_lds, when vq_encode_fast_needs_zero) and meets zero token values.
//   - NKS, the number of contraction steps of 16 (ceil(dg / 16)), is a compile-time value: the tile's work is then
//     one basic block, and every LDS read of a tile (16 of norms, 4 NKS of codeword fragments) is requested before
//     its first MFMA, so a wavefront waits for the LDS once per tile, not once per pair of MFMAs.
// cb_lds: kEncBufs * kEncCbSlots slots, cn_lds: kEncBufs * kEncCnSlots slots.  Ends with every wavefront
// past its last LDS read only after the caller's next barrier: callers that run several items in a row
// put a barrier between them.
// ------------------------------------------------------------------------------------------------
template <int THREADS>
__device__ __forceinline__ void vq_encode_fast_zero_lds(u32x4* cb_lds) {
    for (int i = threadIdx.x; i < kEncBufs * kEncCbSlots; i += THREADS) cb_lds[i] = u32x4{0u, 0u, 0u, 0u};
}
__device__ __forceinline__ bool vq_encode_fast_needs_zero(int dg) { return (dg & 8) != 0; }

template <int THREADS, int NKS>
__device__ __forceinline__ void vq_encode_fast_body_nks(const EncodeJob& job, int g, int tb, u32x4* cb_lds, f32x4* cn_lds) {
    constexpr int WAVES = THREADS / 64;
    constexpr int TOKENS = WAVES * 32;                  // tokens per workgroup
    constexpr int ITS = kEncCbSlots / THREADS;          // codebook transfers per thread per tile
    constexpr int NORM_LANES = kEncCnSlots / WAVES;     // lanes per wavefront that fetch 4 norms each
    const int K = job.K, dg = job.dg, n_tokens = job.n_tokens;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i32 = lane & 31, h = lane >> 5;
    const int n_pieces = dg >> 3;                       // valid 16-byte pieces per codeword

    const char* __restrict__ cb_g = (const char*)((const uint16_t*)job.codebook + (int64_t)g * K * dg);
    const char* __restrict__ cn_g = (const char*)(job.cnorm + (int64_t)g * K);
    const uint32_t row_b = (uint32_t)dg * 2u;
    const int n_tiles = (K + kEncCw - 1) / kEncCw;
    // Transfer geometry: slot c = tid + THREADS*it is (codeword c/8, physical piece c%8) and receives logical
    // piece (c%8) ^ swz(c/8); swz has period 16 codewords and THREADS/8 codewords separate two `it`.  Every
    // wavefront issues exactly kEncDma transfers per tile (ITS codebook passes + its share of the norms),
    // so "tile t has landed" is a fixed vmcnt threshold.
    constexpr int kEncDma = ITS + 1;
    const int cw_l = tid >> 3;
    const int piece = (tid & 7) ^ enc_swz(cw_l);
    const bool piece_ok = piece < n_pieces;
    // byte offsets of this thread's pieces in tile 0; a tile further on is a wave-uniform step, and offsets past the
    // group's last codeword are clamped to its row K-1 (the last tile of a K that is no multiple of 128)
    uint32_t cb_off[ITS];
#pragma unroll
    for (int it = 0; it < ITS; ++it) cb_off[it] = (uint32_t)(cw_l + (THREADS / 8) * it) * row_b + (uint32_t)piece * 16u;
    const uint32_t cb_off_max = (uint32_t)(K - 1) * row_b + (uint32_t)piece * 16u;
    const uint32_t cn_off = (uint32_t)(4 * NORM_LANES * wave + 4 * lane) * 4u, cn_off_max = (uint32_t)(K - 4) * 4u;
    auto issue_tile = [&](int t) {
        const int buf = t % kEncBufs;
        const uint32_t base = lds_byte_addr(cb_lds + buf * kEncCbSlots);
        const uint32_t tile_b = (uint32_t)t * (uint32_t)kEncCw * row_b;
        if (piece_ok) {
#pragma unroll
            for (int it = 0; it < ITS; ++it)
                dma_global_to_lds_16(cb_g, min(cb_off[it] + tile_b, cb_off_max), base + (uint32_t)(64 * (wave + WAVES * it)) * 16u);
        }
        if (lane < NORM_LANES)                          // 128 norms = WAVES x NORM_LANES lanes x 16 bytes
            dma_global_to_lds_16(cn_g, min(cn_off + (uint32_t)t * (uint32_t)(kEncCw * 4), cn_off_max),
                                 lds_byte_addr(cn_lds + buf * kEncCnSlots) + (uint32_t)wave * (16u * NORM_LANES));
    };
    // the first tiles are on their way before the token values are asked for: the two latencies overlap
#pragma unroll
    for (int t = 0; t < kEncBufs - 1; ++t)
        if (t < n_tiles) issue_tile(t);

    // this lane's token (N side), as -2x so that the MFMA accumulates ||c||^2 - 2 x.c
    const int tok = tb * TOKENS + wave * 32 + i32;
    const int tok_ld = tok < n_tokens ? tok : n_tokens - 1;
    const uint16_t* xrow = (const uint16_t*)job.x + (int64_t)tok_ld * job.ldx + (int64_t)g * dg;
    bf16x8 xfrag[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
        const int k = 16 * ks + 8 * h;
        u32x4 raw = u32x4{0u, 0u, 0u, 0u};
        if (k < dg) raw = *reinterpret_cast<const u32x4*>(xrow + k);
        const bf16x8 xv = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
        for (int e = 0; e < 8; ++e) xfrag[ks][e] = (__bf16)(-2.f * (float)xv[e]);
    }

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
        const u32x4* __restrict__ cb = cb_lds + buf * kEncCbSlots;
        const f32x4* __restrict__ cnb = cn_lds + buf * kEncCnSlots;
        // all LDS reads of the tile, in the order the MFMAs use them
        f32x16 acc[4];
        bf16x8 a[NKS][4];
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const f32x4 cn = cnb[mb * 8 + 2 * vq + h];             // rows 32*mb + 8*vq + 4*h .. +3
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[mb][4 * vq + e] = cn[e];
            }
            const int row = mb * 32 + i32;
            a[0][mb] = __builtin_bit_cast(bf16x8, cb[row * 8 + (h ^ enc_swz(row))]);
        }
#pragma unroll
        for (int ks = 1; ks < NKS; ++ks)
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
                const int row = mb * 32 + i32;
                a[ks][mb] = __builtin_bit_cast(bf16x8, cb[row * 8 + ((2 * ks + h) ^ enc_swz(row))]);
            }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) acc[mb] = mfma_32x32x16(a[ks][mb], xfrag[ks], acc[mb]);
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
    if (h == 0 && tok < n_tokens) {
        if (job.code_bytes == 2) ((uint16_t*)job.codes)[(int64_t)tok * job.G + g] = (uint16_t)arg;
        else ((uint8_t*)job.codes)[(int64_t)tok * job.G + g] = (uint8_t)arg;
    }
}

template <int THREADS>
__device__ __forceinline__ void vq_encode_fast_body(const EncodeJob& job, int g, int tb, u32x4* cb_lds, f32x4* cn_lds) {
    switch ((job.dg + 15) >> 4) {
        case 1: vq_encode_fast_body_nks<THREADS, 1>(job, g, tb, cb_lds, cn_lds); break;
        case 2: vq_encode_fast_body_nks<THREADS, 2>(job, g, tb, cb_lds, cn_lds); break;
        case 3: vq_encode_fast_body_nks<THREADS, 3>(job, g, tb, cb_lds, cn_lds); break;
        default: vq_encode_fast_body_nks<THREADS, 4>(job, g, tb, cb_lds, cn_lds); break;
    }
}

// true when the fast body handles this configuration
inline bool vq_encode_fast_ok(int K, int dg) {
    return dg <= kEncKt && dg % 8 == 0 && K % 4 == 0 && (int64_t)K * dg * 2 < ((int64_t)1 << 31);
}

}  // namespace astra
