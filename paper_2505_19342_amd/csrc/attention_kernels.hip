// Mixed-precision attention of one device (paper Sec. 3.2, Eq. 1): local queries attend to the
// full-precision local keys/values and to keys/values projected from the tokens rebuilt from codes.
// The two key/value sources are never concatenated in memory: the kernels walk the visible
// non-local rows first and the local rows after them (softmax does not depend on key order).
#include "common.h"
#include "vq_encode_body.h"

#include <algorithm>
#include <type_traits>

namespace astra {

// ------------------------------------------------------------------------------------------------
// bf16, matrix cores, flash style (online softmax, nothing of size T_q x T_k is ever stored).
//
// Scores are computed transposed, S^T = K_tile . Q^T (keys on the M side, queries on the N side of the
// 32x32x16 MFMA), so the 16 accumulator values of a lane all belong to ONE query: the running max / sum
// of the online softmax are per-lane scalars, and the probabilities, rounded to bf16 in place, already
// have the register layout of the B operand of O^T += V^T . P^T.
//
// A workgroup of 8 wavefronts owns 128 query rows of one head.  Wavefront w owns the 32 rows of query
// group w & 3 and walks only the key/value tiles of parity w >> 2; the two wavefronts that share a query
// group merge their (max, sum, O) triples through LDS at the end.  The two wavefronts of a SIMD have
// different parities and are kept in opposite phases (see the schedule below): one runs its softmax on
// the vector ALU while the other occupies the matrix core.  (NPAR = 4, for short sequences with 64-wide heads: 64 query
// rows per workgroup, two query groups, and the tiles dealt to four wavefronts per group: twice the workgroups, half the
// iterations; wavefronts 0..3 still run one phase ahead of wavefronts 4..7.)  A wavefront's whole state (O^T 64, S^T 32,
// Q 32, P 16 registers) stays in ordinary vector registers.  Tiles of 64 keys are double-buffered in LDS
// with XOR-swizzled 16-byte pieces and arrive by direct global->LDS transfers, issued one iteration ahead
// by the four wavefronts that will read them.
//
// V is consumed as V^T.  With VT = true it arrives already transposed ([H_kv*dh, T_pad], tokens permuted
// inside blocks of 16 as the projection kernel writes them) and fragments are plain 16-byte LDS reads;
// with VT = false it arrives row-major [T, H_kv, dh] and is transposed by the 64-bit transposing LDS read.
//
// Workgroup order: ids are remapped so that each XCD (own L2) gets a contiguous run of heads, i.e. the
// query heads of as few KV heads as possible, and inside a head the later (heavier under causal
// masking) query blocks come first.
// ------------------------------------------------------------------------------------------------
constexpr int kAttQ = 128;       // query rows per workgroup (64 with four tile parities)
constexpr int kAttKV = 64;       // key/value rows per tile
constexpr int kAttThreads = 512;
constexpr int kXcdsA = 8;
constexpr int kAttCus = 256;     // compute units of the device the launch shapes are chosen for
constexpr float kLazy = 8.f;     // base-2 units

__device__ __forceinline__ int xcd_remap_attn(int wg, int total) {
    const int q = total / kXcdsA, r = total % kXcdsA;
    const int xcd = wg % kXcdsA, slot = wg / kXcdsA;
    return xcd < r ? xcd * (q + 1) + slot : r * (q + 1) + (xcd - r) * q + slot;
}

template <int DH>
__device__ __forceinline__ int swz_k(int r) { return DH == 128 ? (r & 15) : ((r >> 1) & 7); }
// row-major V tile read by the transposing load: 4 consecutive rows x 64 bytes must hit distinct banks
template <int DH>
__device__ __forceinline__ int swz_v(int r) { return DH == 128 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2); }
// transposed V tile: rows of 64 keys = 128 bytes, same rule as the GEMM operand tiles
__device__ __forceinline__ int swz_vt(int r) { return (r >> 1) & 7; }

// LOST: the caller passed a validity bit per non-local token (an instantiation of its own, so that the code for it does
// not disturb the register allocation and schedule of the kernel that runs without)
// ENC: the grid is the attention workgroups followed by e.n_enc_wgs workgroups that run VQ encodes nothing in this launch
// depends on (the layer that quantises K and V after projection sends their codes to its peers): they are dispatched as
// attention workgroups finish, i.e. into the tail that causal masking leaves on the units of the light query blocks.
struct AttnEncode {
    EncodeJob job[2];
    int32_t n_jobs, n_attn_wgs, n_enc_wgs;
};

template <int DH, bool VT, bool LOST = false, int NPAR = 2, bool ENC = false>
__global__ __launch_bounds__(kAttThreads) void attn_bf16_kernel(const AttnParams p, const AttnEncode e) {
    static_assert(NPAR == 2 || NPAR == 4, "two or four tile parities");
    constexpr int NQG = 8 / NPAR;              // query groups of 32 rows (wavefronts per parity)
    constexpr int kQRows = 32 * NQG;           // query rows per workgroup
    constexpr int CPR = DH / 8;                // 16-byte pieces per K (and row-major V) row
    constexpr int NKS = DH / 16;               // contraction steps of Q.K
    constexpr int NDB = DH / 32;               // 32-wide blocks of the head dimension
    constexpr int PIECES = kAttKV * CPR;       // pieces per tile
    constexpr int kParThreads = kAttThreads / NPAR;        // threads of one key parity
    constexpr int LPT = PIECES / kParThreads;  // transfers per thread per tile
    // [buffer][parity] tiles
    __shared__ u32x4 lds_k[2][NPAR][PIECES];
    __shared__ u32x4 lds_v[2][NPAR][PIECES];
    static_assert(sizeof(lds_k) + sizeof(lds_v) <= 128 * 1024, "tile buffers");
    if constexpr (ENC) {
        static_assert(!ENC || (sizeof(lds_k) >= sizeof(u32x4) * kEncBufs * kEncCbSlots && sizeof(lds_v) >= sizeof(f32x4) * kEncBufs * kEncCnSlots),
                      "the encode's ring of codebook tiles fits the key buffers, its norms the value buffers");
        if ((int)blockIdx.x >= e.n_attn_wgs) {
            u32x4* cb = &lds_k[0][0][0];
            f32x4* cn = reinterpret_cast<f32x4*>(&lds_v[0][0][0]);
            // the items of all jobs in one sequence, dealt in consecutive runs (consecutive items share the group)
            const int idx = (int)blockIdx.x - e.n_attn_wgs;
            int n_total = 0;
            for (int j = 0; j < e.n_jobs; ++j) n_total += e.job[j].G * e.job[j].n_tb;
            const int chunk = (n_total + e.n_enc_wgs - 1) / e.n_enc_wgs;
            const int hi = min((idx + 1) * chunk, n_total);
            bool zeroed = false;
            for (int it = idx * chunk; it < hi; ++it) {
                int j = 0, item = it;
                while (item >= e.job[j].G * e.job[j].n_tb) {
                    item -= e.job[j].G * e.job[j].n_tb;
                    ++j;
                }
                const EncodeJob& job = e.job[j];
                if (vq_encode_fast_needs_zero(job.dg) && !zeroed) {       // every job of a launch has the same group length
                    vq_encode_fast_zero_lds<kAttThreads>(cb);
                    __syncthreads();                       // zero fill done before any transfer lands
                    zeroed = true;
                }
                vq_encode_fast_body<kAttThreads>(job, item / job.n_tb, item % job.n_tb, cb, cn);
                __syncthreads();                           // all reads of this item's tiles done before the next item's transfers
            }
            return;
        }
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: keeps the tile bookkeeping in scalar registers
    const int i32 = lane & 31, h = lane >> 5;
    // wavefronts w and w + 4 share a SIMD and run in opposite phases; the NQG wavefronts of a parity are consecutive
    const int phase = wave >> 2;
    const int qg = wave & (NQG - 1), par = 2 * ((wave & 3) / NQG) + phase;
    const int ptid = tid & (kParThreads - 1);

    const int n_qb = (p.Tq + kQRows - 1) / kQRows;
    const int vt_id = xcd_remap_attn(blockIdx.x, ENC ? e.n_attn_wgs : (int)gridDim.x);
    const int head = vt_id / n_qb;
    const int qb = n_qb - 1 - (vt_id % n_qb);
    const int hk = head / (p.Hq / p.Hkv);
    const int q0 = qb * kQRows;
    const int Tq = p.Tq;
    const int64_t q_ld = (int64_t)p.Hq * DH, kv_ld = (int64_t)p.Hkv * DH;

    // this lane's query (N side)
    const int qrow = q0 + 32 * qg + i32;
    bf16x8 qf[NKS];
    {
        const int r = qrow < Tq ? qrow : Tq - 1;
        const uint16_t* __restrict__ Q = (const uint16_t*)p.q + (int64_t)r * q_ld + (int64_t)head * DH;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Q + 16 * ks + 8 * h));
    }

    f32x16 acc_o[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float sl2 = p.scale * 1.4426950408889634f;       // logits in base-2 units

    const int n_hat_tiles = (p.Tn_vis + kAttKV - 1) / kAttKV;
    const int loc_rows = p.causal ? min(q0 + kQRows, Tq) : Tq;    // local keys any row of this block may see
    const int n_tiles = n_hat_tiles + (loc_rows + kAttKV - 1) / kAttKV;
    const int n_pairs = (n_tiles + NPAR - 1) / NPAR;
    const int wave_q_lo = q0 + 32 * qg;

    // ---- tiles of this wavefront's parity: own iteration i works on tile NPAR * i + par of the walk (visible
    // non-local tiles first, local tiles after them).  An index past the end (odd tile count) is the last
    // tile again with every key masked, so all wavefronts run the same number of iterations.
    struct Tile {
        bool is_loc;
        int row0, count;
    };
    auto tile_of = [&](int i) {
        const int t_in = NPAR * i + par;
        const int t = t_in < n_tiles ? t_in : n_tiles - 1;
        Tile tl;
        tl.is_loc = t >= n_hat_tiles;
        tl.row0 = (tl.is_loc ? t - n_hat_tiles : t) * kAttKV;
        tl.count = t_in >= n_tiles ? 0 : (tl.is_loc ? Tq : p.Tn_vis);
        return tl;
    };

    // ---- staging: global -> LDS without passing through registers, by the four wavefronts of the parity that
    // consumes the tile.  One wavefront instruction moves 64 consecutive 16-byte LDS slots; the XOR swizzle is
    // applied on the global side (the lane that owns slot (row, piece) fetches piece ^ swizzle(row) of that row).
    // Slot c = ptid + 256*it of a K tile is (row c / CPR, piece c % CPR); both swizzles are periodic in the row
    // step between two `it`, so the piece a lane fetches is the same for every `it` and only the row changes.
    constexpr int ROW_STEP = kParThreads / CPR;               // K rows between consecutive `it`
    const int kr0 = ptid / CPR, kph = ptid % CPR;
    const uint32_t kcol = (uint32_t)((kph ^ swz_k<DH>(kr0)) * 16);                 // bytes
    const uint32_t vcol = VT ? (uint32_t)(((ptid & 7) ^ swz_vt(ptid >> 3)) * 16)    // V^T: row ptid/8 + 32*it, piece ptid%8
                             : (uint32_t)((kph ^ swz_v<DH>(kr0)) * 16);
    const uint32_t kv_ld_b = (uint32_t)kv_ld * 2u;
    const uint32_t wave_slot = (uint32_t)(64 * qg) * 16u;                      // this wavefront's 64 slots inside a pass of its parity
    constexpr uint32_t kPassBytes = (uint32_t)kParThreads * 16u;
    // byte offset of row kr0 inside a tile; the rows of pass `it` lie ROW_STEP rows further (a scalar product), and a
    // row beyond the source's last one is replaced by that last row by clamping the offset: no per-lane multiply
    const uint32_t krow_b = (uint32_t)kr0 * kv_ld_b;
    auto dma_k = [&](const Tile& tl, int buf, int it) {
        const char* __restrict__ Kb = (const char*)(tl.is_loc ? p.k_loc : p.k_hat) + ((int64_t)tl.row0 * kv_ld + (int64_t)hk * DH) * 2;
        const int lim = (tl.is_loc ? Tq : p.Tn_vis) - 1 - tl.row0;                 // last valid row of the tile
        const uint32_t off = min(krow_b + (uint32_t)(ROW_STEP * it) * kv_ld_b, (uint32_t)min(lim, kAttKV - 1) * kv_ld_b);
        dma_global_to_lds_16(Kb, off + kcol, lds_byte_addr(&lds_k[buf][par][0]) + wave_slot + (uint32_t)it * kPassBytes);
    };
    auto dma_v = [&](const Tile& tl, int buf, int it) {
        const uint32_t dst = lds_byte_addr(&lds_v[buf][par][0]) + wave_slot + (uint32_t)it * kPassBytes;
        if (VT) {
            const uint32_t v_ld_b = (uint32_t)(tl.is_loc ? p.ldv_loc : p.ldv_hat) * 2u;
            const char* __restrict__ Vb = (const char*)(tl.is_loc ? p.v_loc : p.v_hat) + ((int64_t)hk * DH * v_ld_b + (int64_t)tl.row0 * 2);
            // row ptid / 8 + (kParThreads / 8) * it of the transposed tile: one per-lane product per tile source, the pass adds a scalar
            dma_global_to_lds_16(Vb, (uint32_t)(ptid >> 3) * v_ld_b + (uint32_t)((kParThreads / 8) * it) * v_ld_b + vcol, dst);
        } else {
            const char* __restrict__ Vb = (const char*)(tl.is_loc ? p.v_loc : p.v_hat) + ((int64_t)tl.row0 * kv_ld + (int64_t)hk * DH) * 2;
            const int lim = (tl.is_loc ? Tq : p.Tn_vis) - 1 - tl.row0;
            const uint32_t off = min(krow_b + (uint32_t)(ROW_STEP * it) * kv_ld_b, (uint32_t)min(lim, kAttKV - 1) * kv_ld_b);
            dma_global_to_lds_16(Vb, off + vcol, dst);
        }
    };

    // ---- matrix-core phase of iteration i: O^T += V^T(i-1) . P^T(i-1) (PV, 16 MFMAs for dh = 128), then
    // S^T(i) = K(i) . Q^T (QK, 16 MFMAs), in units of NDB / 4 MFMAs.  The fragments of unit u+1 are requested from
    // LDS before the MFMAs of unit u are issued, and the transfers of the tiles needed one iteration later (K(i+1),
    // V(i)) are issued one per unit between the MFMAs, so that no wavefront stalls on the memory pipeline's queue.
    f32x16 acc_s[2];
    bf16x8 pf[4];
    constexpr int QK_UNITS = NKS / 2;
    auto mm_phase = [&](int i, auto parity_tag) {
        constexpr int IB = decltype(parity_tag)::value;          // = i & 1, static: the buffer addresses become immediates
        constexpr int NPV = 4, NU = NPV + QK_UNITS;
        constexpr int NDMA = 2 * LPT;
        const u32x4* __restrict__ Kt = lds_k[IB][par];
        const u32x4* __restrict__ Vt = lds_v[IB ^ 1][par];
        const Tile t_k = tile_of(i + 1), t_v = tile_of(i);
        auto load_unit = [&](int u, bf16x8(&f)[4]) {
            if (u < NPV) {
                const int kstep = u;
#pragma unroll
                for (int db = 0; db < NDB; ++db) {
                    if (VT) {
                        const int d = db * 32 + i32;
                        f[db] = __builtin_bit_cast(bf16x8, Vt[d * 8 + ((2 * kstep + h) ^ swz_vt(d))]);
                    } else {
                        const int s16 = lane & 15, q4 = lane >> 4;
                        const int c = db * 4 + 2 * (q4 & 1) + ((s16 & 3) >> 1);
                        const int r_lo = 16 * kstep + 4 * h + (s16 >> 2);
                        const int r_hi = r_lo + 8;
                        const char* base = reinterpret_cast<const char*>(Vt);
                        const s16x4 lo = lds_read_tr16_b64(base + (r_lo * CPR + (c ^ swz_v<DH>(r_lo))) * 16 + 8 * (s16 & 1));
                        const s16x4 hi = lds_read_tr16_b64(base + (r_hi * CPR + (c ^ swz_v<DH>(r_hi))) * 16 + 8 * (s16 & 1));
                        u32x4 packed;
                        packed.x = (uint16_t)lo[0] | ((uint32_t)(uint16_t)lo[1] << 16);
                        packed.y = (uint16_t)lo[2] | ((uint32_t)(uint16_t)lo[3] << 16);
                        packed.z = (uint16_t)hi[0] | ((uint32_t)(uint16_t)hi[1] << 16);
                        packed.w = (uint16_t)hi[2] | ((uint32_t)(uint16_t)hi[3] << 16);
                        f[db] = __builtin_bit_cast(bf16x8, packed);
                    }
                }
            } else {
                const int g = u - NPV;
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb) {
                        const int r = mb * 32 + i32, ks = 2 * g + j;
                        f[j * 2 + mb] = __builtin_bit_cast(bf16x8, Kt[r * CPR + ((2 * ks + h) ^ swz_k<DH>(r))]);
                    }
            }
        };
        auto compute_unit = [&](int u, const bf16x8(&f)[4]) {
            if (u < NPV) {
#pragma unroll
                for (int db = 0; db < NDB; ++db) acc_o[db] = mfma_32x32x16(f[db], pf[u], acc_o[db]);
            } else {
                const int g = u - NPV;
                if (g == 0) {
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc_s[mb][v] = 0.f;
                }
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb) acc_s[mb] = mfma_32x32x16(f[j * 2 + mb], qf[2 * g + j], acc_s[mb]);
            }
        };
        bf16x8 fa[4], fb[4];
        load_unit(0, fa);
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            if (u + 1 < NU) load_unit(u + 1, (u & 1) ? fa : fb);
            // spread the NDMA transfers over the NU units
#pragma unroll
            for (int x = u * NDMA / NU; x < (u + 1) * NDMA / NU; ++x) {
                if (x < LPT) dma_k(t_k, IB ^ 1, x);
                else dma_v(t_v, IB, x - LPT);
            }
            compute_unit(u, (u & 1) ? fb : fa);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- vector-ALU phase of iteration i: masking and online softmax of S^T(i), in base-2 units, leaving the
    // probabilities as the bf16 B operand of the next PV.  The reference maximum m_run is only raised when a score
    // exceeds it by more than kLazy (2^kLazy fits bf16 and fp32 easily): after the first tiles the accumulators are
    // almost never rescaled.
    auto softmax_phase = [&](int i) {
        const Tile tl = tile_of(i);
        const bool diag = tl.is_loc && p.causal && (tl.row0 + kAttKV - 1 > wave_q_lo);     // some pair of this wave is hidden
        // non-local keys of this tile whose codes never arrived (bit = key index inside the tile; tiles start at
        // multiples of 64 keys, one word of the caller's bit array each; a wave-uniform scalar load)
        unsigned long long lost = 0ull;
        if (LOST && !tl.is_loc && tl.count > 0) lost = ~load_uniform_u64(p.valid_bits + (tl.row0 >> 6));
        const bool masked = diag || (tl.row0 + kAttKV > tl.count) || lost != 0ull;
        // masking (ragged source tail, causal diagonal, lost codes): a wave-uniform pass of its own
        if (LOST && masked && !diag && tl.row0 + kAttKV <= tl.count) {
            // only lost codes.  Key index inside the tile = 32*mb + 4*h + c(v) with c(v) = acc_row(v, 0): the 32 lanes of
            // a half-wave look at the same key, so the lanes to drop are one scalar word per score, built on the scalar
            // unit from two bits of the tile's word, and each score costs a single select.
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k0 = 32 * mb + acc_row(v, 0);
                    const unsigned long long lanes = (((lost >> k0) & 1ull) ? 0x00000000ffffffffull : 0ull) |
                                                     (((lost >> (k0 + 4)) & 1ull) ? 0xffffffff00000000ull : 0ull);
                    acc_s[mb][v] = __builtin_amdgcn_inverse_ballot_w64(lanes) ? -INFINITY : acc_s[mb][v];
                }
        } else if (masked) {
            // key index inside the tile = 32*mb + 4*h + c(v) with c(v) = acc_row(v, 0) <= 27: one shifted word per half
            const uint32_t lost_w[2] = {(uint32_t)(lost >> (4 * h)), (uint32_t)(lost >> (32 + 4 * h))};
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = tl.row0 + mb * 32 + acc_row(v, h);
                    const bool drop = (key >= tl.count) | (diag & (key > qrow)) | (((lost_w[mb] >> acc_row(v, 0)) & 1u) != 0u);
                    acc_s[mb][v] = drop ? -INFINITY : acc_s[mb][v];
                }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, acc_s[mb][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32)) * sl2;
        float alpha = 1.f;
        const bool rescale = mx > m_run + kLazy;          // also true for the first visible key (m_run = -inf)
        if (rescale) {
            alpha = __builtin_amdgcn_exp2f(m_run - mx);
            m_run = mx;
        }
        const float m_ref = m_run == -INFINITY ? 0.f : m_run;
        float lsum = 0.f;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float e = __builtin_amdgcn_exp2f(fmaf(acc_s[mb][v], sl2, -m_ref));
                lsum += e;
                pf[mb * 2 + (v >> 3)][v & 7] = (__bf16)e;
            }
        l_run = l_run * alpha + lsum;
        if (__builtin_amdgcn_ballot_w64(rescale) != 0) {
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc_o[db][v] *= alpha;
        }
    };

    // ---- schedule.  The two wavefronts of a SIMD have different parities; parity 1 runs one phase behind parity 0,
    // and a workgroup barrier closes every phase, so while one wavefront of a SIMD occupies the matrix core the
    // other runs its softmax on the vector ALU:
    //   parity 0:  QK(0) | sm(0) | PV(0) QK(1) | sm(1) | ... | sm(n-1) | PV(n-1) |
    //   parity 1:        | QK(0) | sm(0) | PV(0) QK(1) | ... | PV(n-2) QK(n-1) | sm(n-1) | PV(n-1)
    // A tile's buffer is rewritten (by transfers issued in a matrix-core phase) one barrier-closed iteration after
    // its last reader, and every wavefront waits for its own transfers at the end of its softmax phase, before the
    // barrier that precedes the phase which reads them.
    // The loop body is the same for every iteration: the first PV multiplies zero probabilities with a zeroed V
    // buffer and the last QK (on a finite copy of the last tile) is discarded, 32 of about 1000 MFMAs.
    const int n_it = n_pairs;
    {
        const Tile t0 = tile_of(0);
#pragma unroll
        for (int it = 0; it < LPT; ++it) dma_k(t0, 0, it);
        u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int it = 0; it < LPT; ++it) lds_v[1][par][ptid + kParThreads * it] = zero;
#pragma unroll
        for (int j = 0; j < 4; ++j) pf[j] = __builtin_bit_cast(bf16x8, zero);
    }
    wait_vmem_all();
    __syncthreads();
    if (phase == 1) __syncthreads();
    for (int i = 0;; i += 2) {          // two iterations per trip: the tile buffers alternate, so each copy knows its own
        __builtin_amdgcn_s_setprio(2);      // the matrix-core phase goes first when both wavefronts of the SIMD can issue
        mm_phase(i, std::integral_constant<int, 0>{});
        __builtin_amdgcn_s_setprio(0);
        __syncthreads();
        if (i == n_it) break;
        softmax_phase(i);
        wait_vmem_all();
        __syncthreads();
        __builtin_amdgcn_s_setprio(2);
        mm_phase(i + 1, std::integral_constant<int, 1>{});
        __builtin_amdgcn_s_setprio(0);
        __syncthreads();
        if (i + 1 == n_it) break;
        softmax_phase(i + 1);
        wait_vmem_all();
        __syncthreads();
    }
    wait_vmem_all();          // transfers issued by the last matrix-core phase land in buffers the merge reuses
    if (phase == 0) __syncthreads();
    __syncthreads();

    // ---- merge the parities of each query group through LDS (the tile buffers are free now): parities 1.. hand their
    // triples to parity 0, which adds them in ascending parity
    float* xch = reinterpret_cast<float*>(&lds_k[0][0][0]);        // NDB*16*64 floats per (query group, parity > 0)
    float* xml = reinterpret_cast<float*>(&lds_v[0][0][0]);        // m, l per (query group, parity > 0, lane)
    static_assert(sizeof(lds_k) >= sizeof(float) * NQG * (NPAR - 1) * NDB * 16 * 64, "the exchange fits the key tiles");
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (par > 0) {
        const int sl = qg * (NPAR - 1) + par - 1;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) xch[((sl * NDB + db) * 16 + v) * 64 + lane] = acc_o[db][v];
        xml[(sl * 2 + 0) * 64 + lane] = m_run;
        xml[(sl * 2 + 1) * 64 + lane] = l_tot;
    }
    __syncthreads();
    if (par == 0) {
        float mo[NPAR - 1], lo[NPAR - 1];
        float m = m_run;
#pragma unroll
        for (int q = 0; q < NPAR - 1; ++q) {
            mo[q] = xml[((qg * (NPAR - 1) + q) * 2 + 0) * 64 + lane];
            lo[q] = xml[((qg * (NPAR - 1) + q) * 2 + 1) * 64 + lane];
            m = fmaxf(m, mo[q]);
        }
        const float m_safe = m == -INFINITY ? 0.f : m;
        const float a0 = __builtin_amdgcn_exp2f(m_run - m_safe);
        float ao[NPAR - 1];
        float l = l_tot * a0;
#pragma unroll
        for (int q = 0; q < NPAR - 1; ++q) {
            ao[q] = __builtin_amdgcn_exp2f(mo[q] - m_safe);
            l += lo[q] * ao[q];
        }
        const float inv = l > 0.f ? 1.f / l : 0.f;
        const float c0 = a0 * inv;
        float co[NPAR - 1];
#pragma unroll
        for (int q = 0; q < NPAR - 1; ++q) co[q] = ao[q] * inv;
        if (qrow < Tq) {
            uint16_t* __restrict__ O = (uint16_t*)p.out + (int64_t)qrow * q_ld + (int64_t)head * DH;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    float o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = 4 * vq + e;
                        o[e] = acc_o[db][v] * c0;
#pragma unroll
                        for (int q = 0; q < NPAR - 1; ++q)
                            o[e] += xch[(((qg * (NPAR - 1) + q) * NDB + db) * 16 + v) * 64 + lane] * co[q];
                    }
                    u32x2 w;
                    w.x = pack_bf16x2(o[0], o[1]);
                    w.y = pack_bf16x2(o[2], o[3]);
                    *reinterpret_cast<u32x2*>(O + db * 32 + 8 * vq + 4 * h) = w;
                }
            if (p.lse && h == 0) p.lse[(int64_t)head * Tq + qrow] = (m + log2f(l)) * 0.6931471805599453f;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// fp32, vector ALU: one workgroup of four wavefronts per (query row, head).  The keys ([K-hat | K], 64 at a time: one
// key per lane for the logits, head-dim values spread over lanes for the output) are dealt to the wavefronts chunk by
// chunk, each wavefront runs an online softmax over its chunks, and the four partial results are merged through LDS
// in wavefront order.  U = ceil(dh / 64) output values per lane.
// ------------------------------------------------------------------------------------------------
template <int U>
__global__ __launch_bounds__(256) void attn_f32_kernel(const AttnParams p, int dh) {
    constexpr int kWaves = 4;
    constexpr int kRows = U <= 2 ? 16 : 8;           // value rows in flight
    __shared__ float part[kWaves][U * kWave + 2];
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int head = blockIdx.x / p.Tq, row = blockIdx.x % p.Tq;
    const int hk = head / (p.Hq / p.Hkv);
    const int64_t q_ld = (int64_t)p.Hq * dh, kv_ld = (int64_t)p.Hkv * dh;
    const float* __restrict__ q = (const float*)p.q + (int64_t)row * q_ld + (int64_t)head * dh;

    const int n_hat = p.Tn_vis;
    const int n_loc = p.causal ? row + 1 : p.Tq;
    const int chunks_hat = (n_hat + kWave - 1) / kWave, chunks = chunks_hat + (n_loc + kWave - 1) / kWave;
    float m_run = -INFINITY, l_run = 0.f;
    float o[U];                                      // head-dim values lane, lane + 64, ... (those beyond dh are never stored)
#pragma unroll
    for (int u = 0; u < U; ++u) o[u] = 0.f;
    const bool vec4 = dh % 4 == 0 && ((uintptr_t)p.q | (uintptr_t)p.k_loc | (uintptr_t)p.k_hat) % 16 == 0;

    for (int c = wave; c < chunks; c += kWaves) {
        const int src = c < chunks_hat ? 0 : 1;
        const int count = src == 0 ? n_hat : n_loc;
        const int base = (src == 0 ? c : c - chunks_hat) * kWave;
        const float* __restrict__ Kp = (const float*)(src == 0 ? p.k_hat : p.k_loc) + (int64_t)hk * dh;
        const float* __restrict__ Vp = (const float*)(src == 0 ? p.v_hat : p.v_loc) + (int64_t)hk * dh;
        const int j = base + lane;
        float s = -INFINITY;
        const bool arrived = src != 0 || p.valid_bits == nullptr || j >= count || ((p.valid_bits[j >> 6] >> (j & 63)) & 1ull);
        if (j < count && arrived) {
            const float* kr = Kp + (int64_t)j * kv_ld;
            float dot = 0.f;
            int d = 0;
            if (vec4) {                   // ascending order of additions, four elements per load
                // 32 elements at a time: the eight key loads are issued together, then consumed in ascending order
                for (; d + 32 <= dh; d += 32) {
                    f32x4 kv[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) kv[u] = *reinterpret_cast<const f32x4*>(kr + d + 4 * u);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const f32x4 qv = *reinterpret_cast<const f32x4*>(q + d + 4 * u);
                        dot = fmaf(qv.x, kv[u].x, dot);
                        dot = fmaf(qv.y, kv[u].y, dot);
                        dot = fmaf(qv.z, kv[u].z, dot);
                        dot = fmaf(qv.w, kv[u].w, dot);
                    }
                }
                for (; d + 4 <= dh; d += 4) {
                    const f32x4 kv = *reinterpret_cast<const f32x4*>(kr + d);
                    const f32x4 qv = *reinterpret_cast<const f32x4*>(q + d);
                    dot = fmaf(qv.x, kv.x, dot);
                    dot = fmaf(qv.y, kv.y, dot);
                    dot = fmaf(qv.z, kv.z, dot);
                    dot = fmaf(qv.w, kv.w, dot);
                }
            }
            for (; d < dh; ++d) dot = fmaf(q[d], kr[d], dot);
            s = dot * p.scale;
        }
        float mx = s;
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        const float m_new = fmaxf(m_run, mx);          // -inf only while every key so far was lost
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = expf(m_run - m_safe);
        const float e = (j < count && arrived) ? expf(s - m_safe) : 0.f;
        float sum = e;
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
        l_run = l_run * alpha + sum;
        m_run = m_new;
#pragma unroll
        for (int u = 0; u < U; ++u) o[u] *= alpha;
        const int cnt = min(kWave, count - base);
        // kRows value rows in flight; rows beyond the chunk repeat its last row with weight zero
        for (int jj = 0; jj < cnt; jj += kRows) {
            float pj[kRows], vv[kRows][U];
#pragma unroll
            for (int b = 0; b < kRows; ++b) {
                const int jb = min(jj + b, cnt - 1);
                pj[b] = jj + b < cnt ? __shfl(e, jb) : 0.f;
                const float* vr = Vp + (int64_t)(base + jb) * kv_ld;
#pragma unroll
                for (int u = 0; u < U; ++u) vv[b][u] = vr[min(lane + 64 * u, dh - 1)];
            }
#pragma unroll
            for (int b = 0; b < kRows; ++b)
#pragma unroll
                for (int u = 0; u < U; ++u) o[u] = fmaf(pj[b], vv[b][u], o[u]);
        }
    }
    // merge: wavefront w leaves (o, m, l); the first wavefront adds the four in order
#pragma unroll
    for (int u = 0; u < U; ++u) part[wave][u * kWave + lane] = o[u];
    if (lane == 0) {
        part[wave][U * kWave] = m_run;
        part[wave][U * kWave + 1] = l_run;
    }
    __syncthreads();
    if (wave != 0) return;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, part[w][U * kWave]);
    const float m_safe = M == -INFINITY ? 0.f : M;
    float L = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) o[u] = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const float wgt = expf(part[w][U * kWave] - m_safe);       // exp(-inf) = 0 for a wavefront without keys
        L = fmaf(wgt, part[w][U * kWave + 1], L);
#pragma unroll
        for (int u = 0; u < U; ++u) o[u] = fmaf(wgt, part[w][u * kWave + lane], o[u]);
    }
    const float inv = L > 0.f ? 1.f / L : 0.f;
    float* __restrict__ out = (float*)p.out + (int64_t)row * q_ld + (int64_t)head * dh;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int d = lane + 64 * u;
        if (d < dh) out[d] = o[u] * inv;
    }
    if (p.lse && lane == 0) p.lse[(int64_t)head * p.Tq + row] = M + logf(L);
}

int launch_attention(int dtype, const AttnParams& p_in, int head_dim, hipStream_t s, bool plan_only, const EncodeJob* enc, int n_enc,
                     bool* enc_fused) {
    AttnParams p = p_in;
    if (enc_fused) *enc_fused = false;
    if (p.Tq == 0) return ASTRA_OK;
    AttnEncode ae{};
    if (dtype == ASTRA_BF16) {
        int64_t total = (int64_t)ceil_div(p.Tq, kAttQ) * p.Hq;
        if (total > 0x7fffffff) return ASTRA_ERR_SHAPE;
        // short sequences with 64-wide heads: when 128-row query blocks would leave half of the compute units without a
        // workgroup, 64-row blocks whose tiles are dealt to four wavefronts per query group (half the iterations each)
        const bool four = head_dim == 64 && total <= kAttCus / 2;
        if (four) total = (int64_t)ceil_div(p.Tq, kAttQ / 2) * p.Hq;
        const bool vt = p.v_transposed != 0;
        const bool lost = p.valid_bits != nullptr;
        if (head_dim != 64 && head_dim != 128) return ASTRA_ERR_UNSUPPORTED;
        // the kernel forms byte offsets inside one head's tile source in 32 bits: rows of the transposed V buffers
        // (head_dim of them, ldv tokens each) and 64 key rows of H_kv * head_dim elements
        if (vt && (int64_t)max(p.ldv_loc, p.ldv_hat) * 2 * head_dim >= (1ll << 32)) return ASTRA_ERR_UNSUPPORTED;
        if ((int64_t)p.Hkv * head_dim * 2 * kAttKV >= (1ll << 32)) return ASTRA_ERR_UNSUPPORTED;
        // encodes offered by the caller ride in the launch's tail (128-wide heads on transposed V: the instantiations built)
        if (enc && enc_fused && n_enc >= 1 && n_enc <= 2 && head_dim == 128 && vt && total + kAttCus <= 0x7fffffff) {
            bool ok = true;
            int64_t items = 0;
            for (int j = 0; j < n_enc; ++j) {
                ok = ok && enc[j].n_tokens > 0 && vq_encode_fast_ok(enc[j].K, enc[j].dg);
                const int64_t n_tb = ceil_div(enc[j].n_tokens, kAttThreads / 2);
                ok = ok && n_tb * enc[j].G <= 0x3fffffff && enc[j].dg == enc[0].dg;
                items += n_tb * enc[j].G;
            }
            if (ok && items > 0) {
                ae.n_jobs = n_enc;
                for (int j = 0; j < n_enc; ++j) {
                    ae.job[j] = enc[j];
                    ae.job[j].n_tb = (int)ceil_div(enc[j].n_tokens, kAttThreads / 2);
                }
                ae.n_attn_wgs = (int)total;
                ae.n_enc_wgs = (int)std::min<int64_t>(items, kAttCus);
                for (int j = 0; j < n_enc; ++j) ae.job[j].n_wgs = ae.n_enc_wgs;
                *enc_fused = true;
            }
        }
        if (plan_only) return ASTRA_OK;
        if (ae.n_enc_wgs > 0) {
            if (lost) attn_bf16_kernel<128, true, true, 2, true><<<(int)total + ae.n_enc_wgs, kAttThreads, 0, s>>>(p, ae);
            else attn_bf16_kernel<128, true, false, 2, true><<<(int)total + ae.n_enc_wgs, kAttThreads, 0, s>>>(p, ae);
        } else if (head_dim == 128) {
            if (vt && lost) attn_bf16_kernel<128, true, true><<<(int)total, kAttThreads, 0, s>>>(p, ae);
            else if (vt) attn_bf16_kernel<128, true><<<(int)total, kAttThreads, 0, s>>>(p, ae);
            else if (lost) attn_bf16_kernel<128, false, true><<<(int)total, kAttThreads, 0, s>>>(p, ae);
            else attn_bf16_kernel<128, false><<<(int)total, kAttThreads, 0, s>>>(p, ae);
        } else if (four) {
            if (vt && lost) attn_bf16_kernel<64, true, true, 4><<<(int)total, kAttThreads, 0, s>>>(p, ae);
            else if (vt) attn_bf16_kernel<64, true, false, 4><<<(int)total, kAttThreads, 0, s>>>(p, ae);
            else if (lost) attn_bf16_kernel<64, false, true, 4><<<(int)total, kAttThreads, 0, s>>>(p, ae);
            else attn_bf16_kernel<64, false, false, 4><<<(int)total, kAttThreads, 0, s>>>(p, ae);
        } else if (head_dim == 64) {
            if (vt && lost) attn_bf16_kernel<64, true, true><<<(int)total, kAttThreads, 0, s>>>(p, ae);
            else if (vt) attn_bf16_kernel<64, true><<<(int)total, kAttThreads, 0, s>>>(p, ae);
            else if (lost) attn_bf16_kernel<64, false, true><<<(int)total, kAttThreads, 0, s>>>(p, ae);
            else attn_bf16_kernel<64, false><<<(int)total, kAttThreads, 0, s>>>(p, ae);
        } else {
            return ASTRA_ERR_UNSUPPORTED;
        }
    } else {
        if (head_dim > 256 || p.v_transposed) return ASTRA_ERR_UNSUPPORTED;
        const int64_t blocks = (int64_t)p.Hq * p.Tq;
        if (blocks > 0x7fffffff) return ASTRA_ERR_SHAPE;
        if (plan_only) return ASTRA_OK;
        switch ((head_dim + 63) / 64) {
            case 1: attn_f32_kernel<1><<<(int)blocks, 256, 0, s>>>(p, head_dim); break;
            case 2: attn_f32_kernel<2><<<(int)blocks, 256, 0, s>>>(p, head_dim); break;
            case 3: attn_f32_kernel<3><<<(int)blocks, 256, 0, s>>>(p, head_dim); break;
            default: attn_f32_kernel<4><<<(int)blocks, 256, 0, s>>>(p, head_dim); break;
        }
    }
    return launch_status();
}

}  // namespace astra
