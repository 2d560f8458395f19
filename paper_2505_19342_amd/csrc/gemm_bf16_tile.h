// The bf16 matrix-core GEMM tile kernel C[M,N] = A[M,K] . B[N,K]^T shared by the attention layer's projection launches
// (paper: the projections named under Eq. 1) and by the MLP of the block around the layer (Sec. 3.1).
#pragma once
#include "common.h"
#include "vq_encode_body.h"

#include <type_traits>

namespace astra {

struct GemmBatch {
    int32_t n;
    int32_t tile_begin[kMaxGemmProblems + 1];
    int32_t tiles_m[kMaxGemmProblems];     // tiles along M of each problem (tile index = tn * tiles_m + tm)
    GemmProblem p[kMaxGemmProblems];
    int32_t n_enc_wgs;                     // fused launch: workgroups beyond the GEMM tiles that run the VQ encode
    EncodeJob enc;
    int32_t n_split, k_split;              // split contraction (one problem): the grid is n_split copies of the tiles, copy s
                                           // contracts k in [s * k_split, (s + 1) * k_split) into slice s of an fp32 buffer
};

__device__ __forceinline__ int find_problem(const GemmBatch& b, int tile) {
    int p = 0;
    while (p + 1 < b.n && tile >= b.tile_begin[p + 1]) ++p;
    return p;
}

// ------------------------------------------------------------------------------------------------
// bf16, matrix cores.  A workgroup of WM x WN wavefronts owns a BM x BN output tile; each wavefront
// owns a (BM/WM) x (BN/WN) sub-tile made of 32x32x16 MFMA tiles.  The contraction runs in steps of 64
// through double-buffered LDS.  Operand tiles travel from memory straight into LDS (one wavefront instruction
// fills 64 consecutive 16-byte slots, nothing passes through registers): while the matrix cores work on tile kt
// out of one buffer, tile kt+1 has landed in the other, tile kt+2 is sent into the first as soon as the barrier
// of iteration kt has passed and, for gathered A rows, the codes of tile kt+3 are being fetched.  LDS tiles are
// [rows][8 pieces of 8 bf16]; piece p of row r sits at p ^ ((r >> 1) & 7): rows are 128 bytes, the
// LDS has 64 four-byte banks, so the 16-byte fragment reads of 16 consecutive rows touch every bank once.
//
// Workgroup -> tile mapping: hardware hands consecutive workgroup ids to the 8 XCDs round-robin, each
// with its own L2.  Ids are remapped so that every XCD gets one contiguous range of tiles, walked with
// the M index fastest: the tiles an XCD runs at the same time share their weight (B) panel and draw
// their A panels from a few rows, so most operand traffic is served by that XCD's L2.
// ------------------------------------------------------------------------------------------------
constexpr int kBK = 64;
constexpr int kXcds = 8;
constexpr int kCus = 256;         // compute units of the device the launch shapes are chosen for

__device__ __forceinline__ int xcd_remap(int wg, int total) {
    const int q = total / kXcds, r = total % kXcds;
    const int xcd = wg % kXcds, slot = wg / kXcds;
    return xcd < r ? xcd * (q + 1) + slot : r * (q + 1) + (xcd - r) * q + slot;
}

__device__ __forceinline__ int swz(int r) { return (r >> 1) & 7; }

// Activations of the position-wise MLP that follows the attention layer inside a block (paper Sec. 3.1), applied in
// the epilogue.  x * sigmoid(2u) is 0.5 x (1 + tanh u).  FAST uses the hardware exponential (results are rounded to
// bf16 afterwards); otherwise the library routines.
template <bool FAST>
__device__ __forceinline__ float silu(float v) { return v / (1.f + (FAST ? __expf(-v) : expf(-v))); }
template <bool FAST>
__device__ __forceinline__ float apply_act(float v, int act) {
    if (act == kActGeluTanh) {
        const float u = 0.7978845608028654f * (v + 0.044715f * v * v * v);
        return FAST ? v / (1.f + __expf(-2.f * u)) : 0.5f * v * (1.f + tanhf(u));
    }
    if (act == kActGeluErf) return 0.5f * v * (1.f + erff(v * 0.7071067811865476f));
    return v;
}

// Fused launch of T GEMM tiles and E encode workgroups (E a multiple of 8): every XCD gets a contiguous range of
// tiles, as with xcd_remap, followed by E/8 encode workgroups, so both kinds of work are spread over all XCDs.
struct FusedId {
    bool enc;
    int idx;
};
__device__ __forceinline__ FusedId fused_id(int wg, int T, int E) {
    const int xcd = wg % kXcds, slot = wg / kXcds;
    const int tq = T / kXcds, tr = T % kXcds;
    const int t_x = tq + (xcd < tr ? 1 : 0);
    if (slot < t_x) return {false, xcd * tq + (xcd < tr ? xcd : tr) + slot};
    return {true, xcd * (E / kXcds) + slot - t_x};
}

// position of token offset o (0..15) inside a 16-token block of the transposed-V layout: the 8 tokens
// one half-wave holds of an MFMA accumulator column ({4h..4h+3} and {8+4h..8+4h+3}) become contiguous,
// which is also the order the attention kernel's P^T operand keeps its 16 keys in.
__device__ __forceinline__ int vt_pos(int o) { return 8 * ((o >> 2) & 1) + (o & 3) + 4 * (o >> 3); }

int launch_gemm_mlp(int epi, bool big, const GemmBatch& batch, int grid, hipStream_t s);
int launch_gemm_mlp_small(int epi, const GemmBatch& batch, int grid, hipStream_t s);
int launch_split_reduce(const float* part, int n_split, const GemmProblem& p, hipStream_t s);
int gemm_split_factor(int dtype, int64_t M, int64_t N, int64_t K);

// EPI selects the epilogue at compile time.  kEpiLayer is the attention layer's: the store follows the problem's c_mode
// (bf16, fp32, transposed V).  The others belong to the block around the layer (one plain-A problem per launch) and each
// carries exactly one form, so that the tail of a launch that runs as a single round of workgroups stays short:
//   kEpiResidualF32  fp32 store of A.B^T + bias, accumulation started from `residual` when it is set
//   kEpiSplit        the contraction slice batch.k_split of copy blockIdx / tiles, raw fp32 partial sums
//   kEpiGeluTanh / kEpiGeluErf   bf16 store of gelu(A.B^T + bias)
//   kEpiSwiGLU       bf16 store of silu(A.gate^T + b_g) * (A.up^T + b_u)
enum { kEpiLayer = 0, kEpiResidualF32 = 1, kEpiSplit = 2, kEpiGeluTanh = 3, kEpiGeluErf = 4, kEpiSwiGLU = 5 };

// KS = 2: two groups of WM x WN wavefronts work on the same output tile, group g contracting the k ranges
// [128 t + 64 g, 128 t + 64 g + 64), each with its own operand buffers and the full loop below; their accumulators are
// added through LDS at the end.  A small tile then keeps its 64 x 64 wave tiles (1 KiB of LDS reads per MFMA) and still
// has two wavefronts per SIMD to hide each other's staging.
template <int BM, int BN, int WM, int WN, bool CODE16, bool ENC = false, int EPI = kEpiLayer, int KS = 1>
__global__ __launch_bounds__(64 * WM * WN * KS) void gemm_nt_bf16_kernel(const GemmBatch batch) {
    constexpr int THREADS = 64 * WM * WN;                      // threads of one group
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;        // MFMA tiles per wavefront
    constexpr int RPP = THREADS / 8;                           // rows staged per pass
    constexpr int PA = BM / RPP, PB = BN / RPP;                // staging passes per thread
    static_assert(KS == 1 || KS == 2, "one or two contraction groups");
    static_assert(RPP % 16 == 0, "direct transfers: the row swizzle has to be periodic in the pass stride");
    __shared__ u32x4 lds_a[2 * KS][BM * kBK / 8];              // [2 * group + buffer]
    __shared__ u32x4 lds_b[2 * KS][BN * kBK / 8];

    int vt;
    if (ENC) {
        // The grid is the GEMM tiles plus batch.n_enc_wgs workgroups that encode the local rows (nothing in the
        // projections depends on the codes or the other way round): they fill compute units the tiles leave idle.
        // The encode reuses the operand buffers: its ring of codebook tiles is exactly the one of 256 rows, the norms sit in the other.
        constexpr size_t kRing = sizeof(u32x4) * kEncBufs * kEncCbSlots, kNorms = sizeof(f32x4) * kEncBufs * kEncCnSlots;
        constexpr bool RING_IN_A = sizeof(lds_a) == kRing;
        static_assert(!ENC || (RING_IN_A && sizeof(lds_b) >= kNorms) || (sizeof(lds_b) == kRing && sizeof(lds_a) >= kNorms),
                      "encode ring must be one of the operand buffers");
        const FusedId id = fused_id(blockIdx.x, gridDim.x - batch.n_enc_wgs, batch.n_enc_wgs);
        if (id.enc) {
            u32x4* cb = RING_IN_A ? &lds_a[0][0] : &lds_b[0][0];
            f32x4* cn = reinterpret_cast<f32x4*>(RING_IN_A ? &lds_b[0][0] : &lds_a[0][0]);
            const EncodeJob& job = batch.enc;
            constexpr int WG_THREADS = THREADS * KS;          // the encode uses every wavefront of the workgroup
            if (vq_encode_fast_needs_zero(job.dg)) {
                vq_encode_fast_zero_lds<WG_THREADS>(cb);
                __syncthreads();                           // zero fill done before any transfer lands
            }
            const int n_items = job.G * job.n_tb;
            const int chunk = (n_items + batch.n_enc_wgs - 1) / batch.n_enc_wgs;     // consecutive items share the group
            const int hi = min((id.idx + 1) * chunk, n_items);
            for (int item = id.idx * chunk; item < hi; ++item) {
                vq_encode_fast_body<WG_THREADS>(job, item / job.n_tb, item % job.n_tb, cb, cn);
                __syncthreads();                           // all reads of this item's tiles done before the next item's transfers
            }
            return;
        }
        vt = id.idx;
    } else {
        vt = xcd_remap(blockIdx.x, gridDim.x);
    }
    int split = 0;
    if (EPI == kEpiSplit) {
        const int tiles = batch.tile_begin[batch.n];
        split = vt / tiles;
        vt -= split * tiles;
    }
    const int pi = find_problem(batch, vt);
    const GemmProblem& P = batch.p[pi];
    const int tile = vt - batch.tile_begin[pi];
    const int tiles_m = batch.tiles_m[pi];
    const int tm = tile % tiles_m, tn = tile / tiles_m;
    const int m0 = tm * BM, n0 = tn * BN;
    const int M = P.M, N = P.N, K = P.K;

    const int kgrp = KS == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x / THREADS);      // contraction group (wave-uniform)
    const int kg2 = 2 * kgrp;
    const int tid = KS == 1 ? (int)threadIdx.x : (int)threadIdx.x % THREADS;
    const int lane = tid & 63, wave = tid >> 6;
    const int i32 = lane & 31, h = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;
    const int r0 = tid >> 3;                    // staging: 16-byte piece kc of rows r0 + RPP * it
    // With direct global -> LDS transfers a lane's LDS slot is fixed by its lane number (slot tid & 7 of its row), so the
    // swizzle moves to the global side: the lane fetches the piece that belongs into its slot.
    const int kc = (tid & 7) ^ swz(r0);

    // One straight-line loader serves plain and gathered A rows.  For gathered rows the piece at
    // contraction index k lies in group g = k / dg at offset j = k - g*dg of codeword codes[row, g];
    // for plain rows the code load is a harmless read of the first bytes of A and the gathered offset is
    // discarded by a select.  k / dg is a multiply-high by ceil(2^32 / dg), exact for k, dg < 2^16.
    // Addresses are a wave-uniform base (scalar registers, advanced once per tile) plus a 32-bit byte
    // offset per thread, which keeps the per-row state to one register.
    const bool gather = P.codes != nullptr;
    const int dg = gather ? P.dg : 1, Kc = gather ? P.Kc : 1, G = gather ? P.G : 0;
    const uint32_t magic = gather ? (uint32_t)(0x100000000ull / (uint32_t)dg) + 1u : 0u;
    const char* __restrict__ a_base = (const char*)(gather ? P.codebook : P.a);   // plain A advances 128 bytes per tile
    const int a_step = gather ? 0 : kBK * 2 * KS;
    const uint32_t gmask = gather ? 0xffffffffu : 0u;                           // keeps the gathered offset, or zeroes it
    const char* __restrict__ b_base = (const char*)P.b;
    if (KS > 1) {                              // this group's first 64 of every 128 along the contraction
        if (!gather) a_base += kgrp * kBK * 2;
        b_base += kgrp * kBK * 2;
    }
    if (EPI == kEpiSplit) {                    // plain A only: both operands start at this copy's slice of the contraction
        a_base += (int64_t)split * batch.k_split * 2;
        b_base += (int64_t)split * batch.k_split * 2;
    }
    const char* __restrict__ c_base = (const char*)(gather ? P.codes : P.a);
    uint32_t aoff[PA], coff[PA], boff[PB];
#pragma unroll
    for (int it = 0; it < PA; ++it) {
        int ra = m0 + r0 + RPP * it;
        ra = ra < M ? ra : M - 1;
        aoff[it] = gather ? 0u : ((uint32_t)ra * (uint32_t)P.lda + kc * 8) * 2u;
        coff[it] = (uint32_t)ra * (uint32_t)G * (CODE16 ? 2u : 1u);
    }
#pragma unroll
    for (int it = 0; it < PB; ++it) {
        int rb = n0 + r0 + RPP * it;
        rb = rb < N ? rb : N - 1;
        if (EPI == kEpiSwiGLU) {
            // tile row r of B -> weight row such that, in every wavefront, MFMA column tiles b < TN/2 hold gate rows and
            // tiles b + TN/2 the up rows of the same BN/WN/2 output columns: both factors of an output meet in one lane
            const int rr = r0 + RPP * it, Fh = N >> 1;
            const int wn_r = rr / (32 * TN), b_r = (rr % (32 * TN)) / 32, i_r = rr % 32;
            int col = n0 / 2 + wn_r * (16 * TN) + (b_r % (TN / 2)) * 32 + i_r;
            col = col < Fh ? col : Fh - 1;
            rb = (b_r >= TN / 2 ? Fh : 0) + col;
        }
        boff[it] = ((uint32_t)rb * (uint32_t)(P.ldb ? P.ldb : K) + kc * 8) * 2u;
    }
    int k_code = kc * 8 + kgrp * kBK; // contraction index of this thread's piece in the tile whose codes are fetched next
    int k_use = kc * 8 + kgrp * kBK;  // ... in the tile whose operand pieces are fetched next
    int code[PA];

    auto load_codes = [&]() {
        const uint32_t g_ = __umulhi((uint32_t)k_code, magic) * (CODE16 ? 2u : 1u);
#pragma unroll
        for (int it = 0; it < PA; ++it) {
            if (CODE16) code[it] = *reinterpret_cast<const uint16_t*>(c_base + (coff[it] + g_));
            else code[it] = *reinterpret_cast<const uint8_t*>(c_base + (coff[it] + g_));
        }
        k_code += kBK * KS;
    };
    // direct transfer of the tile at k_use into LDS buffer buf_: the lanes of a wavefront fill 64 consecutive slots
    // (8 rows of 8 pieces), nothing passes through registers; pass it_ of the A rows, then of the B rows
    const uint32_t wave_rows = (uint32_t)__builtin_amdgcn_readfirstlane(8 * (tid >> 6));
    auto dma_piece = [&](int buf_, int j_it) {
        if (j_it < PA) {
            const int it = j_it;
            const uint32_t g_ = __umulhi((uint32_t)k_use, magic);
            const uint32_t j_ = (uint32_t)k_use - g_ * (uint32_t)dg;
            int code_here = code[it];
            asm volatile("" : "+v"(code_here));      // the code is first touched here: an earlier use would wait for the transfers issued before its load
            const uint32_t c_ = (uint32_t)(code_here < Kc ? code_here : Kc - 1);
            const uint32_t goff_ = ((g_ * (uint32_t)Kc + c_) * (uint32_t)dg + j_) * 2u;
            dma_global_to_lds_16(a_base, (goff_ & gmask) + aoff[it], lds_byte_addr(&lds_a[kg2 + buf_][(wave_rows + RPP * it) * 8]));
        } else {
            const int it = j_it - PA;
            dma_global_to_lds_16(b_base, boff[it], lds_byte_addr(&lds_b[kg2 + buf_][(wave_rows + RPP * it) * 8]));
        }
    };
    auto dma_advance = [&]() {
        a_base += a_step;
        b_base += kBK * 2 * KS;
        k_use += kBK * KS;
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    if (EPI == kEpiResidualF32 && P.residual != nullptr && kgrp == 0) {
        // The residual is where the accumulation starts: its loads are issued here, all at once, and land while the first
        // operand tiles are fetched.  (Added in the epilogue, every load would be a round trip to memory in front of a store.)
        // Rows and columns beyond the problem are clamped: those accumulators are never stored.
        const char* __restrict__ R = (const char*)P.residual;
        const uint32_t ldc = (uint32_t)P.ldc;
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int n = min(n0 + wn * (BN / WN) + b * 32 + i32, N - 1);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = min(m0 + wm * (BM / WM) + a * 32 + acc_row(v, h), M - 1);
                    acc[a][b][v] = *reinterpret_cast<const float*>(R + ((uint32_t)m * ldc + (uint32_t)n) * 4u);
                }
        }
    }

    // fragment rows
    int arow[TM], brow[TN];
#pragma unroll
    for (int a = 0; a < TM; ++a) arow[a] = wm * (BM / WM) + a * 32 + i32;
#pragma unroll
    for (int b = 0; b < TN; ++b) brow[b] = wn * (BN / WN) + b * 32 + i32;

    // ---- main loop.  One tile of 64 along the contraction is four MFMA steps of 16.  Per step a wavefront
    // issues TM*TN MFMAs on fragments it requested from LDS one step earlier (two fragment slots), and between those
    // MFMAs, in program order, the "side jobs" of the step: the TM+TN fragment reads of the next step and, in step 3,
    // the transfers of tile kt+2.  LDS and global latencies are covered by the MFMAs issued meanwhile.  The workgroup
    // barrier follows step 2, after which step 3 may read the first fragments of tile kt+1 from the other buffer, and
    // the buffer of tile kt (all of whose fragments were requested before the barrier) is free for the transfers.
    const int n_kt = (EPI == kEpiSplit ? batch.k_split : K) / (kBK * KS);
    bf16x8 fa[2][TM], fb[2][TN];
    auto read_frag = [&](int buf_, int ks, int slot, int j) {
        if (j < TM) fa[slot][j] = __builtin_bit_cast(bf16x8, lds_a[kg2 + buf_][arow[j] * 8 + ((2 * ks + h) ^ swz(arow[j]))]);
        else fb[slot][j - TM] = __builtin_bit_cast(bf16x8, lds_b[kg2 + buf_][brow[j - TM] * 8 + ((2 * ks + h) ^ swz(brow[j - TM]))]);
    };
    constexpr int NR = TM + TN, NM = TM * TN;
    {
        // Tiles go from memory straight into LDS.  Buffer kt & 1 is free once every wavefront has passed the barrier of
        // iteration kt (all reads of tile kt were requested and awaited before it): tile kt + 2 is sent there during step 3
        // of iteration kt and has until the wait in front of the barrier of iteration kt + 1 to land.
        // buf_tag: std::integral_constant<int, kt & 1> makes the buffer static (LDS addresses become immediates; steady
        // state, where tiles kt + 1, kt + 2 and the codes of kt + 3 all exist), std::integral_constant<int, -1> reads it from kt
        // (the last few tiles, with the run-time guards)
        auto tile_steps_dma = [&](int kt, auto buf_tag) {
            constexpr bool FULL = decltype(buf_tag)::value >= 0;
            const int buf = FULL ? decltype(buf_tag)::value : (kt & 1);
            const bool nx = FULL || kt + 1 < n_kt, nx2 = FULL || kt + 2 < n_kt;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int cur = ks & 1, nxt = cur ^ 1;
                const int nd = ks == 3 ? PA + PB : 0;
                const int nj = NR + nd;
                const bool rd = ks < 3 || nx;
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    const int a = m / TN, b = m % TN;
                    acc[a][b] = mfma_32x32x16(fa[cur][a], fb[cur][b], acc[a][b]);
#pragma unroll
                    for (int j = m * nj / NM; j < (m + 1) * nj / NM; ++j) {
                        if (j < NR) {
                            if (rd) read_frag(ks < 3 ? buf : buf ^ 1, (ks + 1) & 3, nxt, j);
                        } else if (nx2) {
                            dma_piece(buf, j - NR);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (ks == 2) {
                    wait_vmem_all();          // this wavefront's transfers of tile kt + 1 have landed
                    __syncthreads();
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (nx2) dma_advance();
            if (FULL || kt + 3 < n_kt) load_codes();
        };
        load_codes();                 // codes of tile 0
#pragma unroll
        for (int j = 0; j < PA + PB; ++j) dma_piece(0, j);
        dma_advance();
        if (n_kt > 1) {
            load_codes();             // codes of tile 1
#pragma unroll
            for (int j = 0; j < PA + PB; ++j) dma_piece(1, j);
            dma_advance();
        }
        if (n_kt > 2) load_codes();   // codes of tile 2
        wait_vmem_all();
        __syncthreads();
#pragma unroll
        for (int j = 0; j < NR; ++j) read_frag(0, 0, 0, j);
        int kt = 0;
        for (; kt + 4 < n_kt; kt += 2) {
            tile_steps_dma(kt, std::integral_constant<int, 0>{});
            tile_steps_dma(kt + 1, std::integral_constant<int, 1>{});
        }
        for (; kt < n_kt; ++kt) tile_steps_dma(kt, std::integral_constant<int, -1>{});
    }

    if constexpr (KS == 2) {
        // the second group hands its accumulators over through the operand buffers (all fragment reads are done)
        static_assert(KS == 1 || sizeof(lds_a) >= sizeof(float) * BM * BN, "accumulator exchange fits the A buffers");
        float* xch = reinterpret_cast<float*>(&lds_a[0][0]);
        __syncthreads();
        if (kgrp == 1) {
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) xch[(((wave * TM + a) * TN + b) * 16 + v) * 64 + lane] = acc[a][b][v];
        }
        __syncthreads();
        if (kgrp == 1) return;
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][v] += xch[(((wave * TM + a) * TN + b) * 16 + v) * 64 + lane];
    }

    // epilogue.  acc[a][b][v] is C[m, n] with m = wave row base + 32a + acc_row(v, h), n = wave column base + 32b + lane % 32.
    const uint16_t* __restrict__ bias = (const uint16_t*)P.bias;
    if constexpr (EPI == kEpiSplit) {
        // partial sums: slice `split` of the fp32 buffer, [M, N] dense; bias and residual are added by the reduction
        float* __restrict__ C = (float*)P.c + (int64_t)split * M * N;
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int n = n0 + wn * (BN / WN) + b * 32 + i32;
            if (n >= N) continue;
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * (BM / WM) + a * 32 + acc_row(v, h);
                    if (m < M) C[(int64_t)m * N + n] = acc[a][b][v];
                }
        }
    } else if constexpr (EPI == kEpiSwiGLU) {
        static_assert(EPI != kEpiSwiGLU || TN % 2 == 0, "gate and up tiles pair up inside a wavefront");
        const int Fh = N >> 1;
        uint16_t* __restrict__ C = (uint16_t*)P.c;
#pragma unroll
        for (int b = 0; b < TN / 2; ++b) {
            const int col = n0 / 2 + wn * (16 * TN) + b * 32 + i32;
            if (col >= Fh) continue;
            const float bg = bias ? bf16_bits_to_f32(bias[col]) : 0.f, bu = bias ? bf16_bits_to_f32(bias[Fh + col]) : 0.f;
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * (BM / WM) + a * 32 + acc_row(v, h);
                    if (m < M) C[(int64_t)m * P.ldc + col] = f32_to_bf16_bits(silu<true>(acc[a][b][v] + bg) * (acc[a][b + TN / 2][v] + bu));
                }
        }
    } else {
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int n = n0 + wn * (BN / WN) + b * 32 + i32;
            if (n >= N) continue;
            const float bv = bias ? bf16_bits_to_f32(bias[n]) : 0.f;
            if (EPI == kEpiLayer && P.c_mode == kCTransposedV) {
                // C^T with tokens permuted inside 16-token blocks; P.ldc is the padded token count.  Rows
                // m >= M of the last tile are finite copies of row M-1 (clamped loads) and are written too,
                // so the padding never holds uninitialised bits.
                uint16_t* __restrict__ C = (uint16_t*)P.c + (int64_t)n * P.ldc;
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int blk = 0; blk < 2; ++blk) {
                        const int mb = m0 + wm * (BM / WM) + a * 32 + 16 * blk;
                        if (mb < P.ldc) {
                            u32x4 w;
                            w.x = pack_bf16x2(acc[a][b][8 * blk + 0] + bv, acc[a][b][8 * blk + 1] + bv);
                            w.y = pack_bf16x2(acc[a][b][8 * blk + 2] + bv, acc[a][b][8 * blk + 3] + bv);
                            w.z = pack_bf16x2(acc[a][b][8 * blk + 4] + bv, acc[a][b][8 * blk + 5] + bv);
                            w.w = pack_bf16x2(acc[a][b][8 * blk + 6] + bv, acc[a][b][8 * blk + 7] + bv);
                            *reinterpret_cast<u32x4*>(C + mb + 8 * h) = w;
                        }
                    }
            } else if (EPI == kEpiResidualF32 || (EPI == kEpiLayer && P.c_mode == kCF32)) {
                float* C = (float*)P.c;                       // may be the residual itself (already inside acc): no restrict
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int m = m0 + wm * (BM / WM) + a * 32 + acc_row(v, h);
                        if (m < M) C[(int64_t)m * P.ldc + n] = acc[a][b][v] + bv;
                    }
            } else {
                constexpr int ACT = EPI == kEpiGeluTanh ? kActGeluTanh : EPI == kEpiGeluErf ? kActGeluErf : kActNone;
                uint16_t* __restrict__ C = (uint16_t*)P.c;
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int m = m0 + wm * (BM / WM) + a * 32 + acc_row(v, h);
                        if (m < M) C[(int64_t)m * P.ldc + n] = f32_to_bf16_bits(apply_act<true>(acc[a][b][v] + bv, ACT));
                    }
            }
        }
    }
}

}  // namespace astra
