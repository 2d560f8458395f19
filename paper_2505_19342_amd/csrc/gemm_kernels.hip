// Linear projections C[M,N] = A[M,K] . B[N,K]^T (+ bias) for the attention layer (the projections
// named under Eq. 1 of the paper): Q, K, V of the local rows, K-hat, V-hat of the rows rebuilt from
// codes, and the output projection.  Several problems run in one grouped launch; a problem may take
// its A rows straight from the codebook through the token codes (decode fused into the operand load).
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
};

__device__ __forceinline__ int find_problem(const GemmBatch& b, int tile) {
    int p = 0;
    while (p + 1 < b.n && tile >= b.tile_begin[p + 1]) ++p;
    return p;
}

// ------------------------------------------------------------------------------------------------
// bf16, matrix cores.  A workgroup of WM x WN wavefronts owns a BM x BN output tile; each wavefront
// owns a (BM/WM) x (BN/WN) sub-tile made of 32x32x16 MFMA tiles.  The contraction runs in steps of 64
// through double-buffered LDS: while the matrix cores work on tile kt, the registers hold tile kt+1
// (fetched one iteration earlier) on its way to the other LDS buffer, the loads of tile kt+2 are in
// flight and, for gathered A rows, the codes of tile kt+3 are being fetched.  LDS tiles are
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

// MLP: the instantiation carries the epilogues of the block's MLP (activation, gated product, residual add); the
// projection launches of the attention layer use the instantiation without them.
template <int BM, int BN, int WM, int WN, bool CODE16, bool ENC = false, bool MLP = false>
__global__ __launch_bounds__(64 * WM * WN) void gemm_nt_bf16_kernel(const GemmBatch batch) {
    constexpr int THREADS = 64 * WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;        // MFMA tiles per wavefront
    constexpr int RPP = THREADS / 8;                           // rows staged per pass
    constexpr int PA = BM / RPP, PB = BN / RPP;                // staging passes per thread
    __shared__ u32x4 lds_a[2][BM * kBK / 8];
    __shared__ u32x4 lds_b[2][BN * kBK / 8];

    int vt;
    if (ENC) {
        // The grid is the GEMM tiles plus batch.n_enc_wgs workgroups that encode the local rows (nothing in the
        // projections depends on the codes or the other way round): they fill compute units the tiles leave idle.
        // The encode reuses the operand buffers: its ring of codebook tiles is exactly lds_a, the norms sit in lds_b.
        static_assert(!ENC || (sizeof(lds_a) == sizeof(u32x4) * kEncBufs * kEncCbSlots && sizeof(lds_b) >= sizeof(f32x4) * kEncBufs * kEncCnSlots),
                      "encode ring must fit the operand buffers");
        const FusedId id = fused_id(blockIdx.x, gridDim.x - batch.n_enc_wgs, batch.n_enc_wgs);
        if (id.enc) {
            u32x4* cb = &lds_a[0][0];
            f32x4* cn = reinterpret_cast<f32x4*>(&lds_b[0][0]);
            const EncodeJob& job = batch.enc;
            vq_encode_fast_zero_lds<THREADS>(cb);
            __syncthreads();                               // zero fill done before any transfer lands
            const int n_items = job.G * job.n_tb;
            const int chunk = (n_items + batch.n_enc_wgs - 1) / batch.n_enc_wgs;     // consecutive items share the group
            const int hi = min((id.idx + 1) * chunk, n_items);
            for (int item = id.idx * chunk; item < hi; ++item) {
                if (job.code_bytes == 2) vq_encode_fast_body<THREADS, uint16_t>(job, item / job.n_tb, item % job.n_tb, cb, cn);
                else vq_encode_fast_body<THREADS, uint8_t>(job, item / job.n_tb, item % job.n_tb, cb, cn);
                __syncthreads();                           // all reads of this item's tiles done before the next item's transfers
            }
            return;
        }
        vt = id.idx;
    } else {
        vt = xcd_remap(blockIdx.x, gridDim.x);
    }
    const int pi = find_problem(batch, vt);
    const GemmProblem& P = batch.p[pi];
    const int tile = vt - batch.tile_begin[pi];
    const int tiles_m = batch.tiles_m[pi];
    const int tm = tile % tiles_m, tn = tile / tiles_m;
    const int m0 = tm * BM, n0 = tn * BN;
    const int M = P.M, N = P.N, K = P.K;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int i32 = lane & 31, h = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;
    const int kc = tid & 7, r0 = tid >> 3;      // staging: 16-byte piece kc of rows r0 + RPP * it

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
    const int a_step = gather ? 0 : kBK * 2;
    const uint32_t gmask = gather ? 0xffffffffu : 0u;                           // keeps the gathered offset, or zeroes it
    const char* __restrict__ b_base = (const char*)P.b;
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
        if (MLP && TN % 2 == 0 && P.c_mode == kCSwiGLU) {
            // tile row r of B -> weight row such that, in every wavefront, MFMA column tiles b < TN/2 hold gate rows and
            // tiles b + TN/2 the up rows of the same BN/WN/2 output columns: both factors of an output meet in one lane
            const int rr = r0 + RPP * it, Fh = N >> 1;
            const int wn_r = rr / (32 * TN), b_r = (rr % (32 * TN)) / 32, i_r = rr % 32;
            int col = n0 / 2 + wn_r * (16 * TN) + (b_r % (TN / 2)) * 32 + i_r;
            col = col < Fh ? col : Fh - 1;
            rb = (b_r >= TN / 2 ? Fh : 0) + col;
        }
        boff[it] = ((uint32_t)rb * (uint32_t)K + kc * 8) * 2u;
    }
    int k_code = kc * 8;              // contraction index of this thread's piece in the tile whose codes are fetched next
    int k_use = kc * 8;               // ... in the tile whose operand pieces are fetched next
    int code[PA];
    u32x4 ra[PA], rb[PB];

    auto load_codes = [&]() {
        const uint32_t g_ = __umulhi((uint32_t)k_code, magic) * (CODE16 ? 2u : 1u);
#pragma unroll
        for (int it = 0; it < PA; ++it) {
            if (CODE16) code[it] = *reinterpret_cast<const uint16_t*>(c_base + (coff[it] + g_));
            else code[it] = *reinterpret_cast<const uint8_t*>(c_base + (coff[it] + g_));
        }
        k_code += kBK;
    };
    auto load_tile = [&]() {
        const uint32_t g_ = __umulhi((uint32_t)k_use, magic);
        const uint32_t j_ = (uint32_t)k_use - g_ * (uint32_t)dg;
        const uint32_t gbase_ = g_ * (uint32_t)Kc;
#pragma unroll
        for (int it = 0; it < PA; ++it) {
            const uint32_t c_ = (uint32_t)(code[it] < Kc ? code[it] : Kc - 1);
            const uint32_t goff_ = ((gbase_ + c_) * (uint32_t)dg + j_) * 2u;
            ra[it] = *reinterpret_cast<const u32x4*>(a_base + ((goff_ & gmask) + aoff[it]));
        }
#pragma unroll
        for (int it = 0; it < PB; ++it) rb[it] = *reinterpret_cast<const u32x4*>(b_base + boff[it]);
        a_base += a_step;
        b_base += kBK * 2;
        k_use += kBK;
    };
    auto store_tile = [&](int buf_) {
#pragma unroll
        for (int it = 0; it < PA; ++it) {
            const int r_ = r0 + RPP * it;
            lds_a[buf_][r_ * 8 + (kc ^ swz(r_))] = ra[it];
        }
#pragma unroll
        for (int it = 0; it < PB; ++it) {
            const int r_ = r0 + RPP * it;
            lds_b[buf_][r_ * 8 + (kc ^ swz(r_))] = rb[it];
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // fragment rows
    int arow[TM], brow[TN];
#pragma unroll
    for (int a = 0; a < TM; ++a) arow[a] = wm * (BM / WM) + a * 32 + i32;
#pragma unroll
    for (int b = 0; b < TN; ++b) brow[b] = wn * (BN / WN) + b * 32 + i32;

    // ---- main loop.  One tile of 64 along the contraction is four MFMA steps of 16.  Per step a wavefront
    // issues TM*TN MFMAs on fragments it requested from LDS one step earlier (two fragment slots), and between those
    // MFMAs, in program order, the "side jobs" of the step: the TM+TN fragment reads of the next step and a slice of
    // the staging work (registers holding tile kt+1 -> other LDS buffer, refilled at once with the global loads of
    // tile kt+2).  Nothing else is needed to keep a single wavefront per SIMD busy: LDS and global latencies are
    // covered by the MFMAs issued meanwhile.  Staging is spread over steps 0..2; the workgroup barrier follows step 2,
    // after which step 3 may read the first fragments of tile kt+1 from the buffer just filled, and the buffer of
    // tile kt (all of whose fragments were requested before the barrier) is free for the next iteration's staging.
    const int n_kt = K / kBK;
    bf16x8 fa[2][TM], fb[2][TN];
    auto read_frag = [&](int buf_, int ks, int slot, int j) {
        if (j < TM) fa[slot][j] = __builtin_bit_cast(bf16x8, lds_a[buf_][arow[j] * 8 + ((2 * ks + h) ^ swz(arow[j]))]);
        else fb[slot][j - TM] = __builtin_bit_cast(bf16x8, lds_b[buf_][brow[j - TM] * 8 + ((2 * ks + h) ^ swz(brow[j - TM]))]);
    };
    constexpr int NR = TM + TN, NM = TM * TN;
    auto tile_steps = [&](int kt, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;       // steady state: tiles kt+1, kt+2 and codes kt+3 all exist
        const int buf = kt & 1;
        const bool st = FULL || kt + 1 < n_kt, ld = FULL || kt + 2 < n_kt;
        const uint32_t g_ = __umulhi((uint32_t)k_use, magic);
        const uint32_t j_ = (uint32_t)k_use - g_ * (uint32_t)dg;
        const uint32_t gbase_ = g_ * (uint32_t)Kc;
        auto stage_a = [&](int it) {
            const int r_ = r0 + RPP * it;
            if (st) lds_a[buf ^ 1][r_ * 8 + (kc ^ swz(r_))] = ra[it];
            if (ld) {
                const uint32_t c_ = (uint32_t)(code[it] < Kc ? code[it] : Kc - 1);
                const uint32_t goff_ = ((gbase_ + c_) * (uint32_t)dg + j_) * 2u;
                ra[it] = *reinterpret_cast<const u32x4*>(a_base + ((goff_ & gmask) + aoff[it]));
            }
        };
        auto stage_b = [&](int it) {
            const int r_ = r0 + RPP * it;
            if (st) lds_b[buf ^ 1][r_ * 8 + (kc ^ swz(r_))] = rb[it];
            if (ld) rb[it] = *reinterpret_cast<const u32x4*>(b_base + boff[it]);
        };
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            // side jobs of this step: NR fragment reads, then (steps 0..2) the staging slice
            const int a_lo = ks < 3 ? ks * PA / 3 : PA, a_hi = ks < 3 ? (ks + 1) * PA / 3 : PA;
            const int b_lo = ks < 3 ? ks * PB / 3 : PB, b_hi = ks < 3 ? (ks + 1) * PB / 3 : PB;
            const int nj = NR + (a_hi - a_lo) + (b_hi - b_lo);
            const bool rd = ks < 3 || st;                     // step 3 reads the next tile, if there is one
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int a = m / TN, b = m % TN;
                acc[a][b] = mfma_32x32x16(fa[cur][a], fb[cur][b], acc[a][b]);
#pragma unroll
                for (int j = m * nj / NM; j < (m + 1) * nj / NM; ++j) {
                    if (j < NR) {
                        if (rd) read_frag(ks < 3 ? buf : buf ^ 1, (ks + 1) & 3, nxt, j);
                    } else if (j - NR < a_hi - a_lo) {
                        stage_a(a_lo + j - NR);
                    } else {
                        stage_b(b_lo + j - NR - (a_hi - a_lo));
                    }
                }
                __builtin_amdgcn_sched_barrier(0);        // keep this order: the compiler would bunch the memory operations
            }
            if (ks == 2) __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
        }
        if (ld) {
            a_base += a_step;
            b_base += kBK * 2;
            k_use += kBK;
        }
        if (FULL || kt + 3 < n_kt) load_codes();
    };

    load_codes();                 // codes of tile 0
    load_tile();                  // tile 0
    if (n_kt > 1) load_codes();   // codes of tile 1
    store_tile(0);
    if (n_kt > 1) load_tile();    // tile 1
    if (n_kt > 2) load_codes();   // codes of tile 2
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NR; ++j) read_frag(0, 0, 0, j);
    int kt = 0;
    for (; kt + 3 < n_kt; ++kt) tile_steps(kt, std::true_type{});
    for (; kt < n_kt; ++kt) tile_steps(kt, std::false_type{});

    // epilogue.  acc[a][b][v] is C[m, n] with m = wave row base + 32a + acc_row(v, h), n = wave column base + 32b + lane % 32.
    const uint16_t* __restrict__ bias = (const uint16_t*)P.bias;
    if (MLP && P.c_mode == kCSwiGLU) {
        if constexpr (MLP && TN % 2 == 0) {
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
        }
        return;
    }
    const int act = MLP ? P.act : kActNone;
#pragma unroll
    for (int b = 0; b < TN; ++b) {
        const int n = n0 + wn * (BN / WN) + b * 32 + i32;
        if (n >= N) continue;
        const float bv = bias ? bf16_bits_to_f32(bias[n]) : 0.f;
        if (P.c_mode == kCTransposedV) {
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
        } else if (P.c_mode == kCF32) {
            float* C = (float*)P.c;                       // may be the residual itself: no restrict
            const float* R = MLP ? P.residual : nullptr;
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * (BM / WM) + a * 32 + acc_row(v, h);
                    if (m < M) {
                        const int64_t at = (int64_t)m * P.ldc + n;
                        const float r = apply_act<true>(acc[a][b][v] + bv, act);
                        C[at] = R ? r + R[at] : r;
                    }
                }
        } else {
            uint16_t* __restrict__ C = (uint16_t*)P.c;
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * (BM / WM) + a * 32 + acc_row(v, h);
                    if (m < M) C[(int64_t)m * P.ldc + n] = f32_to_bf16_bits(apply_act<true>(acc[a][b][v] + bv, act));
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
    const int tm = tile % batch.tiles_m[pi], tn = tile / batch.tiles_m[pi];
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
    float* C = (float*)P.c;                               // may be the residual itself: no restrict
    const float* __restrict__ bias = (const float*)P.bias;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n < N) {
                const int64_t at = (int64_t)m * P.ldc + n;
                const float r = apply_act<false>(acc[i][j] + (bias ? bias[n] : 0.f), P.act);
                C[at] = P.residual ? r + P.residual[at] : r;
            }
        }
    }
}

int g_gemm_force_cfg = -1;      // development override: 0 = 128x128 tiles, 1 = 256x256 tiles
extern const int g_gemm_problem_size = (int)sizeof(GemmProblem);   // lets a development harness detect a stale header

static int fill_batch(GemmBatch& batch, int dtype, const GemmProblem* problems, int n_problems, int bm, int bn, int* total_out) {
    int total = 0, n = 0;
    for (int i = 0; i < n_problems; ++i) {
        const GemmProblem& p = problems[i];
        if (p.M <= 0 || p.N <= 0) continue;
        if (p.K <= 0) return ASTRA_ERR_SHAPE;
        if (dtype == ASTRA_BF16) {
            // whole 64-wide contraction tiles; 16-byte operand pieces must not straddle rows or codewords
            if (p.K % kBK != 0 || (!p.codes && p.lda % 8 != 0) || (p.codes && p.dg % 8 != 0)) return ASTRA_ERR_UNSUPPORTED;
            if (p.c_mode == kCTransposedV && (p.ldc % 64 != 0 || p.ldc < p.M)) return ASTRA_ERR_SHAPE;
            if (p.c_mode == kCSwiGLU && (p.N % 2 != 0 || p.ldc < p.N / 2)) return ASTRA_ERR_SHAPE;
            if (p.c_mode != kCF32 && p.residual) return ASTRA_ERR_UNSUPPORTED;
            if ((p.c_mode == kCTransposedV || p.c_mode == kCSwiGLU) && p.act != kActNone) return ASTRA_ERR_UNSUPPORTED;
            // operands are addressed with 32-bit byte offsets from their base
            const int64_t lim = (int64_t)1 << 31;
            if ((int64_t)p.M * p.lda * 2 >= lim || (int64_t)p.N * p.K * 2 >= lim) return ASTRA_ERR_UNSUPPORTED;
            if (p.codes && ((int64_t)p.G * p.Kc * p.dg * 2 >= lim || (int64_t)p.M * p.G * 2 >= lim)) return ASTRA_ERR_UNSUPPORTED;
        } else if (p.c_mode != kCF32) {
            return ASTRA_ERR_UNSUPPORTED;
        }
        const int64_t tm = ceil_div(p.M, bm), tn = ceil_div(p.N, bn);
        const int64_t nt = tm * tn;
        if (nt + total > 0x7fffffff) return ASTRA_ERR_SHAPE;
        batch.p[n] = p;
        batch.tile_begin[n] = total;
        batch.tiles_m[n] = (int)tm;
        total += (int)nt;
        ++n;
    }
    batch.n = n;
    for (int i = n; i <= kMaxGemmProblems; ++i) batch.tile_begin[i] = total;
    *total_out = total;
    return ASTRA_OK;
}

int launch_gemm_batch(int dtype, const GemmProblem* problems, int n_problems, hipStream_t s, const EncodeJob* enc, bool* enc_fused,
                      bool plan_only) {
    if (enc_fused) *enc_fused = false;
    if (n_problems > kMaxGemmProblems) return ASTRA_ERR_UNSUPPORTED;
    GemmBatch batch{};
    int total = 0;
    if (dtype != ASTRA_BF16) {
        int rc = fill_batch(batch, dtype, problems, n_problems, kFM, kFN, &total);
        if (rc) return rc;
        if (total == 0 || plan_only) return ASTRA_OK;
        gemm_nt_f32_kernel<<<total, 256, 0, s>>>(batch);
        return launch_status();
    }
    bool code16 = false, mlp = false;
    for (int i = 0; i < n_problems; ++i) {
        if (problems[i].codes && problems[i].code_bytes == 2) code16 = true;
        if (problems[i].c_mode == kCSwiGLU || problems[i].act != kActNone || problems[i].residual) mlp = true;
    }
    if (mlp) {
        // the MLP's GEMMs and the residual-adding output projection: plain A rows, one problem per launch
        if (n_problems != 1 || problems[0].codes) return ASTRA_ERR_UNSUPPORTED;
        int rc = fill_batch(batch, dtype, problems, n_problems, 256, 256, &total);
        if (rc) return rc;
        if (total >= 128) {
            if (!plan_only) gemm_nt_bf16_kernel<256, 256, 2, 4, false, false, true><<<total, 512, 0, s>>>(batch);
            return plan_only ? ASTRA_OK : launch_status();
        }
        rc = fill_batch(batch, dtype, problems, n_problems, 128, 128, &total);
        if (rc) return rc;
        if (total == 0 || plan_only) return ASTRA_OK;
        gemm_nt_bf16_kernel<128, 128, 2, 2, false, false, true><<<total, 256, 0, s>>>(batch);
        return launch_status();
    }
    // Large tiles quarter the operand traffic per flop; use them once they still fill most of the chip.
    int rc = fill_batch(batch, dtype, problems, n_problems, 256, 256, &total);
    if (rc) return rc;
    bool big = total >= 128;
    if (g_gemm_force_cfg >= 0) big = g_gemm_force_cfg >= 1;
    // Fuse the encode into the launch when the tiles leave a good part of the last round of compute units idle.
    if (big && enc && enc_fused && g_gemm_force_cfg < 0 && vq_encode_fast_ok(enc->K, enc->dg) && enc->n_tokens > 0) {
        const int rem = total % kCus;
        const int E = rem == 0 ? 0 : ((kCus - rem) & ~7);
        const int64_t n_tb = ceil_div(enc->n_tokens, 256);
        if (E >= 8 && E <= kCus / 2 && n_tb * enc->G <= 0x7fffffff) {
            batch.n_enc_wgs = E;
            batch.enc = *enc;
            batch.enc.n_tb = (int)n_tb;
            batch.enc.n_wgs = E;
            *enc_fused = true;
            if (plan_only) return ASTRA_OK;
            if (code16) gemm_nt_bf16_kernel<256, 256, 2, 4, true, true><<<total + E, 512, 0, s>>>(batch);
            else gemm_nt_bf16_kernel<256, 256, 2, 4, false, true><<<total + E, 512, 0, s>>>(batch);
            return launch_status();
        }
    }
    if (plan_only) return ASTRA_OK;
    if (big && g_gemm_force_cfg == 2) {
        if (code16) gemm_nt_bf16_kernel<256, 256, 2, 2, true><<<total, 256, 0, s>>>(batch);
        else gemm_nt_bf16_kernel<256, 256, 2, 2, false><<<total, 256, 0, s>>>(batch);
        return launch_status();
    }
    if (big) {
        if (total == 0) return ASTRA_OK;
        if (code16) gemm_nt_bf16_kernel<256, 256, 2, 4, true><<<total, 512, 0, s>>>(batch);
        else gemm_nt_bf16_kernel<256, 256, 2, 4, false><<<total, 512, 0, s>>>(batch);
        return launch_status();
    }
    rc = fill_batch(batch, dtype, problems, n_problems, 128, 128, &total);
    if (rc) return rc;
    if (total == 0) return ASTRA_OK;
    if (code16) gemm_nt_bf16_kernel<128, 128, 2, 2, true><<<total, 256, 0, s>>>(batch);
    else gemm_nt_bf16_kernel<128, 128, 2, 2, false><<<total, 256, 0, s>>>(batch);
    return launch_status();
}

}  // namespace astra
