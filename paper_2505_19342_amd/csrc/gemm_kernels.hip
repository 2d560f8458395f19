// Linear projections C[M,N] = A[M,K] . B[N,K]^T (+ bias) for the attention layer (the projections
// named under Eq. 1 of the paper): Q, K, V of the local rows, K-hat, V-hat of the rows rebuilt from
// codes, and the output projection.  Several problems run in one grouped launch; a problem may take
// its A rows straight from the codebook through the token codes (decode fused into the operand load).
// This file holds the layer's instantiations of the bf16 tile kernel, the fp32 kernel and the launcher;
// the instantiations for the MLP of the surrounding block are compiled in gemm_mlp_kernels.hip.
#include "gemm_bf16_tile.h"

namespace astra {

// ------------------------------------------------------------------------------------------------
// fp32, vector ALU: 64x64 output tile, 256 threads x (4x4) outputs, contraction in steps of 16 through
// LDS.  Used for the small fp32 configuration; sums in ascending k with fused multiply-add.
// ------------------------------------------------------------------------------------------------
constexpr int kFK = 64;

// TILE x TILE outputs per workgroup (64, or 32 for launches that would leave most of the chip without a workgroup),
// TILE / 16 x TILE / 16 per thread
template <int TILE>
__global__ __launch_bounds__(256) void gemm_nt_f32_kernel(const GemmBatch batch) {
    constexpr int kFM = TILE, kFN = TILE, RT = TILE / 16;
    constexpr int kFL = TILE / 4;     // consecutive k one thread stages per row: TILE rows x 64 k over 256 threads
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
    // staging: thread loads kFL consecutive k of one row
    const int lr = tid / (kFK / kFL), lk = (tid % (kFK / kFL)) * kFL;
    const int am = m0 + lr < M ? m0 + lr : M - 1;
    const int bn = n0 + lr < N ? n0 + lr : N - 1;

    // the values of the next step are fetched into registers while the current step is multiplied.  No load is guarded (a
    // guarded load compiles to a branch with a wait of its own, 32 of them in a row per step): addresses are clamped into
    // the row and values beyond the contraction replaced by zeros afterwards; four consecutive k are one 16-byte load
    // when every row start and the group length allow it.
    float av[kFL], bv[kFL];
    const int64_t ldb = P.ldb ? P.ldb : K;
    const bool vec = K % 4 == 0 && P.lda % 4 == 0 && ldb % 4 == 0 && (!gather || P.dg % 4 == 0) &&
                     (reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(CB)) % 16 == 0;
    auto a_ptr = [&](int k) -> const float* {           // address of element (am, k), k < K
        if (!gather) return A + (int64_t)am * P.lda + k;
        const int g = k / P.dg, jj = k - g * P.dg;
        int code;
        if (P.code_bytes == 1) code = ((const uint8_t*)P.codes)[(int64_t)am * P.G + g];
        else code = ((const uint16_t*)P.codes)[(int64_t)am * P.G + g];
        code = code < P.Kc ? code : P.Kc - 1;
        return CB + ((int64_t)g * P.Kc + code) * P.dg + jj;
    };
    auto fetch = [&](int k0) {
        if (vec) {
#pragma unroll
            for (int j = 0; j < kFL; j += 4) {
                const int k = k0 + lk + j;
                const int kc = k < K ? k : K - 4;
                const float4 a4 = *reinterpret_cast<const float4*>(a_ptr(kc));
                const float4 b4 = *reinterpret_cast<const float4*>(B + (int64_t)bn * ldb + kc);
                const bool in = k < K;
                av[j] = in ? a4.x : 0.f; av[j + 1] = in ? a4.y : 0.f; av[j + 2] = in ? a4.z : 0.f; av[j + 3] = in ? a4.w : 0.f;
                bv[j] = in ? b4.x : 0.f; bv[j + 1] = in ? b4.y : 0.f; bv[j + 2] = in ? b4.z : 0.f; bv[j + 3] = in ? b4.w : 0.f;
            }
        } else {
#pragma unroll
            for (int j = 0; j < kFL; ++j) {
                const int k = k0 + lk + j;
                const int kc = k < K ? k : K - 1;
                const float a1 = *a_ptr(kc), b1 = B[(int64_t)bn * ldb + kc];
                av[j] = k < K ? a1 : 0.f;
                bv[j] = k < K ? b1 : 0.f;
            }
        }
    };

    float acc[RT][RT] = {};
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += kFK) {
#pragma unroll
        for (int j = 0; j < kFL; ++j) {
            sa[lk + j][lr] = av[j];
            sb[lk + j][lr] = bv[j];
        }
        __syncthreads();
        if (k0 + kFK < K) fetch(k0 + kFK);
#pragma unroll
        for (int k = 0; k < kFK; ++k) {
            float a[RT], b[RT];
#pragma unroll
            for (int i = 0; i < RT; ++i) { a[i] = sa[k][ty * RT + i]; b[i] = sb[k][tx * RT + i]; }
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int j = 0; j < RT; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    float* C = (float*)P.c;                               // may be the residual itself: no restrict
    const float* __restrict__ bias = (const float*)P.bias;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        const int m = m0 + ty * RT + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < RT; ++j) {
            const int n = n0 + tx * RT + j;
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
            const int64_t lim = (int64_t)1 << 31;
            // whole 64-wide contraction tiles; 16-byte operand pieces must not straddle rows or codewords
            if (p.K % kBK != 0 || (!p.codes && p.lda % 8 != 0) || (p.codes && p.dg % 8 != 0)) return ASTRA_ERR_UNSUPPORTED;
            if (p.c_mode == kCTransposedV && (p.ldc % 64 != 0 || p.ldc < p.M)) return ASTRA_ERR_SHAPE;
            if (p.c_mode == kCSwiGLU && (p.N % 2 != 0 || p.ldc < p.N / 2)) return ASTRA_ERR_SHAPE;
            if (p.residual && (p.c_mode != kCF32 || p.act != kActNone || (int64_t)p.M * p.ldc * 4 >= lim)) return ASTRA_ERR_UNSUPPORTED;
            if ((p.c_mode == kCTransposedV || p.c_mode == kCSwiGLU) && p.act != kActNone) return ASTRA_ERR_UNSUPPORTED;
            // operands are addressed with 32-bit byte offsets from their base
            if (p.ldb != 0 && (p.ldb < p.K || p.ldb % 8 != 0)) return ASTRA_ERR_UNSUPPORTED;
            if ((int64_t)p.M * p.lda * 2 >= lim || (int64_t)p.N * (p.ldb ? p.ldb : p.K) * 2 >= lim) return ASTRA_ERR_UNSUPPORTED;
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

// Tiles of a set of problems at a tile shape (0 when a problem is rejected: the caller's own pass reports the error).
static int64_t count_tiles(const GemmProblem* problems, int n_problems, int bm, int bn) {
    int64_t t = 0;
    for (int i = 0; i < n_problems; ++i)
        if (problems[i].M > 0 && problems[i].N > 0) t += ceil_div(problems[i].M, bm) * ceil_div(problems[i].N, bn);
    return t;
}

// Rough duration (us) of one bf16 projection launch under the shape rules of launch_gemm_batch: rounds of 256 x 256 tiles
// (about 105 us per 4096 of contraction), one round of 128 x 256 tiles (70), or 128 x 128 tiles (48 for a single round of
// one workgroup per unit, 80 per round of two per unit).  Used only to compare ways of cutting a launch in two.
static double estimate_launch_us(const GemmProblem* problems, int n_problems) {
    int k_max = 0;
    for (int i = 0; i < n_problems; ++i) k_max = problems[i].K > k_max ? problems[i].K : k_max;
    const double kf = k_max / 4096.0;
    const int64_t big = count_tiles(problems, n_problems, 256, 256);
    if (big == 0) return 0.0;
    if (big > 128) return (double)ceil_div(big, (int64_t)kCus) * 105.0 * kf + 8.0;
    const int64_t mid = count_tiles(problems, n_problems, 128, 256);
    if (mid > kCus / 2 && mid <= kCus) return 70.0 * kf + 8.0;
    if (big == 128) return 105.0 * kf + 8.0;
    const int64_t small = count_tiles(problems, n_problems, 128, 128);
    return (small <= kCus ? 48.0 : (double)ceil_div(small, (int64_t)(2 * kCus)) * 80.0) * kf + 8.0;
}

int launch_gemm_batch(int dtype, const GemmProblem* problems, int n_problems, hipStream_t s, const EncodeJob* enc, bool* enc_fused,
                      bool plan_only, void* split_ws, size_t split_ws_bytes, bool may_cut) {
    if (enc_fused) *enc_fused = false;
    if (n_problems > kMaxGemmProblems) return ASTRA_ERR_UNSUPPORTED;
    // A launch whose last round of 256 x 256 tiles is nearly empty lasts a whole tile longer for a few tiles.  When the
    // problems can be dealt into two launches that are shorter together (say one that fills its rounds and a small one
    // on smaller tiles), run those: the launches are independent and follow each other on the stream.
    if (dtype == ASTRA_BF16 && may_cut && n_problems >= 2 && g_gemm_force_cfg < 0) {
        bool plain = true;
        for (int i = 0; i < n_problems; ++i)
            plain = plain && problems[i].c_mode != kCSwiGLU && problems[i].act == kActNone && !problems[i].residual;
        const int64_t big = count_tiles(problems, n_problems, 256, 256);
        if (plain && big > kCus && big % kCus != 0 && big % kCus <= 3 * kCus / 8) {
            const double whole = estimate_launch_us(problems, n_problems);
            double best = whole - 10.0;        // a second launch has to pay for itself with some margin
            unsigned best_mask = 0;
            GemmProblem a[kMaxGemmProblems], b[kMaxGemmProblems];
            for (unsigned mask = 1; mask + 1 < (1u << n_problems); ++mask) {
                int na = 0, nb = 0;
                for (int i = 0; i < n_problems; ++i) ((mask >> i) & 1u ? a[na++] : b[nb++]) = problems[i];
                const double t = estimate_launch_us(a, na) + estimate_launch_us(b, nb);
                if (t < best) { best = t; best_mask = mask; }
            }
            if (best_mask != 0) {
                int na = 0, nb = 0;
                for (int i = 0; i < n_problems; ++i) ((best_mask >> i) & 1u ? a[na++] : b[nb++]) = problems[i];
                bool fused_a = false, fused_b = false;
                int rc;
                if (!plan_only) {               // every problem is checked before the first of the two launches
                    rc = launch_gemm_batch(dtype, a, na, s, nullptr, nullptr, true, nullptr, 0, false);
                    if (rc) return rc;
                    rc = launch_gemm_batch(dtype, b, nb, s, nullptr, nullptr, true, nullptr, 0, false);
                    if (rc) return rc;
                }
                rc = launch_gemm_batch(dtype, a, na, s, enc, enc ? &fused_a : nullptr, plan_only, nullptr, 0, false);
                if (rc) return rc;
                rc = launch_gemm_batch(dtype, b, nb, s, fused_a ? nullptr : enc, enc && !fused_a ? &fused_b : nullptr, plan_only,
                                       nullptr, 0, false);
                if (enc_fused) *enc_fused = fused_a || fused_b;
                return rc;
            }
        }
    }
    GemmBatch batch{};
    int total = 0;
    if (dtype != ASTRA_BF16) {
        int rc = fill_batch(batch, dtype, problems, n_problems, 64, 64, &total);
        if (rc) return rc;
        if (total == 0 || plan_only) return ASTRA_OK;
        if (total >= 128) {
            gemm_nt_f32_kernel<64><<<total, 256, 0, s>>>(batch);
        } else {
            rc = fill_batch(batch, dtype, problems, n_problems, 32, 32, &total);
            if (rc) return rc;
            gemm_nt_f32_kernel<32><<<total, 256, 0, s>>>(batch);
        }
        return launch_status();
    }
    bool code16 = false, mlp = false;
    for (int i = 0; i < n_problems; ++i) {
        if (problems[i].codes && problems[i].code_bytes == 2) code16 = true;
        if (problems[i].c_mode == kCSwiGLU || problems[i].act != kActNone || problems[i].residual) mlp = true;
    }
    if (mlp) {
        // the MLP's GEMMs and the residual-adding output projection of a block: plain A rows, one problem per launch
        if (n_problems != 1 || problems[0].codes) return ASTRA_ERR_UNSUPPORTED;
        const GemmProblem& p0 = problems[0];
        int epi;
        if (p0.c_mode == kCSwiGLU) epi = kEpiSwiGLU;
        else if (p0.c_mode == kCBf16 && p0.act == kActGeluTanh) epi = kEpiGeluTanh;
        else if (p0.c_mode == kCBf16 && p0.act == kActGeluErf) epi = kEpiGeluErf;
        else if (p0.c_mode == kCF32 && p0.act == kActNone) epi = kEpiResidualF32;
        else return ASTRA_ERR_UNSUPPORTED;
        int rc = fill_batch(batch, dtype, problems, n_problems, 256, 256, &total);
        if (rc) return rc;
        if (total == 0) return ASTRA_OK;
        if (total >= 128) return plan_only ? ASTRA_OK : launch_gemm_mlp(epi, true, batch, total, s);
        const int ns = epi == kEpiResidualF32 && p0.ldc % 4 == 0 ? gemm_split_factor(dtype, p0.M, p0.N, p0.K) : 1;
        if (ns > 1 && split_ws && split_ws_bytes >= (size_t)ns * p0.M * p0.N * sizeof(float)) {
            if (plan_only) return ASTRA_OK;
            batch.n_split = ns;
            batch.k_split = p0.K / ns;
            batch.p[0].c = split_ws;
            rc = launch_gemm_mlp(kEpiSplit, true, batch, total * ns, s);
            if (rc) return rc;
            return launch_split_reduce((const float*)split_ws, ns, p0, s);
        }
        rc = fill_batch(batch, dtype, problems, n_problems, 128, 128, &total);
        if (rc) return rc;
        if (plan_only) return ASTRA_OK;
        if (total <= kCus / 2 && epi != kEpiSwiGLU && p0.K % (2 * kBK) == 0 && g_gemm_force_cfg < 0) {      // few tiles: see below
            GemmBatch sb{};
            int st = 0;
            rc = fill_batch(sb, dtype, problems, n_problems, 64, 64, &st);
            if (rc) return rc;
            if (st <= kCus) return launch_gemm_mlp_small(epi, sb, st, s);
        }
        return launch_gemm_mlp(epi, false, batch, total, s);
    }
    // Large tiles quarter the operand traffic per flop; use them once they still fill most of the chip.
    int rc = fill_batch(batch, dtype, problems, n_problems, 256, 256, &total);
    if (rc) return rc;
    bool big = total >= 128;
    if (g_gemm_force_cfg >= 0) big = g_gemm_force_cfg >= 1;
    // In between, 128 x 256 tiles: when they run as a single round of workgroups that fills more than half of the chip,
    // the launch lasts one such tile (about two thirds of a 256 x 256 one), where 256 x 256 tiles would leave half of
    // the units idle and 128 x 128 tiles would need a second workgroup per unit at a lower rate each.
    bool mid = false;
    if (g_gemm_force_cfg < 0 && total <= 128) {
        GemmBatch mb{};
        int mt = 0;
        rc = fill_batch(mb, dtype, problems, n_problems, 128, 256, &mt);
        if (rc) return rc;
        if (mt > kCus / 2 && mt <= kCus) {
            mid = true;
            big = false;
            batch = mb;
            total = mt;
        }
    }
    // Fuse the encode into the launch when the tiles leave a good part of the last round of compute units idle.
    if ((big || mid) && enc && enc_fused && g_gemm_force_cfg < 0 && vq_encode_fast_ok(enc->K, enc->dg) && enc->n_tokens > 0) {
        const int rem = total % kCus;
        const int E = rem == 0 ? 0 : ((kCus - rem) & ~7);
        const int64_t n_tb = ceil_div(enc->n_tokens, 256);
        // The encode workgroups must not outlast the tiles: an item (256 tokens of one group against its K codewords)
        // takes about 1 us per 2^20 codeword elements (16.5 us measured at K = 1024, dg = 64), a 256 x 256 tile about
        // 105 us per 4096 of contraction, a 128 x 256 tile about 70.
        int k_max = 0;
        for (int i = 0; i < batch.n; ++i) k_max = batch.p[i].K > k_max ? batch.p[i].K : k_max;
        const double tile_us = (mid ? 70.0 : 105.0) * k_max / 4096.0;
        const double enc_us = E > 0 ? (double)ceil_div(n_tb * enc->G, (int64_t)E) * 256.0 * enc->K * enc->dg / 1048576.0 : 0.0;
        if (E >= 8 && E <= kCus / 2 && n_tb * enc->G <= 0x7fffffff && enc_us <= 1.05 * tile_us) {
            batch.n_enc_wgs = E;
            batch.enc = *enc;
            batch.enc.n_tb = (int)n_tb;
            batch.enc.n_wgs = E;
            *enc_fused = true;
            if (plan_only) return ASTRA_OK;
            if (mid) {
                if (code16) gemm_nt_bf16_kernel<128, 256, 2, 4, true, true><<<total + E, 512, 0, s>>>(batch);
                else gemm_nt_bf16_kernel<128, 256, 2, 4, false, true><<<total + E, 512, 0, s>>>(batch);
            } else {
                if (code16) gemm_nt_bf16_kernel<256, 256, 2, 4, true, true><<<total + E, 512, 0, s>>>(batch);
                else gemm_nt_bf16_kernel<256, 256, 2, 4, false, true><<<total + E, 512, 0, s>>>(batch);
            }
            return launch_status();
        }
    }
    if (mid) {
        if (plan_only) return ASTRA_OK;
        if (code16) gemm_nt_bf16_kernel<128, 256, 2, 4, true><<<total, 512, 0, s>>>(batch);
        else gemm_nt_bf16_kernel<128, 256, 2, 4, false><<<total, 512, 0, s>>>(batch);
        return launch_status();
    }
    if (big && g_gemm_force_cfg == 2) {
        if (plan_only) return ASTRA_OK;
        if (code16) gemm_nt_bf16_kernel<256, 256, 2, 2, true><<<total, 256, 0, s>>>(batch);
        else gemm_nt_bf16_kernel<256, 256, 2, 2, false><<<total, 256, 0, s>>>(batch);
        return launch_status();
    }
    if (big) {
        if (total == 0 || plan_only) return ASTRA_OK;
        if (code16) gemm_nt_bf16_kernel<256, 256, 2, 4, true><<<total, 512, 0, s>>>(batch);
        else gemm_nt_bf16_kernel<256, 256, 2, 4, false><<<total, 512, 0, s>>>(batch);
        return launch_status();
    }
    rc = fill_batch(batch, dtype, problems, n_problems, 128, 128, &total);
    if (rc) return rc;
    if (total == 0) return ASTRA_OK;
    // one workgroup per compute unit at most: two contraction groups of four wavefronts (when every contraction is a
    // multiple of 128); more tiles than that: eight wavefronts on one contraction, two workgroups fit a compute unit
    bool ks2 = total <= kCus;
    for (int i = 0; i < batch.n; ++i) ks2 = ks2 && batch.p[i].K % (2 * kBK) == 0;
    if (ks2) {
        // Half-width tiles (128 x 64) when they still make a single round: a compute unit takes its operands in at 64 bytes per
        // clock whatever the others do, and a 128 x 64 tile needs three quarters of a 128 x 128 tile's bytes per step
        // (or 64 x 128, whichever makes fewer tiles: row counts just above a multiple of 128 waste less that way)
        bool narrow = false, flat = false;
        if (g_gemm_force_cfg < 0 && total <= kCus / 2) {
            GemmBatch nb{}, fb{};
            int nt = 0, ft = 0;
            rc = fill_batch(nb, dtype, problems, n_problems, 128, 64, &nt);
            if (rc) return rc;
            rc = fill_batch(fb, dtype, problems, n_problems, 64, 128, &ft);
            if (rc) return rc;
            if (nt <= kCus - 8 && nt <= ft) {
                narrow = true;
                batch = nb;
                total = nt;
            } else if (ft <= kCus - 8) {
                narrow = flat = true;
                batch = fb;
                total = ft;
            }
        }
        // a single round that leaves compute units idle: they take the encode of the local rows, as in the large-tile launches
        // (an item = 256 tokens of one group; about 1 us per 2^20 codeword elements; a 128 x 128 tile about 48 us per 4096 of
        // contraction plus 8 us of fixed cost)
        if (enc && enc_fused && g_gemm_force_cfg < 0 && vq_encode_fast_ok(enc->K, enc->dg) && enc->n_tokens > 0) {
            const int E = (kCus - total) & ~7;
            const int64_t n_tb = ceil_div(enc->n_tokens, 256);
            int k_max = 0;
            for (int i = 0; i < batch.n; ++i) k_max = batch.p[i].K > k_max ? batch.p[i].K : k_max;
            const double tile_us = (narrow ? 36.0 : 48.0) * k_max / 4096.0 + 8.0;
            const double enc_us = E > 0 ? (double)ceil_div(n_tb * enc->G, (int64_t)E) * 256.0 * enc->K * enc->dg / 1048576.0 + 4.0 : 0.0;
            if (E >= 8 && n_tb * enc->G <= 0x7fffffff && enc_us <= tile_us) {
                batch.n_enc_wgs = E;
                batch.enc = *enc;
                batch.enc.n_tb = (int)n_tb;
                batch.enc.n_wgs = E;
                *enc_fused = true;
                if (plan_only) return ASTRA_OK;
                if (flat) {
                    if (code16) gemm_nt_bf16_kernel<64, 128, 2, 2, true, true, kEpiLayer, 2><<<total + E, 512, 0, s>>>(batch);
                    else gemm_nt_bf16_kernel<64, 128, 2, 2, false, true, kEpiLayer, 2><<<total + E, 512, 0, s>>>(batch);
                } else if (narrow) {
                    if (code16) gemm_nt_bf16_kernel<128, 64, 2, 2, true, true, kEpiLayer, 2><<<total + E, 512, 0, s>>>(batch);
                    else gemm_nt_bf16_kernel<128, 64, 2, 2, false, true, kEpiLayer, 2><<<total + E, 512, 0, s>>>(batch);
                } else {
                    if (code16) gemm_nt_bf16_kernel<128, 128, 2, 2, true, true, kEpiLayer, 2><<<total + E, 512, 0, s>>>(batch);
                    else gemm_nt_bf16_kernel<128, 128, 2, 2, false, true, kEpiLayer, 2><<<total + E, 512, 0, s>>>(batch);
                }
                return launch_status();
            }
        }
        if (plan_only) return ASTRA_OK;
        // few tiles and no gathered rows (the output projection of a short sequence): a compute unit takes its operands in
        // at 64 bytes per clock whatever the others do, so the launch is spread over four times as many units on 64 x 64
        // tiles when those still make a single round
        bool plain = true;
        for (int i = 0; i < batch.n; ++i) plain = plain && batch.p[i].codes == nullptr;
        if (plain && g_gemm_force_cfg < 0) {
            GemmBatch sb{};
            int st = 0;
            rc = fill_batch(sb, dtype, problems, n_problems, 64, 64, &st);
            if (rc) return rc;
            if (st <= kCus) {                              // still a single round of workgroups
                gemm_nt_bf16_kernel<64, 64, 2, 2, false, false, kEpiLayer, 2><<<st, 512, 0, s>>>(sb);
                return launch_status();
            }
        }
        if (flat) {
            if (code16) gemm_nt_bf16_kernel<64, 128, 2, 2, true, false, kEpiLayer, 2><<<total, 512, 0, s>>>(batch);
            else gemm_nt_bf16_kernel<64, 128, 2, 2, false, false, kEpiLayer, 2><<<total, 512, 0, s>>>(batch);
            return launch_status();
        }
        if (narrow) {
            if (code16) gemm_nt_bf16_kernel<128, 64, 2, 2, true, false, kEpiLayer, 2><<<total, 512, 0, s>>>(batch);
            else gemm_nt_bf16_kernel<128, 64, 2, 2, false, false, kEpiLayer, 2><<<total, 512, 0, s>>>(batch);
            return launch_status();
        }
        if (code16) gemm_nt_bf16_kernel<128, 128, 2, 2, true, false, kEpiLayer, 2><<<total, 512, 0, s>>>(batch);
        else gemm_nt_bf16_kernel<128, 128, 2, 2, false, false, kEpiLayer, 2><<<total, 512, 0, s>>>(batch);
    } else {
        if (plan_only) return ASTRA_OK;
        if (code16) gemm_nt_bf16_kernel<128, 128, 4, 2, true><<<total, 512, 0, s>>>(batch);
        else gemm_nt_bf16_kernel<128, 128, 4, 2, false><<<total, 512, 0, s>>>(batch);
    }
    return launch_status();
}

}  // namespace astra
