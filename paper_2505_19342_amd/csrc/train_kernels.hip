// Training-side operations of the VQ module (paper Sec. 3.2: K-means initialisation, exponential-moving-average
// updates, the commitment term of Eq. 2; Sec. 3.3: NAVQ).  Forward arithmetic only.  All three are bound by memory
// traffic; every result is independent of the run (no floating-point atomics: tokens are first sorted by code with a
// stable counting sort, then every codeword's rows are added in ascending token order, partial sums in a fixed tree).
#include "common.h"

#include <algorithm>

namespace astra {

constexpr int kTrThreads = 256;

template <typename T>
__device__ __forceinline__ float tr_ld(const T* p);
template <>
__device__ __forceinline__ float tr_ld<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float tr_ld<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }

__device__ __forceinline__ int tr_code(const void* codes, int code16, int64_t i, int K) {
    const int c = code16 ? (int)((const uint16_t*)codes)[i] : (int)((const uint8_t*)codes)[i];
    return c < K ? c : K - 1;
}

// ---- stable counting sort of the tokens of every group by code, in three launches.  The tokens are cut into segments
// of seg_len; (1) every (segment, group) counts its codes (integer LDS atomics: exact); (2) per group, the counters are
// turned into counts[g, k], offs[g, 0..K] (exclusive prefix sums over k) and, in place, the first write position of
// every (segment, k): offs[k] + the counts of the earlier segments; (3) every (segment, group) places its tokens, 256
// at a time in ascending order: position = next position of the code + number of earlier tokens of the pass with the same
// code.  Result: perm[g, pos] = token index, sorted by (code, token).
__global__ __launch_bounds__(kTrThreads) void sort_count_kernel(const void* __restrict__ codes, int code16, int T, int G, int K,
                                                                int seg_len, int32_t* __restrict__ hist) {
    extern __shared__ int lds_i[];
    const int seg = blockIdx.x, g = blockIdx.y, tid = threadIdx.x;
    for (int k = tid; k < K; k += kTrThreads) lds_i[k] = 0;
    __syncthreads();
    const int t_hi = min((seg + 1) * seg_len, T);
    for (int t = seg * seg_len + tid; t < t_hi; t += kTrThreads) atomicAdd(&lds_i[tr_code(codes, code16, (int64_t)t * G + g, K)], 1);
    __syncthreads();
    int32_t* __restrict__ h = hist + ((int64_t)g * gridDim.x + seg) * K;
    for (int k = tid; k < K; k += kTrThreads) h[k] = lds_i[k];
}

// one workgroup per group.  Consecutive threads take consecutive codes (coalesced rows of the counters); the totals of the
// codes are scanned through LDS: a contiguous run of codes per thread, a wavefront scan of the runs' sums, the wavefronts'
// totals added in order.
__global__ __launch_bounds__(kTrThreads) void sort_scan_kernel(int32_t* __restrict__ hist, int n_seg, int K, int32_t* __restrict__ counts,
                                                               int32_t* __restrict__ offs) {
    extern __shared__ int lds_i[];          // [K] totals, then exclusive offsets
    __shared__ int wave_sum[kTrThreads / kWave];
    const int g = blockIdx.x, tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
    int32_t* __restrict__ h = hist + (int64_t)g * n_seg * K;
    for (int k = tid; k < K; k += kTrThreads) {
        int c = 0;
#pragma unroll 8
        for (int sg = 0; sg < n_seg; ++sg) c += h[(int64_t)sg * K + k];
        lds_i[k] = c;
        counts[(int64_t)g * K + k] = c;
    }
    __syncthreads();
    const int per = (K + kTrThreads - 1) / kTrThreads;
    const int k_lo = min(tid * per, K), k_hi = min(k_lo + per, K);
    int local = 0;
    for (int k = k_lo; k < k_hi; ++k) local += lds_i[k];
    int incl = local;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
    if (lane == kWave - 1) wave_sum[wave] = incl;
    __syncthreads();
    int base = incl - local;
    for (int w = 0; w < wave; ++w) base += wave_sum[w];
    for (int k = k_lo; k < k_hi; ++k) {
        const int c = lds_i[k];
        offs[(int64_t)g * (K + 1) + k] = base;
        lds_i[k] = base;
        base += c;
    }
    if (tid == kTrThreads - 1) offs[(int64_t)g * (K + 1) + K] = base;
    __syncthreads();
    for (int k = tid; k < K; k += kTrThreads) {
        int run = lds_i[k];
#pragma unroll 8
        for (int sg = 0; sg < n_seg; ++sg) {
            const int n = h[(int64_t)sg * K + k];
            h[(int64_t)sg * K + k] = run;               // first write position of (segment, code)
            run += n;
        }
    }
}

// Tokens of a pass with the same code are found inside a wavefront by comparing code bits across lanes (14 ballots: codes
// below 8192, and the all-ones code of a lane without a token), which gives every lane its rank among them; the four
// wavefronts then take their write positions one after the other, so the order stays the token order.  Also writes the
// sorted codes themselves (scode[g, pos]) for the kernels that walk the sorted sequence.
__global__ __launch_bounds__(kTrThreads) void sort_place_kernel(const void* __restrict__ codes, int code16, int T, int G, int K,
                                                                int seg_len, const int32_t* __restrict__ hist, int32_t* __restrict__ perm,
                                                                uint16_t* __restrict__ scode) {
    extern __shared__ int lds_i[];
    int* nxt = lds_i;                       // [K] next write position of every code
    const int seg = blockIdx.x, g = blockIdx.y, tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
    const int32_t* __restrict__ h = hist + ((int64_t)g * gridDim.x + seg) * K;
    for (int k = tid; k < K; k += kTrThreads) nxt[k] = h[k];
    __syncthreads();
    const int t_hi = min((seg + 1) * seg_len, T);
    for (int t0 = seg * seg_len; t0 < t_hi; t0 += kTrThreads) {
        const int t = t0 + tid;
        const int c = t < t_hi ? tr_code(codes, code16, (int64_t)t * G + g, K) : -1;
        unsigned long long peers = ~0ull;
#pragma unroll
        for (int b = 0; b < 14; ++b) {
            const bool bit = ((c >> b) & 1) != 0;
            const unsigned long long bal = __builtin_amdgcn_ballot_w64(bit);
            peers &= bit ? bal : ~bal;
        }
        const int rank = __popcll(peers & ((1ull << lane) - 1ull));
        const int cnt = __popcll(peers);
#pragma unroll
        for (int w = 0; w < kTrThreads / kWave; ++w) {
            if (wave == w && c >= 0) {
                const int base = nxt[c];            // every lane of the wavefront reads before its first lanes write
                perm[(int64_t)g * T + base + rank] = t;
                scode[(int64_t)g * T + base + rank] = (uint16_t)c;
                if (rank == 0) nxt[c] = base + cnt;
            }
            __syncthreads();
        }
    }
}

// ---- sums of the rows of every codeword and the squared distances to the codeword, for element types and group widths
// without whole 16-byte pieces (fp32, unaligned bf16 slices).  grid (blocks of codewords, G), a channel per thread.
// PH threads share a (codeword, channel) pair: thread ph adds the rows at positions lo + ph, lo + ph + PH, ... of the
// codeword's sorted run (four in flight), and the PH partial sums are added in ascending ph: a fixed order, so the result
// does not depend on the run, while a long run keeps 4 * PH rows in flight.
template <typename T, int PH>
__global__ __launch_bounds__(kTrThreads) void stats_sum_kernel(const T* __restrict__ x, int64_t ldx, const T* __restrict__ codebook,
                                                               const int32_t* __restrict__ offs, const int32_t* __restrict__ perm,
                                                               int Tn, int G, int K, int dg, int kb,
                                                               float* __restrict__ sums, float* __restrict__ sq_part) {
    extern __shared__ float xs_lds[];                      // [kb][PH][dg]
    __shared__ float red[kTrThreads / kWave];
    constexpr int VC = 1;
    const int g = blockIdx.y, tid = threadIdx.x;
    const int tpc = dg / VC;                               // threads per row
    const int kk = tid / (PH * tpc), rem = tid - kk * (PH * tpc);
    const int ph = rem / tpc, j = (rem - ph * tpc) * VC;
    const int k = blockIdx.x * kb + kk;
    const bool on = kk < kb && k < K;
    float sq = 0.f;
    if (on) {
        const int lo = offs[(int64_t)g * (K + 1) + k], hi = offs[(int64_t)g * (K + 1) + k + 1];
        float c[VC], s[VC];
        const T* __restrict__ cw = codebook + ((int64_t)g * K + k) * dg + j;
#pragma unroll
        for (int e = 0; e < VC; ++e) {
            c[e] = tr_ld(cw + e);
            s[e] = 0.f;
        }
        const T* __restrict__ xs = x + (int64_t)g * dg + j;
        const int32_t* __restrict__ pm = perm + (int64_t)g * Tn;
        for (int pos = lo + ph; pos < hi; pos += 4 * PH) {
            float v[4][VC];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int t = pm[min(pos + u * PH, hi - 1)];                     // beyond the run: a repeat, not added
#pragma unroll
                for (int e = 0; e < VC; ++e) v[u][e] = tr_ld(xs + t * ldx + e);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (pos + u * PH < hi)
#pragma unroll
                    for (int e = 0; e < VC; ++e) {
                        s[e] += v[u][e];
                        sq = fmaf(v[u][e] - c[e], v[u][e] - c[e], sq);
                    }
        }
#pragma unroll
        for (int e = 0; e < VC; ++e) xs_lds[(kk * PH + ph) * dg + j + e] = s[e];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
    if (lane_id() == 0) red[tid / kWave] = sq;
    __syncthreads();
    if (on && ph == 0)
#pragma unroll
        for (int e = 0; e < VC; ++e) {
            float t = 0.f;
            for (int q = 0; q < PH; ++q) t += xs_lds[(kk * PH + q) * dg + j + e];
            sums[((int64_t)g * K + k) * dg + j + e] = t;
        }
    if (tid == 0) {
        float t = 0.f;
        for (int w = 0; w < kTrThreads / kWave; ++w) t += red[w];
        sq_part[(int64_t)g * gridDim.x + blockIdx.x] = t;
    }
}

// ---- the same sums for bf16 rows of whole 16-byte pieces, balanced over the sorted sequence instead of over codewords:
// a unit is kUnitRows consecutive positions of a group's sorted sequence, walked by dg / 8 threads (8 channels each) in
// ascending order, 8 rows (and the 8 codeword pieces their squared distances need) in flight.  A codeword whose run lies
// inside one unit gets its sum from that unit; a run that crosses unit boundaries leaves one partial sum per unit
// (part[g, unit, 0] when the run comes in from the previous unit, part[g, unit, 1] when it starts inside the unit and
// goes on), which stats_fix_kernel adds in ascending unit order: a fixed tree, whatever the codes' distribution.
constexpr int kUnitRows = 32;

__global__ __launch_bounds__(kTrThreads) void stats_units_kernel(const uint16_t* __restrict__ x, int64_t ldx, const uint16_t* __restrict__ codebook,
                                                                 const int32_t* __restrict__ perm, const uint16_t* __restrict__ scode, int T, int G,
                                                                 int K, int dg, int units_per_wg, int n_units, float* __restrict__ sums,
                                                                 float* __restrict__ part, float* __restrict__ sq_part) {
    extern __shared__ int lds_i[];
    __shared__ float red[kTrThreads / kWave];
    const int g = blockIdx.y, tid = threadIdx.x;
    const int tpc = dg >> 3;
    const int rows_wg = units_per_wg * kUnitRows;
    const int p_wg = blockIdx.x * rows_wg;
    const int n_wg = min(rows_wg, T - p_wg);
    int* l_perm = lds_i;                    // [rows_wg] token of position p_wg + i
    int* l_code = lds_i + rows_wg;          // [rows_wg + 2] code of position p_wg - 1 + i, -1 outside the sequence
    for (int i = tid; i < rows_wg; i += kTrThreads) l_perm[i] = perm[(int64_t)g * T + min(p_wg + i, T - 1)];
    for (int i = tid; i < rows_wg + 2; i += kTrThreads) {
        const int pos = p_wg - 1 + i;
        l_code[i] = pos >= 0 && pos < T ? (int)scode[(int64_t)g * T + pos] : -1;
    }
    __syncthreads();
    const int ul = tid / tpc, j = (tid - ul * tpc) * 8;
    const int r0 = ul * kUnitRows;
    float sq = 0.f;
    if (ul < units_per_wg && r0 < n_wg) {
        const int n = min(kUnitRows, n_wg - r0);
        const int unit = blockIdx.x * units_per_wg + ul;
        const uint16_t* __restrict__ xs = x + (int64_t)g * dg + j;
        const uint16_t* __restrict__ cbs = codebook + (int64_t)g * K * dg + j;
        float s[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] = 0.f;
        bool from_prev = l_code[r0] == l_code[r0 + 1];
#pragma unroll
        for (int b = 0; b < kUnitRows; b += 8) {
            if (b < n) {
                u32x4 xv[8], cv[8];
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const int i = min(b + r, n - 1);                         // beyond the unit: a repeat, not added
                    xv[r] = *reinterpret_cast<const u32x4*>(xs + (int64_t)l_perm[r0 + i] * ldx);
                    cv[r] = *reinterpret_cast<const u32x4*>(cbs + (int64_t)l_code[r0 + i + 1] * dg);
                }
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const int i = b + r;
                    if (i < n) {
                        const uint32_t xw[4] = {xv[r].x, xv[r].y, xv[r].z, xv[r].w}, cw[4] = {cv[r].x, cv[r].y, cv[r].z, cv[r].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float x0 = __uint_as_float(xw[e] << 16), x1 = __uint_as_float(xw[e] & 0xffff0000u);
                            const float c0 = __uint_as_float(cw[e] << 16), c1 = __uint_as_float(cw[e] & 0xffff0000u);
                            s[2 * e] += x0;
                            s[2 * e + 1] += x1;
                            sq = fmaf(x0 - c0, x0 - c0, sq);
                            sq = fmaf(x1 - c1, x1 - c1, sq);
                        }
                        const int c = l_code[r0 + i + 1], cn = l_code[r0 + i + 2];
                        if (i == n - 1 || cn != c) {                             // last row of this codeword inside the unit
                            const bool to_next = i == n - 1 && cn == c;
                            float* __restrict__ dst = !from_prev && !to_next ? sums + ((int64_t)g * K + c) * dg + j
                                                                             : part + (((int64_t)g * n_units + unit) * 2 + (from_prev ? 0 : 1)) * dg + j;
                            *reinterpret_cast<f32x4*>(dst) = f32x4{s[0], s[1], s[2], s[3]};
                            *reinterpret_cast<f32x4*>(dst + 4) = f32x4{s[4], s[5], s[6], s[7]};
#pragma unroll
                            for (int e = 0; e < 8; ++e) s[e] = 0.f;
                            from_prev = false;
                        }
                    }
                }
            }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
    if (lane_id() == 0) red[tid / kWave] = sq;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int w = 0; w < kTrThreads / kWave; ++w) t += red[w];
        sq_part[(int64_t)g * gridDim.x + blockIdx.x] = t;
    }
}

// sums of the codewords the units left open: none of the rows (zero), or a run over several units (its partial sums in
// ascending unit order).  A thread per (codeword, 8 channels); n = number of such pieces.
__global__ __launch_bounds__(kTrThreads) void stats_fix_kernel(const int32_t* __restrict__ offs, const float* __restrict__ part, int n_units,
                                                               int64_t n, int K, int dg, float* __restrict__ sums) {
    const int64_t i = (int64_t)blockIdx.x * kTrThreads + threadIdx.x;
    if (i >= n) return;
    const int tpc = dg >> 3;
    const int64_t cw = i / tpc;
    const int j = (int)(i - cw * tpc) * 8;
    const int64_t g = cw / K;
    const int k = (int)(cw - g * K);
    const int lo = offs[g * (K + 1) + k], hi = offs[g * (K + 1) + k + 1];
    const int u_lo = lo / kUnitRows, u_hi = (hi - 1) / kUnitRows;
    if (lo != hi && u_lo == u_hi) return;                   // written by its unit
    f32x4 t0 = {0.f, 0.f, 0.f, 0.f}, t1 = {0.f, 0.f, 0.f, 0.f};
    if (lo != hi) {
        const float* __restrict__ p = part + ((g * n_units + u_lo) * 2 + 1) * dg + j;
        t0 = *reinterpret_cast<const f32x4*>(p);
        t1 = *reinterpret_cast<const f32x4*>(p + 4);
        for (int u = u_lo + 1; u <= u_hi; u += 4) {          // four units in flight; beyond the run: a repeat, not added
            f32x4 a[4], b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                p = part + ((g * n_units + min(u + q, u_hi)) * 2) * dg + j;
                a[q] = *reinterpret_cast<const f32x4*>(p);
                b[q] = *reinterpret_cast<const f32x4*>(p + 4);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (u + q <= u_hi) {
                    t0 += a[q];
                    t1 += b[q];
                }
        }
    }
    float* __restrict__ dst = sums + cw * dg + j;
    *reinterpret_cast<f32x4*>(dst) = t0;
    *reinterpret_cast<f32x4*>(dst + 4) = t1;
}

// sqerr[g] = sum of the blocks' partial sums: one workgroup per group, a fixed tree (strided partial sums, then lanes)
__global__ __launch_bounds__(kTrThreads) void stats_sqerr_kernel(const float* __restrict__ sq_part, int n_blocks, float* __restrict__ sqerr) {
    __shared__ float red[kTrThreads / kWave];
    const int g = blockIdx.x, tid = threadIdx.x;
    float t = 0.f;
    for (int b = tid; b < n_blocks; b += kTrThreads) t += sq_part[(int64_t)g * n_blocks + b];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o);
    if (lane_id() == 0) red[tid / kWave] = t;
    __syncthreads();
    if (tid == 0) {
        float r = 0.f;
        for (int w = 0; w < kTrThreads / kWave; ++w) r += red[w];
        sqerr[g] = r;
    }
}

// ---- codebook update: EMA of counts and sums (gamma > 0) or the plain K-means centroid (gamma = 0)
template <typename T>
__global__ __launch_bounds__(kTrThreads) void codebook_update_kernel(const int32_t* __restrict__ counts, const float* __restrict__ sums,
                                                                     float gamma, float* ema_n, float* ema_m,
                                                                     const T* cb_old, int64_t n_cw, int dg, T* cb_new) {   // cb_new may be cb_old: no restrict
    const int64_t i = (int64_t)blockIdx.x * kTrThreads + threadIdx.x;          // (codeword, channel)
    if (i >= n_cw * dg) return;
    const int64_t cw = i / dg;
    float n = (float)counts[cw], m = sums[i];
    if (ema_n) {
        n = gamma * ema_n[cw] + (1.f - gamma) * n;
        m = gamma * ema_m[i] + (1.f - gamma) * m;
        ema_m[i] = m;
    }
    const float v = n > 0.f ? m / n : tr_ld(cb_old + i);
    if constexpr (sizeof(T) == 2) cb_new[i] = f32_to_bf16_bits(v);
    else cb_new[i] = v;
}
// the counts' average is written by a launch of its own after every channel has read the old value
__global__ __launch_bounds__(kTrThreads) void ema_count_kernel(const int32_t* __restrict__ counts, float gamma, float* __restrict__ ema_n, int64_t n_cw) {
    const int64_t i = (int64_t)blockIdx.x * kTrThreads + threadIdx.x;
    if (i < n_cw) ema_n[i] = gamma * ema_n[i] + (1.f - gamma) * (float)counts[i];
}

// ---- NAVQ base: out[t, :] = codeword lookup + lambda * mu (fp32); the matrix product z . F^T is added by the GEMM
template <typename T>
__global__ __launch_bounds__(kTrThreads) void navq_base_kernel(const void* __restrict__ codes, int code16, const T* __restrict__ codebook,
                                                               const float* __restrict__ mu, float lambda, int64_t n, int D, int G, int K,
                                                               int dg, float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * kTrThreads + threadIdx.x;
    if (i >= n) return;
    const int64_t t = i / D;
    const int c = (int)(i - t * D);
    const int g = c / dg;
    const int code = tr_code(codes, code16, t * G + g, K);
    out[i] = tr_ld(codebook + ((int64_t)g * K + code) * dg + (c - g * dg)) + lambda * mu[c];
}

struct StatsPlan {
    int vc, ph, kb, n_blocks, seg_len, n_seg;
    bool units;                       // bf16 rows of whole 16-byte pieces: the balanced kernels
    int units_per_wg, n_units;
    size_t off_offs, off_perm, off_sq, off_hist, off_scode, off_part, total;
};
static int make_stats_plan(const astra_vq_desc& d, int64_t T, StatsPlan* pl) {
    int rc = check_vq_desc(&d);
    if (rc) return rc;
    if (T < 0 || T > (1 << 30)) return ASTRA_ERR_SHAPE;
    const int dg = d.d_model / d.n_groups;
    if (dg > kTrThreads || d.codebook_size > 8192) return ASTRA_ERR_UNSUPPORTED;      // a thread per (codeword, channels); counters in LDS
    pl->vc = d.dtype == ASTRA_BF16 && dg % 8 == 0 && d.d_model % 8 == 0 ? 8 : 1;
    pl->ph = dg / pl->vc * 4 <= kTrThreads ? 4 : 1;                               // threads sharing a (codeword, channels) pair
    pl->kb = kTrThreads / (dg / pl->vc * pl->ph);
    pl->units = pl->vc == 8;
    pl->units_per_wg = pl->units ? std::min(kTrThreads / (dg / 8), 64) : 0;
    pl->n_units = (int)ceil_div(T, kUnitRows);
    pl->n_blocks = pl->units ? (int)ceil_div(T, (int64_t)pl->units_per_wg * kUnitRows) : (int)ceil_div(d.codebook_size, pl->kb);
    // segments of at least 1024 tokens, about four workgroups per compute unit over all groups
    const int64_t want = std::max<int64_t>(1, 4 * 256 / d.n_groups);
    const int64_t n_seg = std::max<int64_t>(1, std::min<int64_t>(want, ceil_div(T, 1024)));
    pl->seg_len = (int)std::max<int64_t>(kTrThreads, ceil_div(ceil_div(T, n_seg), kTrThreads) * kTrThreads);
    pl->n_seg = (int)std::max<int64_t>(1, ceil_div(T, pl->seg_len));
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    pl->off_offs = take((size_t)d.n_groups * (d.codebook_size + 1) * 4);
    pl->off_perm = take((size_t)d.n_groups * T * 4);
    pl->off_sq = take((size_t)d.n_groups * std::max(pl->n_blocks, 1) * 4);
    pl->off_hist = take((size_t)d.n_groups * pl->n_seg * d.codebook_size * 4);
    pl->off_scode = take((size_t)d.n_groups * T * 2);
    pl->off_part = take(pl->units ? (size_t)d.n_groups * pl->n_units * 2 * dg * 4 : 0);
    pl->total = off;
    return ASTRA_OK;
}

}  // namespace astra

using namespace astra;

extern "C" {

size_t astra_codebook_stats_workspace_bytes(const astra_vq_desc* desc, int64_t n_tokens) {
    StatsPlan pl;
    if (!desc || make_stats_plan(*desc, n_tokens, &pl) != ASTRA_OK) return 0;
    return pl.total;
}

int astra_codebook_stats(const astra_vq_desc* desc, const void* x, const void* codes, int64_t n_tokens, const void* codebook,
                         int32_t* counts_out, float* sums_out, float* sqerr_out, void* workspace, size_t workspace_bytes,
                         void* stream) {
    if (!desc) return ASTRA_ERR_NULL;
    StatsPlan pl;
    int rc = make_stats_plan(*desc, n_tokens, &pl);
    if (rc) return rc;
    if (!codebook || !counts_out || !sums_out || !sqerr_out) return ASTRA_ERR_NULL;
    if (n_tokens > 0 && (!x || !codes)) return ASTRA_ERR_NULL;
    if (!workspace || workspace_bytes < pl.total) return ASTRA_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int G = desc->n_groups, K = desc->codebook_size, D = desc->d_model, dg = D / G, T = (int)n_tokens;
    char* ws = (char*)workspace;
    int32_t* offs = (int32_t*)(ws + pl.off_offs);
    int32_t* perm = (int32_t*)(ws + pl.off_perm);
    float* sq_part = (float*)(ws + pl.off_sq);
    const int code16 = desc->code_type == ASTRA_CODE_U16 ? 1 : 0;
    int32_t* hist = (int32_t*)(ws + pl.off_hist);
    uint16_t* scode = (uint16_t*)(ws + pl.off_scode);
    float* part = (float*)(ws + pl.off_part);
    const dim3 sgrid(pl.n_seg, G);
    sort_count_kernel<<<sgrid, kTrThreads, (size_t)K * sizeof(int), s>>>(codes, code16, T, G, K, pl.seg_len, hist);
    sort_scan_kernel<<<G, kTrThreads, (size_t)K * sizeof(int), s>>>(hist, pl.n_seg, K, counts_out, offs);
    sort_place_kernel<<<sgrid, kTrThreads, (size_t)K * sizeof(int), s>>>(codes, code16, T, G, K, pl.seg_len, hist, perm, scode);
    if (pl.units) {
        if (pl.n_blocks > 0) {
            const size_t lds = (size_t)(2 * pl.units_per_wg * kUnitRows + 2) * sizeof(int);
            stats_units_kernel<<<dim3(pl.n_blocks, G), kTrThreads, lds, s>>>((const uint16_t*)x, D, (const uint16_t*)codebook, perm, scode, T, G, K,
                                                                             dg, pl.units_per_wg, pl.n_units, sums_out, part, sq_part);
        }
        const int64_t n = (int64_t)G * K * (dg / 8);
        stats_fix_kernel<<<(int)ceil_div(n, kTrThreads), kTrThreads, 0, s>>>(offs, part, pl.n_units, n, K, dg, sums_out);
    } else {
        const dim3 grid(pl.n_blocks, G);
        const size_t xs_bytes = (size_t)pl.kb * pl.ph * dg * sizeof(float);
#define ASTRA_SUM_LAUNCH(TT, PHH)                                                                                              \
    stats_sum_kernel<TT, PHH><<<grid, kTrThreads, xs_bytes, s>>>((const TT*)x, D, (const TT*)codebook, offs, perm, T, G, K, dg, \
                                                                      pl.kb, sums_out, sq_part)
        if (desc->dtype == ASTRA_BF16 && pl.ph == 4) ASTRA_SUM_LAUNCH(uint16_t, 4);
        else if (desc->dtype == ASTRA_BF16) ASTRA_SUM_LAUNCH(uint16_t, 1);
        else if (pl.ph == 4) ASTRA_SUM_LAUNCH(float, 4);
        else ASTRA_SUM_LAUNCH(float, 1);
#undef ASTRA_SUM_LAUNCH
    }
    stats_sqerr_kernel<<<G, kTrThreads, 0, s>>>(sq_part, pl.n_blocks, sqerr_out);
    return launch_status();
}

int astra_codebook_update(const astra_vq_desc* desc, const int32_t* counts, const float* sums, float gamma, float* ema_n,
                          float* ema_m, const void* codebook_old, void* codebook_new_out, void* stream) {
    int rc = check_vq_desc(desc);
    if (rc) return rc;
    if (!(gamma >= 0.f && gamma < 1.f)) return ASTRA_ERR_SHAPE;
    if (!counts || !sums || !codebook_old || !codebook_new_out) return ASTRA_ERR_NULL;
    if (gamma > 0.f && (!ema_n || !ema_m)) return ASTRA_ERR_NULL;
    if (gamma == 0.f) ema_n = ema_m = nullptr;
    hipStream_t s = (hipStream_t)stream;
    const int dg = desc->d_model / desc->n_groups;
    const int64_t n_cw = (int64_t)desc->n_groups * desc->codebook_size;
    if (ceil_div(n_cw * dg, kTrThreads) > 0x7fffffff) return ASTRA_ERR_SHAPE;
    const int blocks = (int)ceil_div(n_cw * dg, kTrThreads);
    if (desc->dtype == ASTRA_BF16)
        codebook_update_kernel<uint16_t><<<blocks, kTrThreads, 0, s>>>(counts, sums, gamma, ema_n, ema_m, (const uint16_t*)codebook_old, n_cw,
                                                                       dg, (uint16_t*)codebook_new_out);
    else
        codebook_update_kernel<float><<<blocks, kTrThreads, 0, s>>>(counts, sums, gamma, ema_n, ema_m, (const float*)codebook_old, n_cw, dg,
                                                                    (float*)codebook_new_out);
    if (ema_n) ema_count_kernel<<<(int)ceil_div(n_cw, kTrThreads), kTrThreads, 0, s>>>(counts, gamma, ema_n, n_cw);
    return launch_status();
}

int astra_navq_forward(const astra_vq_desc* desc, const void* codes, int64_t n_tokens, const void* codebook, const float* mu,
                       float lambda, const void* z, const void* noise_factor, float* x_tilde_out, void* stream) {
    int rc = check_vq_desc(desc);
    if (rc) return rc;
    if (n_tokens < 0 || n_tokens > (1 << 30) || !(lambda >= 0.f)) return ASTRA_ERR_SHAPE;
    if (n_tokens == 0) return ASTRA_OK;
    if (!codes || !codebook || !mu || !z || !noise_factor || !x_tilde_out) return ASTRA_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    const int D = desc->d_model, G = desc->n_groups, K = desc->codebook_size, dg = D / G;
    // x_tilde = (codeword lookup + lambda mu) + z . F^T, the first part being where the product's accumulation starts
    GemmProblem p = {};
    p.a = z; p.b = noise_factor; p.c = x_tilde_out; p.M = (int)n_tokens; p.N = D; p.K = D; p.lda = D; p.ldc = D;
    p.c_mode = kCF32;
    p.residual = x_tilde_out;
    rc = launch_gemm_batch(desc->dtype, &p, 1, s, nullptr, nullptr, true);
    if (rc) return rc;
    const int64_t n = n_tokens * D;
    if (ceil_div(n, kTrThreads) > 0x7fffffff) return ASTRA_ERR_SHAPE;
    const int blocks = (int)ceil_div(n, kTrThreads);
    const int code16 = desc->code_type == ASTRA_CODE_U16 ? 1 : 0;
    if (desc->dtype == ASTRA_BF16)
        navq_base_kernel<uint16_t><<<blocks, kTrThreads, 0, s>>>(codes, code16, (const uint16_t*)codebook, mu, lambda, n, D, G, K, dg, x_tilde_out);
    else
        navq_base_kernel<float><<<blocks, kTrThreads, 0, s>>>(codes, code16, (const float*)codebook, mu, lambda, n, D, G, K, dg, x_tilde_out);
    return launch_gemm_batch(desc->dtype, &p, 1, s);
}

}  // extern "C"
