// Mixed-precision attention of one device (paper Sec. 3.2, Eq. 1): local queries attend to the
// full-precision local keys/values and to keys/values projected from the tokens rebuilt from codes.
// The two key/value sources are never concatenated in memory: the kernels walk the visible
// non-local rows first and the local rows after them (softmax does not depend on key order).
#include "common.h"

namespace astra {

struct AttnParams {
    const void* q;        // [T_q, H_q, dh]
    const void* k_loc;    // [T_q, H_kv, dh]
    const void* v_loc;
    const void* k_hat;    // [T_n, H_kv, dh]
    const void* v_hat;
    void* out;            // [T_q, H_q, dh]
    float* lse;           // nullable [H_q, T_q]
    int32_t Hq, Hkv, Tq;
    int32_t Tn_vis;       // visible non-local rows (all of them, or those before the chunk when causal)
    int32_t causal;
    float scale;          // logit scale
};

// ------------------------------------------------------------------------------------------------
// bf16, matrix cores, flash style (online softmax, nothing of size T_q x T_k is ever stored).
//
// A workgroup of 4 wavefronts owns 128 query rows of one head; wavefront w owns 32 of them.  Scores
// are computed transposed, S^T = K_tile . Q^T (keys on the M side, queries on the N side of the
// 32x32x16 MFMA), so that the 16 accumulator values of a lane all belong to ONE query: the running
// max / sum of the online softmax are per-lane scalars, and the probabilities, rounded to bf16 in
// place, already have the register layout of the B operand of O^T += V^T . P^T.  The only operand that
// needs a transpose is V; it is read from its row-major LDS tile with the 64-bit transposing LDS read.
// Key/value tiles of 64 rows are staged in LDS with XOR-swizzled 16-byte pieces.
// ------------------------------------------------------------------------------------------------
constexpr int kAttQ = 128;   // query rows per workgroup
constexpr int kAttKV = 64;   // key/value rows per tile

template <int DH>
__device__ __forceinline__ int swz_k(int r) { return DH == 128 ? (r & 15) : ((r >> 1) & 7); }
template <int DH>
__device__ __forceinline__ int swz_v(int r) { return DH == 128 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2); }

template <int DH>
__global__ __launch_bounds__(256) void attn_bf16_kernel(const AttnParams p) {
    constexpr int CPR = DH / 8;                // 16-byte pieces per row
    constexpr int NKS = DH / 16;               // contraction steps of Q.K
    constexpr int NDB = DH / 32;               // 32-wide blocks of the head dimension
    constexpr int PIECES = kAttKV * CPR;       // pieces per tile
    __shared__ uint4 lds_k[PIECES];
    __shared__ uint4 lds_v[PIECES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int i32 = lane & 31, h = lane >> 5;
    const int head = blockIdx.y;
    const int hk = head / (p.Hq / p.Hkv);
    // heavier (later) query blocks first under causal masking
    const int qb = gridDim.x - 1 - blockIdx.x;
    const int q0 = qb * kAttQ;
    const int Tq = p.Tq;
    const int64_t q_ld = (int64_t)p.Hq * DH, kv_ld = (int64_t)p.Hkv * DH;

    const int qrow = q0 + wave * 32 + i32;                 // this lane's query (N side)
    const int qrow_ld = qrow < Tq ? qrow : Tq - 1;
    const uint16_t* __restrict__ Q = (const uint16_t*)p.q + (int64_t)qrow_ld * q_ld + (int64_t)head * DH;
    bf16x8 qf[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(Q + 16 * ks + 8 * h));

    f32x16 acc_o[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float sl2 = p.scale * 1.4426950408889634f;       // logits in base-2 units

    const int n_hat_tiles = (p.Tn_vis + kAttKV - 1) / kAttKV;
    const int loc_rows = p.causal ? min(q0 + kAttQ, Tq) : Tq;     // local keys any row of this block may see
    const int n_loc_tiles = (loc_rows + kAttKV - 1) / kAttKV;
    const int wave_last_q = q0 + wave * 32 + 31;

    for (int t = 0; t < n_hat_tiles + n_loc_tiles; ++t) {
        const bool is_loc = t >= n_hat_tiles;
        const int row0 = (is_loc ? t - n_hat_tiles : t) * kAttKV;
        const int count = is_loc ? Tq : p.Tn_vis;
        const uint16_t* __restrict__ Ks = (const uint16_t*)(is_loc ? p.k_loc : p.k_hat) + (int64_t)hk * DH;
        const uint16_t* __restrict__ Vs = (const uint16_t*)(is_loc ? p.v_loc : p.v_hat) + (int64_t)hk * DH;

        __syncthreads();
#pragma unroll
        for (int it = 0; it < PIECES / 256; ++it) {
            const int c = tid + 256 * it;
            const int r = c / CPR, pc = c % CPR;
            const int rg = row0 + r < count ? row0 + r : count - 1;
            const uint4 kv = *reinterpret_cast<const uint4*>(Ks + (int64_t)rg * kv_ld + pc * 8);
            const uint4 vv = *reinterpret_cast<const uint4*>(Vs + (int64_t)rg * kv_ld + pc * 8);
            lds_k[r * CPR + (pc ^ swz_k<DH>(r))] = kv;
            lds_v[r * CPR + (pc ^ swz_v<DH>(r))] = vv;
        }
        __syncthreads();

        const bool diag = is_loc && p.causal && (row0 + kAttKV - 1 > q0 + wave * 32);   // some (q, k) pair of this wave is hidden
        if (is_loc && p.causal && row0 > wave_last_q) continue;                        // whole tile hidden from this wave
        const bool ragged = row0 + kAttKV > count;

        // S^T tile: 64 keys x 32 queries
        f32x16 acc_s[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc_s[mb][v] = 0.f;
            const int r = mb * 32 + i32;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const bf16x8 kf = as_bf16x8(lds_k[r * CPR + ((2 * ks + h) ^ swz_k<DH>(r))]);
                acc_s[mb] = mfma_32x32x16(kf, qf[ks], acc_s[mb]);
            }
        }
        // scale, mask, running max
        float mx = -INFINITY;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float s = acc_s[mb][v] * sl2;
                if (ragged || diag) {
                    const int key = row0 + mb * 32 + acc_row(v, h);
                    if (key >= count || (diag && key > qrow)) s = -INFINITY;
                }
                acc_s[mb][v] = s;
                mx = fmaxf(mx, s);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = exp2f(m_run - m_safe);
        m_run = m_new;
        float lsum = 0.f;
        bf16x8 pf[4];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float e = exp2f(acc_s[mb][v] - m_safe);
                lsum += e;
                pf[mb * 2 + (v >> 3)][v & 7] = (__bf16)e;
            }
        l_run = l_run * alpha + lsum;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc_o[db][v] *= alpha;

        // O^T += V^T . P^T : contraction over the 64 keys in 4 steps of 16
        const int s16 = lane & 15, q4 = lane >> 4;
#pragma unroll
        for (int kstep = 0; kstep < 4; ++kstep) {
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                const int c = db * 4 + 2 * (q4 & 1) + ((s16 & 3) >> 1);
                const int r_lo = 16 * kstep + 4 * h + (s16 >> 2);
                const int r_hi = r_lo + 8;
                const char* base = reinterpret_cast<const char*>(lds_v);
                const s16x4 lo = lds_read_tr16_b64(base + (r_lo * CPR + (c ^ swz_v<DH>(r_lo))) * 16 + 8 * (s16 & 1));
                const s16x4 hi = lds_read_tr16_b64(base + (r_hi * CPR + (c ^ swz_v<DH>(r_hi))) * 16 + 8 * (s16 & 1));
                uint4 packed;
                packed.x = (uint16_t)lo[0] | ((uint32_t)(uint16_t)lo[1] << 16);
                packed.y = (uint16_t)lo[2] | ((uint32_t)(uint16_t)lo[3] << 16);
                packed.z = (uint16_t)hi[0] | ((uint32_t)(uint16_t)hi[1] << 16);
                packed.w = (uint16_t)hi[2] | ((uint32_t)(uint16_t)hi[3] << 16);
                acc_o[db] = mfma_32x32x16(as_bf16x8(packed), pf[kstep], acc_o[db]);
            }
        }
    }

    // finish: merge the two half-waves' partial sums, normalise, store 4 consecutive head-dim values per lane
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (qrow < Tq) {
        uint16_t* __restrict__ O = (uint16_t*)p.out + (int64_t)qrow * q_ld + (int64_t)head * DH;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                uint2 w;
                w.x = pack_bf16x2(acc_o[db][4 * vq + 0] * inv, acc_o[db][4 * vq + 1] * inv);
                w.y = pack_bf16x2(acc_o[db][4 * vq + 2] * inv, acc_o[db][4 * vq + 3] * inv);
                *reinterpret_cast<uint2*>(O + db * 32 + 8 * vq + 4 * h) = w;
            }
        if (p.lse && h == 0) p.lse[(int64_t)head * Tq + qrow] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
    }
}

// ------------------------------------------------------------------------------------------------
// fp32, vector ALU: one wavefront per (query row, head), online softmax over chunks of 64 keys (one
// key per lane for the logits, head-dim values spread over lanes for the output).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_f32_kernel(const AttnParams p, int dh) {
    const int64_t wid = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    if (wid >= (int64_t)p.Hq * p.Tq) return;
    const int lane = lane_id();
    const int head = (int)(wid / p.Tq), row = (int)(wid % p.Tq);
    const int hk = head / (p.Hq / p.Hkv);
    const int64_t q_ld = (int64_t)p.Hq * dh, kv_ld = (int64_t)p.Hkv * dh;
    const float* __restrict__ q = (const float*)p.q + (int64_t)row * q_ld + (int64_t)head * dh;

    const int n_hat = p.Tn_vis;
    const int n_loc = p.causal ? row + 1 : p.Tq;
    float m_run = -INFINITY, l_run = 0.f;
    float o[4] = {0.f, 0.f, 0.f, 0.f};              // head-dim values lane, lane+64, lane+128, lane+192

    for (int src = 0; src < 2; ++src) {
        const int count = src == 0 ? n_hat : n_loc;
        const float* __restrict__ Kp = (const float*)(src == 0 ? p.k_hat : p.k_loc) + (int64_t)hk * dh;
        const float* __restrict__ Vp = (const float*)(src == 0 ? p.v_hat : p.v_loc) + (int64_t)hk * dh;
        for (int base = 0; base < count; base += kWave) {
            const int j = base + lane;
            float s = -INFINITY;
            if (j < count) {
                const float* kr = Kp + (int64_t)j * kv_ld;
                float dot = 0.f;
                for (int d = 0; d < dh; ++d) dot = fmaf(q[d], kr[d], dot);
                s = dot * p.scale;
            }
            float mx = s;
            for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
            const float m_new = fmaxf(m_run, mx);          // finite: every chunk holds at least one key
            const float alpha = expf(m_run - m_new);
            const float e = j < count ? expf(s - m_new) : 0.f;
            float sum = e;
            for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
            l_run = l_run * alpha + sum;
            m_run = m_new;
#pragma unroll
            for (int u = 0; u < 4; ++u) o[u] *= alpha;
            const int cnt = min(kWave, count - base);
            for (int jj = 0; jj < cnt; ++jj) {
                const float pj = __shfl(e, jj);
                const float* vr = Vp + (int64_t)(base + jj) * kv_ld;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int d = lane + 64 * u;
                    if (d < dh) o[u] = fmaf(pj, vr[d], o[u]);
                }
            }
        }
    }
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
    float* __restrict__ out = (float*)p.out + (int64_t)row * q_ld + (int64_t)head * dh;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int d = lane + 64 * u;
        if (d < dh) out[d] = o[u] * inv;
    }
    if (p.lse && lane == 0) p.lse[(int64_t)head * p.Tq + row] = m_run + logf(l_run);
}

int launch_attention(const astra_attn_desc& d, const void* q, const void* k_local, const void* v_local,
                     const void* k_hat, const void* v_hat, void* out, float* lse, hipStream_t s) {
    AttnParams p{};
    p.q = q; p.k_loc = k_local; p.v_loc = v_local; p.k_hat = k_hat; p.v_hat = v_hat;
    p.out = out; p.lse = lse;
    p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.Tq = d.n_cls + d.n_local;
    p.Tn_vis = d.causal ? d.n_nonlocal_before : d.n_nonlocal;
    p.causal = d.causal;
    p.scale = d.scale != 0.f ? d.scale : 1.f / sqrtf((float)d.head_dim);
    if (p.Tq == 0) return ASTRA_OK;
    if (d.dtype == ASTRA_BF16) {
        dim3 grid((unsigned)ceil_div(p.Tq, kAttQ), (unsigned)p.Hq);
        if (d.head_dim == 128) attn_bf16_kernel<128><<<grid, 256, 0, s>>>(p);
        else if (d.head_dim == 64) attn_bf16_kernel<64><<<grid, 256, 0, s>>>(p);
        else return ASTRA_ERR_UNSUPPORTED;
    } else {
        if (d.head_dim > 256) return ASTRA_ERR_UNSUPPORTED;
        const int64_t blocks = ceil_div((int64_t)p.Hq * p.Tq, 4);
        if (blocks > 0x7fffffff) return ASTRA_ERR_SHAPE;
        attn_f32_kernel<<<(int)blocks, 256, 0, s>>>(p, d.head_dim);
    }
    return launch_status();
}

}  // namespace astra
