// One decoding step over a KV cache whose non-local part is kept as VQ indices (paper App. "Memory Cost Analysis":
// local keys and values at full precision, non-local ones as one index per group per token; Sec. 3.1: after the
// parallel encoding, decoding proceeds on the device that holds the most recent token).  The new token's query
// attends to every cached token.
//
// Three launches:
//   decode_lut_kernel      LUT[h][gi][k] = scale * q[h, slice] . codebook_k[g, k, slice] for the groups g that touch
//                          head h.  The score of a non-local token is then a sum of a few table entries picked by its
//                          key codes: no key is ever rebuilt, and the key side of the index cache costs its codes only.
//   decode_partial_kernel  one workgroup per (chunk of tokens, KV head), serving the H_q / H_kv query heads of that KV
//                          head together: scores (local: dot products on the cached rows; non-local: table sums),
//                          the chunk's softmax statistics, and the unnormalised sum of p * value rows (local rows
//                          streamed from the cache; non-local rows picked from the value codebook, which stays in L2).
//   decode_reduce_kernel   merges the chunks of every query head (log-sum-exp weights) and normalises.
// Everything is fp32 except the stored element type; results do not depend on the run (no atomics).
#include "common.h"

#include <algorithm>
#include <mutex>
#include <type_traits>

namespace astra {

struct DecodeParams {
    const void* q;
    const void* k_loc;
    const void* v_loc;
    const void* codes_k;
    const void* codes_v;
    const unsigned long long* valid_bits;
    const void* cb_k;
    const void* cb_v;
    void* out;
    float* lse;
    float* lut;      // [H_kv][n_gh][K][H_q / H_kv]
    float* part;     // [n_chunks][H_q][dh + 2]: unnormalised o, then m, l
    int32_t Hq, Hkv, dh, n_local, n_nonlocal, G, K, dg, code16, n_gh, chunk_loc, chunk_nl, n_chunks_loc, n_chunks_nl;
    int32_t aux_floats;      // floats of the LDS region shared by the query floats, the table slice and the cross-phase sums
    float scale;
};

constexpr int kDecThreads = 256;
constexpr int kDecMaxRep = 8;       // query heads per KV head served by one workgroup

template <typename T>
__device__ __forceinline__ float ldf(const T* p);
template <>
__device__ __forceinline__ float ldf<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float ldf<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }

// two consecutive elements from an address aligned to both
template <typename T>
__device__ __forceinline__ void ld2(const T* p, float& a, float& b);
template <>
__device__ __forceinline__ void ld2<float>(const float* p, float& a, float& b) {
    const float2 v = *reinterpret_cast<const float2*>(p);
    a = v.x;
    b = v.y;
}
template <>
__device__ __forceinline__ void ld2<uint16_t>(const uint16_t* p, float& a, float& b) {
    const uint32_t v = *reinterpret_cast<const uint32_t*>(p);
    a = __uint_as_float(v << 16);
    b = __uint_as_float(v & 0xffff0000u);
}

__device__ __forceinline__ int load_code(const void* codes, int code16, int64_t i, int K) {
    const int c = code16 ? (int)((const uint16_t*)codes)[i] : (int)((const uint8_t*)codes)[i];
    return c < K ? c : K - 1;
}

// CPL consecutive elements as floats; the address is aligned to the whole segment
template <typename T, int CPL>
__device__ __forceinline__ void ld_seg(const T* p, float (&o)[CPL]) {
    if constexpr (sizeof(T) == 2 && CPL == 8) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(p);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = __uint_as_float(w[i] << 16);
            o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    } else if constexpr (sizeof(T) == 2 && CPL == 2) {
        const uint32_t v = *reinterpret_cast<const uint32_t*>(p);
        o[0] = __uint_as_float(v << 16);
        o[1] = __uint_as_float(v & 0xffff0000u);
    } else if constexpr (sizeof(T) == 2 && CPL == 4) {
        const u32x2 v = *reinterpret_cast<const u32x2*>(p);
        o[0] = __uint_as_float(v.x << 16);
        o[1] = __uint_as_float(v.x & 0xffff0000u);
        o[2] = __uint_as_float(v.y << 16);
        o[3] = __uint_as_float(v.y & 0xffff0000u);
    } else if constexpr (sizeof(T) == 4 && CPL % 4 == 0) {
#pragma unroll
        for (int i = 0; i < CPL / 4; ++i) {
            const f32x4 v = reinterpret_cast<const f32x4*>(p)[i];
            o[4 * i] = v.x;
            o[4 * i + 1] = v.y;
            o[4 * i + 2] = v.z;
            o[4 * i + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < CPL; ++i) o[i] = ldf(p + i);
    }
}

// N consecutive elements kept as the 32-bit words they arrive in (bf16: two per word), unpacked where they are used: a
// row in flight then costs half the registers of its floats.  The address is aligned to the whole segment.
template <typename T, int N>
struct Seg {
    static constexpr int W = sizeof(T) == 2 ? N / 2 : N;
    uint32_t w[W];
    __device__ __forceinline__ void load(const T* p) {
        if constexpr (W % 4 == 0) {
#pragma unroll
            for (int i = 0; i < W / 4; ++i) {
                const u32x4 v = reinterpret_cast<const u32x4*>(p)[i];
                w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
            }
        } else if constexpr (W == 2) {
            const u32x2 v = *reinterpret_cast<const u32x2*>(p);
            w[0] = v.x; w[1] = v.y;
        } else {
#pragma unroll
            for (int i = 0; i < W; ++i) w[i] = reinterpret_cast<const uint32_t*>(p)[i];
        }
    }
    __device__ __forceinline__ float get(int i) const {
        if constexpr (sizeof(T) == 2) return __uint_as_float((i & 1) ? (w[i >> 1] & 0xffff0000u) : (w[i >> 1] << 16));
        else return __uint_as_float(w[i]);
    }
};

// One workgroup: 256 consecutive codewords k of one (query head, group touching its KV head).  The head's slice of q
// sits in LDS as floats; a thread reads its codeword's slice with up to 8 vector loads in flight.
template <typename T>
__global__ __launch_bounds__(kDecThreads) void decode_lut_kernel(const DecodeParams p) {
    __shared__ float qs[256];                        // dg <= dh <= 256 channels of the slice
    const int kb = (p.K + kDecThreads - 1) / kDecThreads;
    const int k = (blockIdx.x % kb) * kDecThreads + threadIdx.x;
    const int gi = (blockIdx.x / kb) % p.n_gh;
    const int h = blockIdx.x / (kb * p.n_gh);
    const int j = h / (p.Hq / p.Hkv);
    const int c_head = j * p.dh;
    const int g = c_head / p.dg + gi;
    const int lo = max(g * p.dg, c_head), hi = min((g + 1) * p.dg, c_head + p.dh);      // empty when g lies beyond the head
    const int n = max(hi - lo, 0);
    for (int c = threadIdx.x; c < n; c += kDecThreads) qs[c] = ldf((const T*)p.q + (int64_t)h * p.dh + (lo - c_head) + c);
    __syncthreads();
    if (k >= p.K) return;
    float acc = 0.f;
    if (n > 0) {
        const T* __restrict__ cw = (const T*)p.cb_k + ((int64_t)g * p.K + k) * p.dg + (lo - g * p.dg);
        const bool vec = n % 8 == 0 && (lo - g * p.dg) % 8 == 0 && p.dg % 8 == 0;
        if (vec) {
            for (int c0 = 0; c0 < n; c0 += 64) {
                float seg[8][8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (c0 + 8 * u < n) ld_seg<T, 8>(cw + c0 + 8 * u, seg[u]);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (c0 + 8 * u < n)
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc = fmaf(qs[c0 + 8 * u + e], seg[u][e], acc);
            }
        } else {
            for (int c = 0; c < n; ++c) acc = fmaf(qs[c], ldf(cw + c), acc);
        }
    }
    // the entries of the query heads that share a KV head sit side by side: a token's code picks all of them with one LDS read
    const int rep = p.Hq / p.Hkv;
    p.lut[((((int64_t)j * p.n_gh + gi) * p.K + k) * rep) + (h - j * rep)] = acc * p.scale;
}

// sum / max over each row of 16 consecutive lanes with data-parallel-primitive moves (no LDS): swap inside pairs, swap
// pairs inside quads, mirror inside half rows, mirror inside rows; afterwards every lane of the row holds the result
template <bool MAX>
__device__ __forceinline__ float row16_reduce(float v) {
    auto step = [&](auto ctrl) {
        const float w = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value, 0xF, 0xF, true));
        v = MAX ? fmaxf(v, w) : v + w;
    };
    step(std::integral_constant<int, 0xB1>{});       // quad_perm [1, 0, 3, 2]
    step(std::integral_constant<int, 0x4E>{});       // quad_perm [2, 3, 0, 1]
    step(std::integral_constant<int, 0x141>{});      // row_half_mirror
    step(std::integral_constant<int, 0x140>{});      // row_mirror
    return v;
}

constexpr int kDecRows = kDecThreads / 16;

// max / sum over the workgroup of REP values at once (two barriers); every thread gets the results
template <bool MAX, int REP>
__device__ __forceinline__ void block_reduce_multi(float (&v)[REP], float (*red)[kDecMaxRep]) {
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        v[r] = row16_reduce<MAX>(v[r]);
        // the four rows of the wavefront, read from their first lanes: pairs of rows, then the two halves
        float a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v[r]), 16 * i));
        v[r] = MAX ? fmaxf(fmaxf(a[0], a[1]), fmaxf(a[2], a[3])) : (a[0] + a[1]) + (a[2] + a[3]);
    }
    __syncthreads();                                 // earlier readers of red are done
    if ((threadIdx.x & (kWave - 1)) == 0)
#pragma unroll
        for (int r = 0; r < REP; ++r) red[threadIdx.x / kWave][r] = v[r];
    __syncthreads();
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        float t = red[0][r];
#pragma unroll
        for (int w = 1; w < kDecThreads / kWave; ++w) t = MAX ? fmaxf(t, red[w][r]) : t + red[w][r];
        v[r] = t;
    }
}

constexpr int kDecSub = 256;    // tokens per pass of a workgroup over the local cache (one per thread)
constexpr int kDecSubNl = 512;  // ... over the index cache (two per thread: half as many barriers and reductions per token)
constexpr int kDecTok = 4;      // cached rows a 16-lane group has in flight in the score pass
constexpr int kDecBatch = 8;    // value rows a thread has in flight in the value pass

// One workgroup: KV head blockIdx.y, tokens [chunk * bx, ...) of the local cache (NL = false) or of the index
// cache (NL = true), walked in passes of 256 tokens with a running maximum (the accumulated sums are rescaled when it
// grows), so a chunk may be arbitrarily long while the LDS holds one pass: s[rep][256] scores then probabilities;
// aux = the table slice [n_gh][K][rep] (index cache), at the end the cross-phase sums; cvs[256][n_gh] the value codes
// of the pass (index cache).
// DH: the head dimension when it is 64 or 128 and the codewords are cut into whole octets (then a lane of the score
// pass holds DH / 16 channels, a thread of the value pass 8, and nothing depends on the lane), or 0: any even dh <= 256,
// 16 channels per lane with the tail masked, two channels per thread in the value pass.
template <typename T, int DH, bool NL, int REP>
__device__ __forceinline__ void decode_partial_body(const DecodeParams& p, const int bx) {
    constexpr int CPL = DH ? DH / 16 : 16;           // channels per lane in the score pass (16 lanes per cached row)
    constexpr int VC = DH ? 8 : 2;                   // channels per thread in the value pass
    extern __shared__ float lds[];
    __shared__ float red[kDecRows][kDecMaxRep];
    const int tid = threadIdx.x;
    const int j = blockIdx.y;
    constexpr int rep = REP;                         // query heads per KV head (the launcher picks the instantiation)
    const int dh = DH ? DH : p.dh, dkv = p.Hkv * dh;
    const int chunk = NL ? p.chunk_nl : p.chunk_loc;
    const int t0 = bx * chunk;
    const int t1 = min(t0 + chunk, NL ? p.n_nonlocal : p.n_local);
    constexpr int SUB = NL ? kDecSubNl : kDecSub;    // tokens per pass
    constexpr int TPT = SUB / kDecThreads;           // tokens per thread and pass
    float* s = lds;                                  // [rep][SUB]
    float* aux = lds + rep * SUB;
    uint16_t* cvs = reinterpret_cast<uint16_t*>(aux + p.aux_floats);    // [SUB][n_gh]
    const int c_head = j * dh;
    const int g_lo = c_head / p.dg, g_hi = (c_head + dh - 1) / p.dg;

    // score pass ownership (local cache): lane sub of a 16-lane row holds channels [c_lo, c_lo + CPL) of q, masked beyond dh
    const int sub = tid & 15, grp = tid >> 4;
    const int c_lo = sub * CPL;
    float qf[NL ? 1 : REP][NL ? 1 : CPL];
    if (!NL) {
#pragma unroll
        for (int r = 0; r < REP; ++r)
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const float v = ldf((const T*)p.q + (int64_t)(j * rep + r) * dh + min(c_lo + c, dh - 1));
                qf[r][c] = (DH || c_lo + c < dh) ? v * p.scale : 0.f;
            }
    } else {
        const int n_tab = rep * p.n_gh * p.K;
        const f32x4* __restrict__ lut = reinterpret_cast<const f32x4*>(p.lut + (int64_t)j * n_tab);      // K % 4 == 0
        for (int i = tid; i < n_tab / 4; i += kDecThreads) reinterpret_cast<f32x4*>(aux)[i] = lut[i];
        __syncthreads();
    }

    // value pass ownership: VC adjacent channels of the head (inside one codeword: dg is a multiple of VC), rows
    // tid / hp, tid / hp + n_ph, ...
    const int tpr = dh / VC;                         // dh is a multiple of VC
    int hp = 1;
    while (hp < tpr) hp <<= 1;                       // threads per row: a power of two >= dh / VC, at most 128 for dh <= 256
    const int n_ph = kDecThreads / hp;
    const int cp = tid % hp, ph = tid / hp;
    const bool v_on = DH ? true : cp < tpr;
    const int cv0 = min(cp, tpr - 1) * VC;           // first channel of this thread inside the head
    const int gv = (c_head + cv0) / p.dg, off = c_head + cv0 - gv * p.dg;
    const T* __restrict__ vb = NL ? (const T*)p.cb_v + (int64_t)gv * p.K * p.dg + off : (const T*)p.v_loc + c_head + cv0;

    float m_run[REP], l_own[REP], acc[REP][VC];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        m_run[r] = -INFINITY;
        l_own[r] = 0.f;
#pragma unroll
        for (int e = 0; e < VC; ++e) acc[r][e] = 0.f;
    }

    // index cache: the codes (and the validity word) of a pass are fetched one pass ahead, while the previous pass gathers
    // its value codewords, when at most kDecPre groups touch a head (otherwise they are loaded where they are used)
    constexpr int kDecPre = 4;
    const int n_g = g_hi - g_lo + 1;
    const bool pre = NL && n_g <= kDecPre;
    int ck_n[TPT][NL ? kDecPre : 1], cv_n[TPT][NL ? kDecPre : 1];
    bool ok_n[TPT];
#pragma unroll
    for (int q = 0; q < TPT; ++q) ok_n[q] = true;
    // a head's codes of a token as one load when they are 4 or 8 aligned bytes (a strided 2-byte load costs the memory
    // pipeline a cache line per lane, as the wide one does)
    const int cb = p.code16 ? 2 : 1;
    const int cw_bytes = n_g * cb;
    const bool wide = NL && n_g <= kDecPre && (cw_bytes == 8 || cw_bytes == 4) && (p.G * cb) % cw_bytes == 0 && (g_lo * cb) % cw_bytes == 0;
    auto unpack_codes = [&](const void* codes, int64_t t, int (&c)[NL ? kDecPre : 1]) {
        const char* at = (const char*)codes + (t * p.G + g_lo) * cb;
        uint32_t lo = 0, hi = 0;
        if (cw_bytes == 8) {
            const u32x2 v = *reinterpret_cast<const u32x2*>(at);
            lo = v.x;
            hi = v.y;
        } else {
            lo = *reinterpret_cast<const uint32_t*>(at);
        }
        if (p.code16) {
            c[0] = lo & 0xffffu;
            if constexpr (NL) { c[1] = lo >> 16; c[2] = hi & 0xffffu; c[3] = hi >> 16; }
        } else {
            c[0] = lo & 0xffu;
            if constexpr (NL) { c[1] = (lo >> 8) & 0xffu; c[2] = (lo >> 16) & 0xffu; c[3] = lo >> 24; }
        }
#pragma unroll
        for (int gi = 0; gi < (NL ? kDecPre : 1); ++gi) c[gi] = min(c[gi], p.K - 1);
    };
    auto fetch_codes = [&](int b0) {
#pragma unroll
        for (int q = 0; q < TPT; ++q) {
            const int64_t t = min(b0 + q * kDecThreads + tid, t1 - 1);      // beyond the chunk: a repeat, unused
            if (wide) {
                unpack_codes(p.codes_k, t, ck_n[q]);
                unpack_codes(p.codes_v, t, cv_n[q]);
            } else {
#pragma unroll
                for (int gi = 0; gi < kDecPre; ++gi)
                    if (gi < n_g) {                       // the same for every thread
                        ck_n[q][gi] = load_code(p.codes_k, p.code16, t * p.G + g_lo + gi, p.K);
                        cv_n[q][gi] = load_code(p.codes_v, p.code16, t * p.G + g_lo + gi, p.K);
                    }
            }
            if (p.valid_bits) ok_n[q] = (p.valid_bits[t >> 6] >> (t & 63)) & 1ull;
        }
    };
    if constexpr (NL) {
        if (pre && t0 < t1) fetch_codes(t0);
    }

    for (int b0 = t0; b0 < t1; b0 += SUB) {
        const int nt = min(SUB, t1 - b0);
        // ---- raw scores of this pass; thread tid ends up with those of tokens b0 + tid (+ 256)
        float sc[TPT][REP];
#pragma unroll
        for (int q = 0; q < TPT; ++q)
#pragma unroll
            for (int r = 0; r < REP; ++r) sc[q][r] = -INFINITY;
        if (!NL) {
            constexpr int STEP = kDecTok * kDecRows;
#pragma unroll
            for (int tb = 0; tb < kDecSub; tb += STEP) {
                float kf[DH ? 1 : kDecTok][DH ? 1 : CPL];
                Seg<T, DH ? CPL : 2> kseg[DH ? kDecTok : 1];
#pragma unroll
                for (int u = 0; u < kDecTok; ++u) {
                    const int t = min(tb + grp + 16 * u, nt - 1);           // rows beyond the pass repeat its last row, unused
                    const T* __restrict__ kr = (const T*)p.k_loc + (int64_t)(b0 + t) * dkv + c_head;
                    if constexpr (DH != 0) {
                        kseg[u].load(kr + c_lo);
                    } else {
#pragma unroll
                        for (int c = 0; c < CPL; ++c) kf[u][c] = ldf(kr + min(c_lo + c, dh - 1));      // masked by the zeros in qf
                    }
                }
#pragma unroll
                for (int u = 0; u < kDecTok; ++u) {
                    const int t = tb + grp + 16 * u;
#pragma unroll
                    for (int r = 0; r < REP; ++r) {
                        float v = 0.f;
#pragma unroll
                        for (int c = 0; c < CPL; ++c) {
                            if constexpr (DH != 0) v = fmaf(qf[r][c], kseg[u].get(c), v);
                            else v = fmaf(qf[r][c], kf[u][c], v);
                        }
                        v = row16_reduce<false>(v);
                        s[r * SUB + t] = t < nt ? v : -INFINITY;      // all 16 lanes of the row store the same value: no branch
                    }
                }
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < REP; ++r) sc[0][r] = s[r * SUB + tid];
        } else if (pre) {
#pragma unroll
            for (int q = 0; q < TPT; ++q) {
                if (q * kDecThreads >= nt) break;         // a short pass: the same for every thread
                const int slot = q * kDecThreads + tid;
                float a[REP];
#pragma unroll
                for (int r = 0; r < REP; ++r) a[r] = 0.f;
#pragma unroll
                for (int gi = 0; gi < kDecPre; ++gi)
                    if (gi < n_g) {
                        cvs[slot * p.n_gh + gi] = (uint16_t)cv_n[q][gi];
#pragma unroll
                        for (int r = 0; r < REP; ++r) a[r] += aux[(gi * p.K + ck_n[q][gi]) * REP + r];
                    }
#pragma unroll
                for (int r = 0; r < REP; ++r)
                    if (ok_n[q] && slot < nt) sc[q][r] = a[r];
            }
        } else {
#pragma unroll
            for (int q = 0; q < TPT; ++q) {
                const int slot = q * kDecThreads + tid;
                if (slot < nt) {
                    const int64_t t = b0 + slot;
                    bool ok = true;
                    if (p.valid_bits) ok = (p.valid_bits[t >> 6] >> (t & 63)) & 1ull;
                    float a[REP];
#pragma unroll
                    for (int r = 0; r < REP; ++r) a[r] = 0.f;
                    for (int g = g_lo; g <= g_hi; ++g) {
                        const int ck = load_code(p.codes_k, p.code16, t * p.G + g, p.K);
                        cvs[slot * p.n_gh + (g - g_lo)] = (uint16_t)load_code(p.codes_v, p.code16, t * p.G + g, p.K);
#pragma unroll
                        for (int r = 0; r < REP; ++r) a[r] += aux[((g - g_lo) * p.K + ck) * REP + r];
                    }
#pragma unroll
                    for (int r = 0; r < REP; ++r)
                        if (ok) sc[q][r] = a[r];
                }
            }
        }
        // ---- running maximum, probabilities, rescale
        float mx[REP];
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            mx[r] = sc[0][r];
#pragma unroll
            for (int q = 1; q < TPT; ++q) mx[r] = fmaxf(mx[r], sc[q][r]);
        }
        block_reduce_multi<true, REP>(mx, red);          // its first barrier also orders the reads of s above before the writes below
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            const float m_new = fmaxf(m_run[r], mx[r]);
            const float alpha = m_new == -INFINITY ? 1.f : __expf(m_run[r] - m_new);      // exp(-inf) = 0 for the first pass
            l_own[r] *= alpha;
#pragma unroll
            for (int q = 0; q < TPT; ++q) {
                if (q * kDecThreads >= nt) break;
                const float pr = sc[q][r] == -INFINITY ? 0.f : __expf(sc[q][r] - m_new);
                s[r * SUB + q * kDecThreads + tid] = pr;
                l_own[r] += pr;
            }
#pragma unroll
            for (int e = 0; e < VC; ++e) acc[r][e] *= alpha;
            m_run[r] = m_new;
        }
        __syncthreads();
        if constexpr (NL) {
            if (pre && b0 + SUB < t1) fetch_codes(b0 + SUB);             // on their way during the gathers below
        }
        // ---- sum of p * value rows of this pass: kDecBatch rows in flight per thread
        if constexpr (DH != 0) {
            for (int tb = ph; tb < nt; tb += n_ph * kDecBatch) {
                Seg<T, VC> raw[kDecBatch];
#pragma unroll
                for (int u = 0; u < kDecBatch; ++u) {
                    const int t = min(tb + u * n_ph, nt - 1);                    // beyond the pass: a repeat with weight 0
                    const int64_t row = NL ? (int64_t)cvs[t * p.n_gh + (gv - g_lo)] * p.dg : (int64_t)(b0 + t) * dkv;
                    raw[u].load(vb + row);
                }
#pragma unroll
                for (int u = 0; u < kDecBatch; ++u) {
                    const int t = tb + u * n_ph;
#pragma unroll
                    for (int r = 0; r < REP; ++r) {
                        const float w = t < nt ? s[r * SUB + t] : 0.f;      // 0 for a lost token, too
#pragma unroll
                        for (int e = 0; e < VC; ++e) acc[r][e] = fmaf(w, raw[u].get(e), acc[r][e]);
                    }
                }
            }
        } else
        for (int tb = ph; tb < nt; tb += n_ph * kDecBatch) {
            float a[kDecBatch][VC];
#pragma unroll
            for (int u = 0; u < kDecBatch; ++u) {
                const int t = min(tb + u * n_ph, nt - 1);                        // beyond the pass: a repeat with weight 0
                const int64_t row = NL ? (int64_t)cvs[t * p.n_gh + (gv - g_lo)] * p.dg : (int64_t)(b0 + t) * dkv;
                ld_seg<T, VC>(vb + row, a[u]);
            }
#pragma unroll
            for (int u = 0; u < kDecBatch; ++u) {
                const int t = tb + u * n_ph;
#pragma unroll
                for (int r = 0; r < REP; ++r) {
                    const float w = t < nt ? s[r * SUB + t] : 0.f;          // 0 for a lost token, too
#pragma unroll
                    for (int e = 0; e < VC; ++e) acc[r][e] = fmaf(w, a[u][e], acc[r][e]);
                }
            }
        }
        __syncthreads();                             // s and cvs are rewritten by the next pass
    }

    // ---- chunk results: phases added in ascending order, softmax statistics
    block_reduce_multi<false, REP>(l_own, red);
    float* xs = aux;                                 // [n_ph][rep][dh]; the table is no longer needed
    if (v_on)
#pragma unroll
        for (int r = 0; r < REP; ++r)
#pragma unroll
            for (int e = 0; e < VC; ++e) xs[(ph * rep + r) * dh + cv0 + e] = acc[r][e];
    __syncthreads();
    const int chunk_id = (NL ? p.n_chunks_loc : 0) + bx;
    float* __restrict__ out = p.part + ((int64_t)chunk_id * p.Hq + (int64_t)j * rep) * (dh + 2);
    for (int i = tid; i < rep * dh; i += kDecThreads) {
        float v = 0.f;
        for (int q = 0; q < n_ph; ++q) v += xs[q * rep * dh + i];
        out[(i / dh) * (dh + 2) + (i % dh)] = v;
    }
    if (tid == 0)
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            out[r * (dh + 2) + dh] = m_run[r];
            out[r * (dh + 2) + dh + 1] = l_own[r];
        }
}

// grid.x = local chunks, then index-cache chunks: both kinds are resident together, so the streaming of the local
// rows from memory overlaps the table look-ups and codebook gathers (served by LDS and L2) of the index cache
template <typename T, int DH, int REP>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(const DecodeParams p) {
    if ((int)blockIdx.x < p.n_chunks_loc) decode_partial_body<T, DH, false, REP>(p, blockIdx.x);
    else decode_partial_body<T, DH, true, REP>(p, blockIdx.x - p.n_chunks_loc);
}

template <typename T>
__device__ __forceinline__ void st_elem(T* p, float v);
template <>
__device__ __forceinline__ void st_elem<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void st_elem<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16_bits(v); }

// gridDim.y workgroups per query head, each with its share of the head's channels (a multiple of gridDim.y): the chunks'
// statistics are combined in parallel (by every workgroup of the head for itself), then thread (c, part) sums output
// channel c over the chunks part, part + n_part, ... (several loads in flight), parts added in ascending order
template <typename T>
__global__ __launch_bounds__(kDecThreads) void decode_reduce_kernel(const DecodeParams p) {
    extern __shared__ float w_lds[];                 // [n_chunks] weights exp(m_i - M)
    __shared__ float red[kDecRows][kDecMaxRep];
    const int h = blockIdx.x, tid = threadIdx.x;
    const int n_chunks = p.n_chunks_loc + p.n_chunks_nl;
    const int64_t stride = (int64_t)p.Hq * (p.dh + 2);
    const float* __restrict__ base = p.part + (int64_t)h * (p.dh + 2);
    float v[1] = {-INFINITY};
    for (int i = tid; i < n_chunks; i += kDecThreads) {
        const float m = base[i * stride + p.dh];
        w_lds[i] = m;
        v[0] = fmaxf(v[0], m);
    }
    block_reduce_multi<true, 1>(v, red);
    const float M = v[0];
    v[0] = 0.f;
    for (int i = tid; i < n_chunks; i += kDecThreads) {
        const float m = w_lds[i];
        const float w = m == -INFINITY ? 0.f : expf(m - M);
        w_lds[i] = w;
        v[0] = fmaf(w, base[i * stride + p.dh + 1], v[0]);
    }
    block_reduce_multi<false, 1>(v, red);            // its barriers also publish w_lds
    const float L = v[0];
    // thread (c, part): channel c over the chunks i = part, part + n_part, ... (16 loads in flight); parts added in order
    const int cs = p.dh / gridDim.y, c_lo = blockIdx.y * cs;      // this workgroup's channels
    int dhp = 1;
    while (dhp < cs) dhp <<= 1;
    const int n_part = kDecThreads / dhp, c = c_lo + tid % dhp, part = tid / dhp;
    float o = 0.f;
    if (tid % dhp < cs) {
        for (int i0 = part; i0 < n_chunks; i0 += 16 * n_part) {
            float x[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) x[u] = base[(int64_t)min(i0 + u * n_part, n_chunks - 1) * stride + c];
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (i0 + u * n_part < n_chunks) o = fmaf(w_lds[i0 + u * n_part], x[u], o);
        }
    }
    __shared__ float os[kDecThreads];
    os[tid] = o;
    __syncthreads();
    if (tid < cs) {
        float t = 0.f;
        for (int q = 0; q < n_part; ++q) t += os[q * dhp + tid];
        st_elem((T*)p.out + (int64_t)h * p.dh + c_lo + tid, L > 0.f ? t / L : 0.f);
    }
    if (tid == 0 && blockIdx.y == 0 && p.lse) p.lse[h] = L > 0.f ? M + logf(L) : -INFINITY;
}

struct DecodePlan {
    int n_gh, chunk_loc, chunk_nl, n_chunks_loc, n_chunks_nl, aux_floats;
    size_t lds_loc, lds_nl, off_lut, off_part, total;
};

// a chunk length (multiple of 128) that cuts T tokens into at most max_chunks chunks
static int chunk_len(int64_t T, int64_t max_chunks) {
    if (T <= 0) return 128;
    const int64_t n = std::max<int64_t>(1, std::min(ceil_div(T, 128), max_chunks));
    return (int)(ceil_div(ceil_div(T, n), 128) * 128);
}

static int make_decode_plan(const astra_decode_desc& d, DecodePlan* pl) {
    int rc = check_vq_desc(&d.vq);
    if (rc) return rc;
    if (d.n_q_heads <= 0 || d.n_kv_heads <= 0 || d.n_q_heads % d.n_kv_heads != 0 || d.head_dim <= 0) return ASTRA_ERR_SHAPE;
    if (d.vq.d_model != d.n_kv_heads * d.head_dim || d.n_local < 0 || d.n_nonlocal < 0 || !(d.scale >= 0.f)) return ASTRA_ERR_SHAPE;
    if (d.n_local > (1 << 30) || d.n_nonlocal > (1 << 30)) return ASTRA_ERR_SHAPE;
    const int rep = d.n_q_heads / d.n_kv_heads, dg = d.vq.d_model / d.vq.n_groups;
    if ((rep != 1 && rep != 2 && rep != 4 && rep != 8) || d.head_dim > 256 || d.head_dim % 2 != 0 || dg % 2 != 0 || d.vq.codebook_size % 4 != 0)
        return ASTRA_ERR_UNSUPPORTED;
    int n_gh = 1;
    for (int j = 0; j < d.n_kv_heads; ++j) {
        const int lo = j * d.head_dim / dg, hi = ((j + 1) * d.head_dim - 1) / dg;
        n_gh = hi - lo + 1 > n_gh ? hi - lo + 1 : n_gh;
    }
    pl->n_gh = n_gh;
    // up to about two workgroups per compute unit of each kind (an index-cache chunk carries the table slice in LDS:
    // two workgroups fit a compute unit, and a stream of rows needs two to keep enough loads in flight)
    pl->chunk_loc = chunk_len(d.n_local, std::max(1, 2 * 256 / d.n_kv_heads));
    pl->chunk_nl = chunk_len(d.n_nonlocal, std::max(1, 2 * 256 / d.n_kv_heads));
    pl->n_chunks_loc = (int)ceil_div(d.n_local, pl->chunk_loc);
    pl->n_chunks_nl = (int)ceil_div(d.n_nonlocal, pl->chunk_nl);
    const size_t tab = (size_t)rep * n_gh * d.vq.codebook_size;
    const size_t xs = (size_t)rep * 8 * kDecThreads;                  // [n_ph][rep][dh] with n_ph * dh / VC <= 256 threads, VC <= 8
    const size_t qf = (size_t)rep * d.head_dim;
    pl->aux_floats = (int)std::max(tab, std::max(xs, qf));
    pl->lds_loc = ((size_t)rep * kDecSub + std::max(xs, qf)) * sizeof(float);
    pl->lds_nl = ((size_t)rep * kDecSubNl + pl->aux_floats) * sizeof(float) + align_up((size_t)kDecSubNl * n_gh * sizeof(uint16_t), 16);
    if (pl->lds_nl > 150 * 1024) return ASTRA_ERR_UNSUPPORTED;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    pl->off_lut = take((size_t)d.n_q_heads * n_gh * d.vq.codebook_size * sizeof(float));
    pl->off_part = take((size_t)(pl->n_chunks_loc + pl->n_chunks_nl) * d.n_q_heads * (d.head_dim + 2) * sizeof(float));
    pl->total = off > 0 ? off : 256;
    return ASTRA_OK;
}

template <typename T, int DH, int REP>
static int launch_partial(const DecodeParams& p, const DecodePlan& pl, hipStream_t s) {
    static bool lds_raised = false;
    if (!lds_raised) {
        // the default cap on dynamic LDS is 64 KiB
        if (hipFuncSetAttribute((const void*)decode_partial_kernel<T, DH, REP>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                150 * 1024) != hipSuccess)
            return ASTRA_ERR_HIP;
        lds_raised = true;
    }
    const int n = p.n_chunks_loc + p.n_chunks_nl;
    if (n > 0)
        decode_partial_kernel<T, DH, REP><<<dim3(n, p.Hkv), kDecThreads, p.n_chunks_nl > 0 ? pl.lds_nl : pl.lds_loc, s>>>(p);
    return ASTRA_OK;
}

template <typename T, int REP>
static int launch_partial_dh(const DecodeParams& p, const DecodePlan& pl, hipStream_t s) {
    if (p.dg % 8 == 0 && p.dh == 128) return launch_partial<T, 128, REP>(p, pl, s);
    if (p.dg % 8 == 0 && p.dh == 64) return launch_partial<T, 64, REP>(p, pl, s);
    return launch_partial<T, 0, REP>(p, pl, s);
}

template <typename T>
static int run_decode(const DecodeParams& p, const DecodePlan& pl, hipStream_t s) {
    if (p.n_chunks_nl > 0) {
        const int64_t n = (int64_t)p.Hq * p.n_gh * ceil_div(p.K, kDecThreads);
        decode_lut_kernel<T><<<(int)n, kDecThreads, 0, s>>>(p);
    }
    int rc;
    switch (p.Hq / p.Hkv) {
        case 1: rc = launch_partial_dh<T, 1>(p, pl, s); break;
        case 2: rc = launch_partial_dh<T, 2>(p, pl, s); break;
        case 4: rc = launch_partial_dh<T, 4>(p, pl, s); break;
        case 8: rc = launch_partial_dh<T, 8>(p, pl, s); break;
        default: return ASTRA_ERR_UNSUPPORTED;
    }
    if (rc) return rc;
    // long caches: a head's channels over four workgroups, so that each thread walks an eighth of the chunks, not half
    const int slices = p.dh % 4 == 0 && p.n_chunks_loc + p.n_chunks_nl > 64 ? 4 : 1;
    decode_reduce_kernel<T><<<dim3(p.Hq, slices), kDecThreads, (size_t)std::max(1, p.n_chunks_loc + p.n_chunks_nl) * sizeof(float), s>>>(p);
    return launch_status();
}

}  // namespace astra

using namespace astra;

extern "C" {

size_t astra_decode_attention_workspace_bytes(const astra_decode_desc* desc) {
    DecodePlan pl;
    if (!desc || make_decode_plan(*desc, &pl) != ASTRA_OK) return 0;
    return pl.total;
}

// Scratch of astra_decode_attention_static: one copy per GPU, held until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress; kernels and the entry point use the per-device address kept below.
constexpr size_t kDecodeStaticBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kDecodeStaticBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_addr[kMaxDevices];          // device address of `scratch` on device i, looked up on first use
static std::mutex g_scratch_mutex;

static int decode_static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ASTRA_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_addr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return ASTRA_ERR_HIP;
        }
        g_scratch_addr[dev] = ptr;
    }
    *out = g_scratch_addr[dev];
    return ASTRA_OK;
}

static int decode_attention_impl(const astra_decode_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                 const void* codes_k, const void* codes_v, const uint64_t* valid_bits, const void* codebook_k,
                                 const void* codebook_v, void* out, float* lse_out, void* workspace, size_t workspace_bytes,
                                 bool library_scratch, void* stream) {
    if (!desc) return ASTRA_ERR_NULL;
    DecodePlan pl;
    int rc = make_decode_plan(*desc, &pl);
    if (rc) return rc;
    if (!q || !out) return ASTRA_ERR_NULL;
    if (desc->n_local > 0 && (!k_cache || !v_cache)) return ASTRA_ERR_NULL;
    if (desc->n_nonlocal > 0 && (!codes_k || !codes_v || !codebook_k || !codebook_v)) return ASTRA_ERR_NULL;
    if (library_scratch) {
        if (pl.total > kDecodeStaticBytes) return ASTRA_ERR_WORKSPACE;
        rc = decode_static_scratch(&workspace);
        if (rc) return rc;
    } else if (!workspace || workspace_bytes < pl.total) {
        return ASTRA_ERR_WORKSPACE;
    }
    DecodeParams p{};
    p.q = q; p.k_loc = k_cache; p.v_loc = v_cache; p.codes_k = codes_k; p.codes_v = codes_v;
    p.valid_bits = (const unsigned long long*)valid_bits;
    p.cb_k = codebook_k; p.cb_v = codebook_v; p.out = out; p.lse = lse_out;
    p.lut = (float*)((char*)workspace + pl.off_lut);
    p.part = (float*)((char*)workspace + pl.off_part);
    p.Hq = desc->n_q_heads; p.Hkv = desc->n_kv_heads; p.dh = desc->head_dim;
    p.n_local = desc->n_local; p.n_nonlocal = desc->n_nonlocal;
    p.G = desc->vq.n_groups; p.K = desc->vq.codebook_size; p.dg = desc->vq.d_model / desc->vq.n_groups;
    p.code16 = desc->vq.code_type == ASTRA_CODE_U16 ? 1 : 0;
    p.n_gh = pl.n_gh; p.chunk_loc = pl.chunk_loc; p.chunk_nl = pl.chunk_nl; p.n_chunks_loc = pl.n_chunks_loc; p.n_chunks_nl = pl.n_chunks_nl;
    p.aux_floats = pl.aux_floats;
    p.scale = desc->scale != 0.f ? desc->scale : 1.f / sqrtf((float)desc->head_dim);
    if (desc->vq.dtype == ASTRA_BF16) return run_decode<uint16_t>(p, pl, (hipStream_t)stream);
    return run_decode<float>(p, pl, (hipStream_t)stream);
}

int astra_decode_attention(const astra_decode_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                           const void* codes_k, const void* codes_v, const uint64_t* valid_bits, const void* codebook_k,
                           const void* codebook_v, void* out, float* lse_out, void* workspace, size_t workspace_bytes,
                           void* stream) {
    return decode_attention_impl(desc, q, k_cache, v_cache, codes_k, codes_v, valid_bits, codebook_k, codebook_v, out, lse_out,
                                 workspace, workspace_bytes, false, stream);
}

size_t astra_decode_attention_static_max_bytes(void) { return kDecodeStaticBytes; }

int astra_decode_attention_static(const astra_decode_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                  const void* codes_k, const void* codes_v, const uint64_t* valid_bits, const void* codebook_k,
                                  const void* codebook_v, void* out, float* lse_out, void* stream) {
    return decode_attention_impl(desc, q, k_cache, v_cache, codes_k, codes_v, valid_bits, codebook_k, codebook_v, out, lse_out,
                                 nullptr, 0, true, stream);
}

}  // extern "C"
