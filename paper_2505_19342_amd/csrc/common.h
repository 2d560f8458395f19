// Internal definitions shared by the HIP sources of the library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/astra.h"

namespace astra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16-byte register value (native vector, stays in registers)
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// ---- bf16 helpers (storage is raw 16-bit patterns) -------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {       // round to nearest even
    __bf16 h = (__bf16)f;
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// D = A(32x16) * B(16x32) + C on one wavefront.  Lane l supplies A[l%32][8*(l/32)+e] and
// B[8*(l/32)+e][l%32], e = 0..7, and holds D[8*(v/4) + 4*(l/32) + v%4][l%32] in acc[v].
__device__ __forceinline__ f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// row of the 32x32 accumulator tile held in acc[v] by a lane of half-wave h = lane / 32
__device__ __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

// 64-bit LDS transpose read: in every 16-lane group, lane s points at 4 consecutive 16-bit
// values (row s/4, columns 4*(s%4)..+3 of a 4x16 block); lane L receives column L, rows 0..3.
__device__ __forceinline__ s16x4 lds_read_tr16_b64(const void* lds_ptr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(lds_ptr));
}

// ---- direct global -> LDS transfers ------------------------------------------------------------
// byte address of a __shared__ object inside the workgroup's LDS allocation
__device__ __forceinline__ uint32_t lds_byte_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)(p);
}
// One wavefront instruction: lane L copies the 16 bytes at its own global address to LDS byte address
// lds_base + 16*L (lds_base wave-uniform).  Nothing passes through vector registers.  Completion is
// counted by vmcnt; the compiler does not know about these transfers, so the caller waits with
// wait_vmem_all() and then synchronises the workgroup before any wavefront reads the data.
__device__ __forceinline__ void dma_global_to_lds_16(const void* gptr, uint32_t lds_base) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base), "v"(gptr) : "memory", "m0");
}
// Same, with the global address split into a wave-uniform base (scalar registers) and a 32-bit byte
// offset per lane.
__device__ __forceinline__ void dma_global_to_lds_16(const void* gbase_uniform, uint32_t byte_off, uint32_t lds_base) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(base), "v"(byte_off), "s"(gbase_uniform)
                 : "memory", "m0");
}
// The waits are emitted through the compiler's own s_waitcnt builtin (gfx9 encoding: vmcnt in bits 3:0 and
// 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima = no wait), not as inline assembly: the compiler's
// wait-count bookkeeping then knows that its own earlier global loads have completed too and does not wait for
// them again inside a pipelined loop, where such a wait would also drain the transfers in flight.
__device__ __forceinline__ void wait_vmem_all() {
    __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("" ::: "memory");
}
// wait until at most N of this wavefront's vector-memory instructions (they complete in order) are outstanding
template <int N>
__device__ __forceinline__ void wait_vmem() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
    asm volatile("" ::: "memory");
}

// A 64-bit word from a wave-uniform global address through the scalar data path (a read: no vector-memory counter
// is involved, so transfers in flight are not waited for).  The caller has no LDS or scalar reads outstanding that it
// cannot afford to wait for: the wait covers them all.
__device__ __forceinline__ unsigned long long load_uniform_u64(const unsigned long long* p) {
    unsigned long long v;
    // readfirstlane returns a signed int: go through uint32_t before widening, or the low half would sign-extend
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)p);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uintptr_t)p >> 32));
    const unsigned long long* up = (const unsigned long long*)(((uintptr_t)hi << 32) | (uintptr_t)lo);
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(up) : "memory");
    return v;
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// ---- host side ---------------------------------------------------------------------------------
inline int elem_bytes(int dtype) { return dtype == ASTRA_BF16 ? 2 : 4; }
inline int code_bytes(int code_type) { return code_type == ASTRA_CODE_U16 ? 2 : 1; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int launch_status() { return hipGetLastError() == hipSuccess ? ASTRA_OK : ASTRA_ERR_HIP; }

int check_vq_desc(const astra_vq_desc* d);
int check_attn_desc(const astra_attn_desc* d);

// ---- kernels' host launchers (each returns an astra_status) ---------------------------------
int launch_vq_prepare(const astra_vq_desc& d, const void* codebook, float* cnorm, hipStream_t s);
int launch_vq_encode(const astra_vq_desc& d, const void* x, int64_t ldx, int64_t n_tokens, const void* codebook,
                     const float* cnorm, void* codes, hipStream_t s);
// wide groups (dg a multiple of 64 above 64), bf16
bool vq_encode_wide_ok(int K, int dg, int64_t ldx);
int launch_vq_encode_wide(const astra_vq_desc& d, const void* x, int64_t ldx, int64_t n_tokens, const void* codebook,
                          const float* cnorm, void* codes, hipStream_t s);
// codes[t, g] = argmin_k cnorm[g, k] - 2 scores[t, g, k] (lowest k on ties); scores fp32 [T, G, K]
int launch_vq_argmin_scores(const astra_vq_desc& d, const float* scores, const float* cnorm, int64_t n_tokens, void* codes, hipStream_t s);
int launch_vq_decode(const astra_vq_desc& d, const void* codes, int64_t n_tokens, const void* codebook,
                     void* x_hat, hipStream_t s);

int launch_vt_pack(const astra_vq_desc& d, const void* src, int64_t ld_src, const void* codes, const void* codebook, int T, int C,
                   void* dst, int ldv, hipStream_t s);
// K-hat rows (row-major) and V-hat (transposed layout) looked up from the peers' codes, and the local V rows into the transposed
// layout, as one launch (bf16)
int launch_kv_pack(const astra_vq_desc& d, const void* codes_k, const void* codes_v, const void* cb_k, const void* cb_v, const void* v_loc,
                   int T_n, int T_q, int C, void* k_hat, void* v_hat_t, int ldv_hat, void* v_loc_t, int ldv_loc, hipStream_t s);

// out[t, n] = bias[n] + sum_g P[g, codes[t, g], n] with P fp32 [G, K, N]: row-major [T, ld] in the element type, or (transposed,
// bf16) [N, ld] in the attention kernel's V^T layout
int launch_preproj_gather(int dtype, int code_type, const void* codes, const float* P, const void* bias, int T, int G, int K, int N,
                          void* dst, int ld, bool transposed, hipStream_t s);

// One C[M,N] = A[M,K] . B[N,K]^T (+ bias[N]) problem of a grouped launch.  When `codes` is set the
// rows of A are not read from `a` but rebuilt on the fly: A[m, g*dg + j] = codebook[g, codes[m, g], j].
enum { kCBf16 = 0,          // bf16, row-major [M, ldc]
       kCF32 = 1,           // fp32 (the unrounded accumulator), row-major [M, ldc]
       kCTransposedV = 2,   // bf16, C^T as [N, ldc] with the M index permuted inside blocks of 16 (see vt_pos)
       kCSwiGLU = 3 };      // B = [gate rows | up rows] ([N, K], N = 2F): C[m, f] = silu(A.gate_f) * (A.up_f), [M, ldc] of F columns
// applied to A.B^T + bias before the store (kCBf16 and kCF32 stores); the constants are those of the stock GPT-2 / ViT MLPs
enum { kActNone = 0, kActGeluTanh = 1, kActGeluErf = 2 };

struct GemmProblem {
    const void* a;
    const void* b;
    const void* bias;
    void* c;
    const void* codes;
    const void* codebook;
    int32_t M, N, K;
    int32_t lda, ldc;
    int32_t ldb;        // row stride of B in elements; 0 = K (dense rows)
    int32_t G, Kc, dg, code_bytes;
    int32_t c_mode;     // how C is stored (bf16 problems; fp32 problems always store fp32 row-major)
    int32_t act;        // kAct*
    const float* residual;   // kCF32 only, nullable: fp32 [M, ldc] added to the result (may be C itself)
};
constexpr int kMaxGemmProblems = 6;
struct EncodeJob;
// enc / enc_fused (both or neither): offers the VQ encode of the local rows to the launch; *enc_fused tells whether the
// launch took it (extra workgroups) or the caller still has to run it.  plan_only: decide and validate, launch nothing.
// split_ws: optional scratch of gemm_split_workspace_bytes() for a single fp32-output problem whose contraction is cut into slices.
int launch_gemm_batch(int dtype, const GemmProblem* problems, int n_problems, hipStream_t s, const EncodeJob* enc = nullptr,
                      bool* enc_fused = nullptr, bool plan_only = false, void* split_ws = nullptr, size_t split_ws_bytes = 0,
                      bool may_cut = true);
size_t gemm_split_workspace_bytes(int dtype, int64_t M, int64_t N, int64_t K);
extern int g_gemm_force_cfg;
extern const int g_gemm_problem_size;

// Row-wise LayerNorm (kind 0) / RMSNorm (kind 1) of the fp32 residual stream x [T, D] into the element type of the layer
// (out [T, D]); gain, bias fp32 [D], nullable.
int launch_rope(int dtype, void* mat, int64_t ld, int rows, int n_heads, int head_dim, int skip, int split, int add_lo, int add_hi,
                float base, hipStream_t s);
int launch_norm(int dtype, int kind, const float* x, int64_t T, int D, float eps, const float* gain, const float* bias, void* out,
                hipStream_t s);
// out[t, f] = silu(a[t, f]) * a[t, F + f] for fp32 a [T, 2F]
int launch_swiglu_f32(const float* a, int64_t T, int F, float* out, hipStream_t s);

struct AttnParams {
    const void* q;        // [T_q, H_q, dh]
    const void* k_loc;    // [T_q, H_kv, dh]
    const void* v_loc;    // [T_q, H_kv, dh], or transposed [H_kv*dh, ldv_loc]
    const void* k_hat;    // [T_n, H_kv, dh]
    const void* v_hat;    // [T_n, H_kv, dh], or transposed [H_kv*dh, ldv_hat]
    void* out;            // [T_q, H_q, dh]
    float* lse;           // nullable [H_q, T_q]
    int32_t Hq, Hkv, Tq;
    int32_t Tn_vis;       // visible non-local rows (all of them, or those before the chunk when causal)
    int32_t causal;
    int32_t v_transposed; // bf16 only: V buffers are V^T in the projection kernel's kCTransposedV layout
    int32_t ldv_loc, ldv_hat;   // padded token counts (multiples of 64) of the transposed V buffers
    float scale;          // logit scale
    // nullable: bit (t % 64) of word t / 64 is 1 if non-local token t's codes arrived; a token whose bit is 0 is
    // dropped from the key/value set
    const unsigned long long* valid_bits;
};
// plan_only: validate the launch (shape limits, kernel availability) and launch nothing
// enc / n_enc / enc_fused: up to two VQ encodes that nothing in the launch depends on, offered to it; *enc_fused tells whether
// the launch took them (extra workgroups in its tail) or the caller still has to run them
int launch_attention(int dtype, const AttnParams& p, int head_dim, hipStream_t s, bool plan_only = false, const EncodeJob* enc = nullptr,
                     int n_enc = 0, bool* enc_fused = nullptr);
int launch_mfma_probe(float* out, int n_blocks, int iters, hipStream_t s);

}  // namespace astra
