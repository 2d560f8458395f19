/*
 * astra.h -- C ABI of the MI355X (gfx950) library for one device's share of an
 * Astra attention layer (arXiv 2505.19342): grouped vector-quantisation encode of
 * the device's local token embeddings, codebook-gather decode of its peers' codes,
 * and mixed-precision attention of local queries over full-precision local K/V
 * plus K/V projected from the decoded tokens.
 *
 * Conventions (all entry points)
 *   - Every data pointer is a DEVICE pointer to a dense row-major array, 16-byte
 *     aligned, owned by the caller.  The library allocates no memory, frees nothing
 *     and keeps no pointer after a call returns; scratch comes from `workspace`.
 *     All work of a call is enqueued on the caller's stream, in order.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work: they never synchronise, and the outputs are ready when the
 *     stream reaches that point.  Calls on distinct streams may overlap.
 *   - The return value is an astra_status.  Argument, shape and dtype errors are
 *     found on the host before anything is launched and leave outputs untouched; a
 *     failed launch returns ASTRA_ERR_HIP.  There is no CPU fallback.
 *   - Element type (`dtype`): ASTRA_F32, or ASTRA_BF16 (bf16 storage, fp32
 *     accumulation; products of two bf16 values are exact in fp32).
 *   - Codes are unpacked unsigned integers, one per (token, group): uint8 when
 *     K <= 256 (ASTRA_CODE_U8) or uint16 (ASTRA_CODE_U16, any K <= 65536).
 *   - Linear weights are stored [out_features, in_features] (the storage order of a
 *     framework linear layer): the paper's Q = X W_q is computed as x . wq^T with
 *     wq of shape [H_q*dh, D].  Both matrix-core operands are then contiguous along
 *     the contraction axis.
 *   - Zero sizes (n_tokens == 0, n_nonlocal == 0) are valid and launch nothing for
 *     the empty part.
 */
#ifndef ASTRA_H
#define ASTRA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ASTRA_OK = 0,
    ASTRA_ERR_NULL = -1,        /* a required pointer is NULL */
    ASTRA_ERR_SHAPE = -2,       /* sizes inconsistent or out of the supported range */
    ASTRA_ERR_DTYPE = -3,       /* unknown dtype / code type, or code type too narrow for K */
    ASTRA_ERR_WORKSPACE = -4,   /* workspace NULL or smaller than astra_layer_workspace_bytes */
    ASTRA_ERR_UNSUPPORTED = -5, /* valid request this build has no kernel for */
    ASTRA_ERR_HIP = -6          /* the HIP runtime refused a launch */
} astra_status;

enum { ASTRA_F32 = 0, ASTRA_BF16 = 1 };
enum { ASTRA_CODE_U8 = 0, ASTRA_CODE_U16 = 1 };

/* Grouped VQ (Sec. 2, "Grouped VQ"): the D-vector is cut into G contiguous
 * slices of dg = D / G values; slice g has its own codebook of K codewords. */
typedef struct {
    int32_t dtype;          /* element type of x, codebook, x_hat */
    int32_t code_type;      /* ASTRA_CODE_U8 requires codebook_size <= 256 */
    int32_t d_model;        /* D */
    int32_t n_groups;       /* G, must divide D */
    int32_t codebook_size;  /* K, 1 .. 65536 */
} astra_vq_desc;

/* Mixed-precision attention (Sec. 3.2, Eq. 1) for one device. */
typedef struct {
    int32_t dtype;
    int32_t n_q_heads;          /* H_q */
    int32_t n_kv_heads;         /* H_kv, divides H_q; query head h uses KV head h / (H_q / H_kv) */
    int32_t head_dim;           /* dh: 64 or 128 for bf16; any multiple of 4 up to 256 for f32 */
    int32_t n_cls;              /* 0 | 1 class-token replica, first row of the local block (Sec. 3.3);
                                   must be 0 when causal */
    int32_t n_local;            /* T_l content rows; local rows T_q = n_cls + n_local */
    int32_t n_nonlocal;         /* T_n rows rebuilt from codes */
    int32_t causal;             /* 0 | 1 */
    int32_t n_nonlocal_before;  /* causal only: non-local rows [0, nb) precede the local chunk in the
                                   sequence (all visible), rows [nb, T_n) follow it (all hidden) */
    float scale;                /* logit scale; 0 means 1 / sqrt(head_dim) */
} astra_attn_desc;

typedef struct {
    astra_vq_desc vq;
    astra_attn_desc attn;       /* attn.dtype must equal vq.dtype; H_q*dh need not equal D */
} astra_layer_desc;

/* ||c||^2 of every codeword, the codeword-only term of the expanded distance
 * ||x - c||^2 = ||x||^2 - 2 x.c + ||c||^2 (Sec. 2, "Vanilla VQ").  Run once per
 * codebook.  codebook [G, K, dg] -> cnorm_out [G, K] fp32. */
int astra_vq_prepare(const astra_vq_desc* desc, const void* codebook, float* cnorm_out, void* stream);

/* Grouped VQ encode (Sec. 2): codes_out[t, g] = argmin_k || x[t, g*dg:(g+1)*dg] - codebook[g, k, :] ||^2,
 * the lowest k among exact ties.  x [n_tokens, D]; cnorm [G, K] from astra_vq_prepare for the same
 * codebook; codes_out [n_tokens, G] of desc->code_type.  The comparison is carried out in fp32 on
 * x.c - ||c||^2 / 2, so a code can differ from exact arithmetic only where the best and second-best
 * distances agree to fp32 rounding. */
int astra_vq_encode(const astra_vq_desc* desc, const void* x, int64_t n_tokens, const void* codebook,
                    const float* cnorm, void* codes_out, void* stream);

/* astra_vq_encode with scratch memory.  For wide groups in bf16 (dg = D / G a multiple of 64 above 64, K a multiple of 8: few
 * groups, down to the vanilla VQ of Sec. 2 with G = 1, the setting of the paper's strongest compression) the distance matrix
 * of a group is a matrix product of its own: scores[t, g, k] = x[t, slice g] . codebook[g, k, :] run on the projection tile
 * kernel into workspace (fp32, n_tokens * G * K * 4 bytes), followed by one pass that picks argmin_k ||c||^2 - 2 score, lowest k
 * on ties (used when a group's codebook has at least 2^17 elements; smaller ones are faster in astra_vq_encode's kernels).
 * Same results as astra_vq_encode under the same near-tie rule; other shapes run astra_vq_encode's kernels and ignore the
 * workspace.  astra_vq_encode_workspace_bytes: the size needed (256 when unused; 0 on an invalid descriptor). */
size_t astra_vq_encode_workspace_bytes(const astra_vq_desc* desc, int64_t n_tokens);
int astra_vq_encode_ws(const astra_vq_desc* desc, const void* x, int64_t n_tokens, const void* codebook, const float* cnorm,
                       void* codes_out, void* workspace, size_t workspace_bytes, void* stream);

/* VQ decode (Sec. 3.2, "Vector-Quantized Non-Local Tokens"): x_hat_out[t, g*dg:(g+1)*dg] =
 * codebook[g, codes[t, g], :], a bit-exact copy.  A code >= K is a caller error; it is read as K-1
 * so that no access leaves the codebook. */
int astra_vq_decode(const astra_vq_desc* desc, const void* codes, int64_t n_tokens, const void* codebook,
                    void* x_hat_out, void* stream);

/* Mixed-precision attention (Eq. 1): out = softmax(q [k_local | k_hat]^T * scale) [v_local | v_hat]
 * per query head over the keys a row may see (all of them, or under `causal` the local rows j <= i and
 * the non-local rows before the chunk).  q, out [T_q, H_q, dh]; k_local, v_local [T_q, H_kv, dh];
 * k_hat, v_hat [T_n, H_kv, dh] (may be NULL when T_n == 0); lse_out nullable [H_q, T_q] fp32, the
 * natural-log softmax denominator (including the row maximum). */
int astra_mixed_attention(const astra_attn_desc* desc, const void* q,
                          const void* k_local, const void* v_local,
                          const void* k_hat, const void* v_hat,
                          void* out, float* lse_out, void* stream);

/* astra_mixed_attention when some non-local tokens' codes never arrived (Sec. 4.5 "Non-Ideal Network
 * Conditions", App. E: packet loss without retransmission; the paper does not say what the receiver does,
 * the reading here: such a token is dropped from the key/value set of every local query).
 * valid_bits: device pointer, ceil(T_n / 64) 64-bit words, bit (t % 64) of word t / 64 set iff the codes
 * of non-local token t arrived (bits at and beyond T_n are ignored); NULL = all arrived, then identical to
 * astra_mixed_attention.  The k_hat / v_hat rows of a lost token may hold anything finite. */
int astra_mixed_attention_valid(const astra_attn_desc* desc, const void* q,
                                const void* k_local, const void* v_local,
                                const void* k_hat, const void* v_hat, const uint64_t* valid_bits,
                                void* out, float* lse_out, void* stream);

/* Scratch bytes astra_layer_forward needs for this shape (0 on an invalid descriptor). */
size_t astra_layer_workspace_bytes(const astra_layer_desc* desc);

/* 1 if astra_layer_forward runs the encode of the local rows inside its projection launch for this shape
 * (Sec. 3.1: the encode and the projections are independent), 0 if as a kernel of its own, an
 * ASTRA_ERR_* code (negative) on an invalid descriptor.  Host-only, touches no device. */
int astra_layer_encode_fused(const astra_layer_desc* desc);

/* One Astra attention layer on one device (Sec. 3.1): encode the local content rows (the indices
 * this device would transmit), rebuild the peers' tokens from their codes, project local rows to
 * Q, K, V and rebuilt rows to K-hat, V-hat with the same weights, attend (Eq. 1), apply W_o.
 *   x_local         [T_q, D], class row first when n_cls == 1 (it is not encoded)
 *   codes_nonlocal  [T_n, G] in sequence order (rows before the local chunk first)
 *   codebook, cnorm as for astra_vq_encode
 *   wq [H_q*dh, D]; wk, wv [H_kv*dh, D]; wo [D, H_q*dh]; biases bq [H_q*dh], bk, bv [H_kv*dh],
 *   bo [D], each nullable
 *   y_out           [T_q, D] fp32 for BOTH element types: the output projection's fp32 accumulator is
 *                   stored unrounded (a bf16 store alone would cost |y| * 2^-9 of accuracy)
 *   codes_local_out [T_l, G]
 *   workspace       at least astra_layer_workspace_bytes(desc) bytes, 256-byte aligned
 * No residual, normalisation or positional encoding is applied. */
int astra_layer_forward(const astra_layer_desc* desc, const void* x_local, const void* codes_nonlocal,
                        const void* codebook, const float* cnorm,
                        const void* wq, const void* wk, const void* wv, const void* wo,
                        const void* bq, const void* bk, const void* bv, const void* bo,
                        void* y_out, void* codes_local_out,
                        void* workspace, size_t workspace_bytes, void* stream);

/* astra_layer_forward with lost non-local tokens: valid_nonlocal_bits as valid_bits of
 * astra_mixed_attention_valid, NULL = all arrived.  The codes_nonlocal row of a lost token may hold any
 * value of the code type (it is read as min(code, K-1) and its projections are ignored). */
int astra_layer_forward_valid(const astra_layer_desc* desc, const void* x_local, const void* codes_nonlocal,
                              const uint64_t* valid_nonlocal_bits,
                              const void* codebook, const float* cnorm,
                              const void* wq, const void* wk, const void* wv, const void* wo,
                              const void* bq, const void* bk, const void* bv, const void* bo,
                              void* y_out, void* codes_local_out,
                              void* workspace, size_t workspace_bytes, void* stream);

/* ---- the peers' K-hat, V-hat from pre-projected codebooks --------------------------------------------
 * A rebuilt row is a concatenation of codewords (Sec. 3.2, "Vector-Quantized Non-Local Tokens"), so its projection with the
 * shared W_k, W_v (text under Eq. 1) is a sum of per-group products that do not depend on the token:
 *     (X-hat W)[t, :] = sum_g codebook[g, codes[t, g], :] . W[g*dg:(g+1)*dg, :] = sum_g P[g, codes[t, g], :].
 * astra_vq_project_codebook computes P once per (codebook, weights); the layer then only gathers and adds G rows of P per
 * token and matrix.  With the paper's strongest compression, G = 1 (Tables 1, 3, 6), K-hat and V-hat are pure lookups and
 * the largest product of the layer disappears; the gather reads G * n_out * 4 bytes per token, so it pays for one or two groups.
 *   w       [n_out, D] in the element type (stored [out, in] like every weight); n_out a multiple of 8
 *   p_out   [G, K, n_out] fp32 (the unrounded accumulators; bias is not included)
 * bf16 needs dg = D / G to be a multiple of 64. */
int astra_vq_project_codebook(const astra_vq_desc* desc, const void* codebook, const void* w, int32_t n_out, float* p_out,
                              void* stream);

/* astra_layer_forward_valid with K-hat, V-hat taken from p_k, p_v = astra_vq_project_codebook(codebook, wk | wv)
 * [G, K, H_kv*dh] instead of projecting rebuilt rows: K-hat[t] = bk + sum_g p_k[g, codes_nonlocal[t, g]] (groups added in
 * ascending order in fp32, rounded once to the element type), V-hat likewise.  Everything else (encode of the local rows,
 * Q/K/V of the local rows, Eq. 1, W_o, the arguments, the workspace size) is as in astra_layer_forward_valid; wk, wv are still
 * needed for the local rows.  The caller keeps p_k, p_v consistent with codebook, wk, wv. */
int astra_layer_forward_preprojected(const astra_layer_desc* desc, const void* x_local, const void* codes_nonlocal,
                                     const uint64_t* valid_nonlocal_bits, const void* codebook, const float* cnorm,
                                     const float* p_k, const float* p_v,
                                     const void* wq, const void* wk, const void* wv, const void* wo,
                                     const void* bq, const void* bk, const void* bv, const void* bo,
                                     void* y_out, void* codes_local_out,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* astra_layer_forward with stage timing for benchmarks: identical work and results, and in addition
 * seven hipEvent_t (created by the caller with timing enabled, passed as void*; a NULL entry is skipped)
 * are recorded on `stream`: [0] at entry, [1] after the launch that computes the Q/K/V/K-hat/V-hat
 * projections, [5] and [6] before and after the encode of the local rows when it runs as a kernel of its
 * own, [2] after the attention, [3] after the output projection, [4] at exit.  Where the shape allows,
 * the encode (Sec. 3.1) runs INSIDE the projection launch, as extra workgroups on compute units the
 * projection tiles leave idle: then [5] and [6] are recorded back to back and the span [0]..[1] covers
 * both.  The attention is the span [6]..[2]. */
int astra_layer_forward_profiled(const astra_layer_desc* desc, const void* x_local, const void* codes_nonlocal,
                                 const void* codebook, const float* cnorm,
                                 const void* wq, const void* wk, const void* wv, const void* wo,
                                 const void* bq, const void* bk, const void* bv, const void* bo,
                                 void* y_out, void* codes_local_out,
                                 void* workspace, size_t workspace_bytes, void* stream,
                                 void* const* stage_events);

/* ---- the layer with keys and values quantised after projection ------------------------------------
 * App. "Memory Cost Analysis" describes Llama-3-8B with C = 2 codebooks per layer of hidden dimension
 * d = 1024 = H_kv * dh (and its 640 = 32 * 2 * 10 bits per token say the same): each device projects its
 * local rows, quantises its K rows with a K codebook and its V rows with a V codebook, transmits both code
 * streams, and looks its peers' K-hat and V-hat up directly: no projection of rebuilt rows, and the received
 * codes are what a KV cache keeps of the non-local tokens.  Eq. 1 is unchanged.
 *   vq                describes BOTH codebooks; vq.d_model must equal n_kv_heads * head_dim
 *   d_model           D, width of x_local and y_out
 *   codes_k_nonlocal, codes_v_nonlocal  [T_n, G] in sequence order; valid_nonlocal_bits as for
 *                     astra_layer_forward_valid (nullable)
 *   codebook_k/v [G, K, dkv/G], cnorm_k/v [G, K] from astra_vq_prepare
 *   y_out             [T_q, D] fp32
 *   codes_k_local_out, codes_v_local_out  [T_l, G]: codes of the content rows of K and V as stored
 *   k_out, v_out      nullable [T_q, dkv] in the element type: receive K and V of the local rows (the rows a
 *                     KV cache keeps at full precision); when NULL they live in the workspace only
 * bf16 needs dkv / G to be a multiple of 8. */
typedef struct {
    astra_vq_desc vq;
    astra_attn_desc attn;
    int32_t d_model;
} astra_layer_kv_desc;

size_t astra_layer_kv_workspace_bytes(const astra_layer_kv_desc* desc);

int astra_layer_forward_kv(const astra_layer_kv_desc* desc, const void* x_local,
                           const void* codes_k_nonlocal, const void* codes_v_nonlocal, const uint64_t* valid_nonlocal_bits,
                           const void* codebook_k, const float* cnorm_k, const void* codebook_v, const float* cnorm_v,
                           const void* wq, const void* wk, const void* wv, const void* wo,
                           const void* bq, const void* bk, const void* bv, const void* bo,
                           void* y_out, void* codes_k_local_out, void* codes_v_local_out, void* k_out, void* v_out,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ---- one decoding step over an index KV cache ------------------------------------------------------
 * App. "Memory Cost Analysis": each device keeps the keys and values of its local tokens at full precision
 * and those of the non-local tokens as VQ indices (one per group per token, the code streams of
 * astra_layer_forward_kv); Sec. 3.1: after the parallel encoding, autoregressive decoding proceeds on the
 * device that holds the most recent token.  The new token's query attends to every cached token:
 *   out[h] = softmax_t( q[h] . [K_cache | K-hat][t, h / (H_q/H_kv)] * scale ) [V_cache | V-hat],
 *   K-hat, V-hat = the rows the codes select from codebook_k, codebook_v (never materialised: key scores are
 *   sums of entries of a per-query table q . codeword, value rows are picked from the codebook).
 *   vq            both codebooks, vq.d_model = n_kv_heads * head_dim; vq.dtype = element type of q, caches,
 *                 codebooks and out; (H_kv*dh)/G and head_dim even, head_dim <= 256, H_q/H_kv <= 8
 *   q [H_q, dh]; k_cache, v_cache [n_local, H_kv, dh] (the new token's own row included by the caller);
 *   codes_k, codes_v [n_nonlocal, G]; valid_bits nullable, as for astra_mixed_attention_valid
 *   out [H_q, dh]; lse_out nullable [H_q] fp32.  With nothing to attend to, out = 0 and lse = -inf.
 *   workspace     astra_decode_attention_workspace_bytes(desc) bytes (the table and per-chunk partial results)
 * Results are independent of the run (no atomics). */
typedef struct {
    astra_vq_desc vq;
    int32_t n_q_heads, n_kv_heads, head_dim;
    int32_t n_local;
    int32_t n_nonlocal;
    float scale;                /* 0 means 1 / sqrt(head_dim) */
} astra_decode_desc;

size_t astra_decode_attention_workspace_bytes(const astra_decode_desc* desc);

int astra_decode_attention(const astra_decode_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                           const void* codes_k, const void* codes_v, const uint64_t* valid_bits,
                           const void* codebook_k, const void* codebook_v, void* out, float* lse_out,
                           void* workspace, size_t workspace_bytes, void* stream);

/* astra_decode_attention for callers that cannot allocate device memory or pass a workspace (work recorded under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation): the table and the per-chunk partial
 * results live in a scratch array that is part of the library's device image, astra_decode_attention_static_max_bytes()
 * = 8 MiB per GPU, held by every GPU the library runs on until the process ends.  Same arguments, kernels and results
 * as astra_decode_attention; the call allocates and frees nothing.  A shape whose
 * astra_decode_attention_workspace_bytes exceeds the array returns ASTRA_ERR_WORKSPACE before anything is launched
 * (the Llama-3-8B shapes of a 128 K-token cache need about 2.6 MiB).  The array's device address is looked up once
 * per device, on the first call with that device current (a caller that records calls into a HIP graph makes one call on
 * the device before it starts capturing, so that the lookup and the kernels' one-time set-up are not part of the capture);
 * a failed lookup returns ASTRA_ERR_HIP.  Nothing in the array
 * has to start at zero (every call writes what it reads), but all calls on one GPU share it: calls that overlap on one
 * GPU (different streams or threads) race; calls that follow each other on one stream do not. */
size_t astra_decode_attention_static_max_bytes(void);
int astra_decode_attention_static(const astra_decode_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                  const void* codes_k, const void* codes_v, const uint64_t* valid_bits,
                                  const void* codebook_k, const void* codebook_v, void* out, float* lse_out, void* stream);

/* ---- one whole Transformer block on one device -------------------------------------------------
 * Sec. 3.1: per block, a device quantises its local token embeddings, exchanges indices, attends with
 * the mixed-precision layer and then runs the position-wise MLP locally, without communication.  The
 * paper keeps the stock ViT / GPT-2 / Llama blocks around the layer; the pre-norm residual form of
 * those models is what this entry point computes:
 *     h     = norm1(x)                 stored in the layer's element type; h is the tensor that is
 *                                      quantised (codes_local_out) and projected
 *     r     = x + astra_layer_forward(h, ...)
 *     x_out = r + mlp(norm2(r))
 * norm_kind  ASTRA_NORM_LAYER: (v - mean) / sqrt(var + eps) * gain + bias (biased variance)
 *            ASTRA_NORM_RMS:   v / sqrt(mean(v^2) + eps) * gain (the bias pointers are ignored)
 * mlp_kind   ASTRA_MLP_GELU_TANH: fc2(gelu(fc1(v))), gelu(a) = a/2 (1 + tanh(sqrt(2/pi)(a + 0.044715 a^3)))
 *            ASTRA_MLP_GELU_ERF:  the same with gelu(a) = a/2 (1 + erf(a / sqrt 2))
 *            ASTRA_MLP_SWIGLU:    down(silu(gate(v)) * up(v)), silu(a) = a / (1 + exp(-a)); w1 holds the gate
 *                                 rows first, then the up rows
 * The residual stream (x, x_out) is fp32 for both element types; h, the MLP's hidden rows and everything
 * inside the layer use the element type (products accumulate in fp32).
 * rope_base  0: no positional encoding is applied (the paper names none).  > 0 (optional; causal layers only, head_dim
 *            even): rotary position embedding inside the layer (Su et al., "RoFormer", Eq. 34, interleaved pairs): before
 *            Eq. 1, every head's vector of Q, K and K-hat at sequence position m has its pairs (v[2i], v[2i+1]) turned by
 *            the angle m * rope_base^(-2i / head_dim); a local content row i sits at position n_nonlocal_before + i, a visible
 *            non-local row j at position j; a class row is not turned, values never are. */
enum { ASTRA_NORM_LAYER = 0, ASTRA_NORM_RMS = 1 };
enum { ASTRA_MLP_GELU_TANH = 0, ASTRA_MLP_GELU_ERF = 1, ASTRA_MLP_SWIGLU = 2 };

typedef struct {
    astra_layer_desc layer;
    int32_t norm_kind;
    int32_t mlp_kind;
    int32_t d_ff;               /* hidden width of the MLP; a multiple of 64 for bf16 */
    float eps;                  /* >= 0, inside the square root of both norms */
    float rope_base;            /* 0 = none; e.g. 10000 or 500000 */
} astra_block_desc;

/* Device pointers, owned by the caller.  Matrices and their biases are in the element type and stored
 * [out_features, in_features]; norm parameters are fp32 [D].  Nullable: every bias, the gains (= 1) and the
 * norm biases (= 0). */
typedef struct {
    const void* codebook;       /* [G, K, dg] */
    const float* cnorm;         /* [G, K] from astra_vq_prepare */
    const void *wq, *wk, *wv, *wo, *bq, *bk, *bv, *bo;      /* as for astra_layer_forward */
    const float *norm1_gain, *norm1_bias, *norm2_gain, *norm2_bias;
    const void* w1;             /* [d_ff, D], or [2 d_ff, D] for ASTRA_MLP_SWIGLU (gate rows, then up rows) */
    const void* b1;             /* [d_ff] or [2 d_ff] */
    const void* w2;             /* [D, d_ff] */
    const void* b2;             /* [D] */
} astra_block_weights;

/* Scratch bytes astra_block_forward needs (the layer's workspace included; 0 on an invalid descriptor). */
size_t astra_block_workspace_bytes(const astra_block_desc* desc);

/*   x               [T_q, D] fp32 residual stream entering the block, class row first when n_cls == 1
 *   codes_nonlocal  [T_n, G]: the peers' codes of THEIR norm1 outputs for this block
 *   valid_nonlocal_bits  nullable, as for astra_layer_forward_valid
 *   x_out           [T_q, D] fp32; may be x itself (in place)
 *   codes_local_out [T_l, G]: codes of the content rows of h
 *   h_out           nullable [T_q, D] in the element type: receives h
 *   workspace       at least astra_block_workspace_bytes(desc) bytes, 256-byte aligned
 * All shapes are validated before the first launch. */
int astra_block_forward(const astra_block_desc* desc, const astra_block_weights* weights, const float* x,
                        const void* codes_nonlocal, const uint64_t* valid_nonlocal_bits,
                        float* x_out, void* codes_local_out, void* h_out,
                        void* workspace, size_t workspace_bytes, void* stream);

/* n_layers blocks in sequence on one device's share of the model (Sec. 3.1: the model is L such blocks; between
 * two blocks the only thing a device needs from its peers is their codes for the next block).  Block l reads the
 * stream block l-1 wrote; every block has the shape `desc` and its own weights and codes:
 *   weights              HOST array of n_layers astra_block_weights (each holding device pointers)
 *   x, x_out             as for astra_block_forward (device; may alias)
 *   codes_nonlocal       HOST array of n_layers device pointers, [T_n, G] each: what the peers sent for block l
 *   valid_nonlocal_bits  NULL, or a HOST array of n_layers device pointers (entries may be NULL)
 *   codes_local_out      HOST array of n_layers device pointers, [T_l, G] each: what this device sends for block l
 *   workspace            astra_block_workspace_bytes(desc) bytes, shared by all blocks
 * Everything is validated before the first launch; the host arrays are not referenced after the call returns.
 * The distributed class token's final mean over the devices' replicas (Sec. 3.3) crosses devices and is not part
 * of this call. */
int astra_stack_forward(const astra_block_desc* desc, int32_t n_layers, const astra_block_weights* weights,
                        const float* x, const void* const* codes_nonlocal, const uint64_t* const* valid_nonlocal_bits,
                        float* x_out, void* const* codes_local_out,
                        void* workspace, size_t workspace_bytes, void* stream);

/* ---- training-side operations of the VQ module (forward arithmetic only) ---------------------------
 * Sec. 3.2: the codebook is initialised by K-means over token embeddings and updated by exponential moving average
 * during fine-tuning, with the commitment term beta * ||X - sg(X-hat)||_2^2 of Eq. 2 in the loss; Sec. 3.3: NAVQ adds
 * noise fitted to the quantisation residuals to the quantised embeddings during training.  Gradients are not part of
 * this library.  All results are independent of the run (tokens are sorted by code with a stable sort, rows added in a fixed order: no
 * floating-point atomics). */

/* Statistics of an assignment codes [T, G] (astra_vq_encode's output for x [T, D]):
 *   counts_out [G, K] int32   tokens per codeword
 *   sums_out   [G, K, dg] fp32   sum of the slices x[t, g*dg:(g+1)*dg] assigned to the codeword
 *   sqerr_out  [G] fp32       sum_t ||x[t, slice g] - codebook[g, codes[t, g]]||^2; Eq. 2's commitment term is beta times
 *                             the sum over g (the paper does not say whether it is averaged: the plain sum is returned)
 * dg <= 256 and K <= 8192.  workspace: astra_codebook_stats_workspace_bytes(desc, n_tokens) bytes. */
size_t astra_codebook_stats_workspace_bytes(const astra_vq_desc* desc, int64_t n_tokens);
int astra_codebook_stats(const astra_vq_desc* desc, const void* x, const void* codes, int64_t n_tokens, const void* codebook,
                         int32_t* counts_out, float* sums_out, float* sqerr_out,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Codebook update from those statistics.  gamma in (0, 1): ema_n [G, K] and ema_m [G, K, dg] (fp32, in place) become
 * gamma * old + (1 - gamma) * (counts | sums) and the codeword is ema_m / ema_n; gamma == 0: one K-means (Lloyd)
 * centroid step, sums / counts (ema_n, ema_m ignored, may be NULL).  A codeword whose (averaged) count is zero keeps
 * its old value (the paper gives no rule for dead codewords; no smoothing term is applied).  codebook_new_out
 * [G, K, dg] in the element type; it may be codebook_old itself. */
int astra_codebook_update(const astra_vq_desc* desc, const int32_t* counts, const float* sums, float gamma,
                          float* ema_n, float* ema_m, const void* codebook_old, void* codebook_new_out, void* stream);

/* NAVQ (Sec. 3.3): x_tilde = X-hat + lambda * xi, xi ~ N(mu, Sigma).  The standard normal draws z [T, D] are an input
 * (element type), and so is the factor: noise_factor [D, D] (element type, row-major) = lambda * L with L L^T = Sigma,
 * so that x_tilde_out[t] = codebook rows selected by codes[t] + lambda * mu + noise_factor . z[t]   (fp32 [T, D]).
 * mu [D] fp32.  bf16 needs D to be a multiple of 64. */
int astra_navq_forward(const astra_vq_desc* desc, const void* codes, int64_t n_tokens, const void* codebook,
                       const float* mu, float lambda, const void* z, const void* noise_factor,
                       float* x_tilde_out, void* stream);

/* Measurement probe, not part of the method: n_blocks workgroups of 512 threads each run `iters` rounds of
 * four independent 32x32x16 bf16 MFMAs per wavefront on register operands (no memory traffic in the loop)
 * and store one float per thread to out [n_blocks * 512] (device).  Work = n_blocks * 8 * iters * 4 * 32768
 * flop: the on-box matrix-core rate a benchmark can quote beside the published peak. */
int astra_probe_mfma_bf16(float* out, int n_blocks, int iters, void* stream);

const char* astra_status_string(int status);
int astra_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ASTRA_H */
