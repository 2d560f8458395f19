/*
 * CPU oracle for one device's share of an Astra attention layer.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is the slow, plain, fp64
 * statement of what the GPU path must compute, written from the paper's
 * definitions.  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg may load it.  It shares no source, header, table or helper with the HIP
 * library and never calls it.
 *
 * All arithmetic is IEEE double.  Inputs arrive as float arrays that hold the
 * exact bits given to the GPU (for bf16 workloads they are bf16-representable
 * values widened to float); nothing is rounded between steps.
 *
 * What each function follows:
 *   oracle_vq_encode        Sec. 2 "Vanilla VQ" (i = argmin_i ||e_i - z||^2) and
 *                           "Grouped VQ" (G equal sub-vectors, one codebook each)
 *   oracle_vq_decode        Sec. 3.2 "Vector-Quantized Non-Local Tokens"
 *                           (receiver rebuilds X-hat from the index alone)
 *   oracle_linear           the linear projections named under Eq. 1
 *   oracle_mixed_attention  Sec. 3.2 Eq. 1, sigma(Q [K | K-hat]^T / sqrt(d_k)) [V | V-hat]
 *   oracle_layer_forward    Sec. 3.1 (per-block procedure on one device)
 *   oracle_block_forward    Sec. 3.1, the whole block: norms, residuals and the local MLP around the layer
 *   oracle_rope, *_rope     optional rotary position embedding (outside the paper; Su et al., RoFormer, Eq. 34)
 *   oracle_layer_forward_kv the layer with K and V quantised after projection (App. memory cost: C = 2, d = 1024)
 *   oracle_decode_attention one decoding step over a KV cache whose non-local part is VQ indices (App. memory cost)
 *   oracle_codebook_stats / oracle_codebook_update / oracle_navq   training-side VQ operations (Sec. 3.2, Eq. 2, Sec. 3.3)
 *
 * Readings taken where the paper is silent (they are the library's too):
 *   - groups are contiguous slices [g*dg, (g+1)*dg) of the D-vector;
 *   - argmin ties go to the lowest index;
 *   - the mask M of Eq. 1 excludes a (query, key) pair from the softmax, it
 *     does not multiply a logit by zero; at inference it carries causality only;
 *   - causality is on global positions with contiguous chunks, so non-local
 *     rows [0, n_before) precede the local chunk (all visible) and rows
 *     [n_before, T_n) follow it (all hidden);
 *   - multi-head: Eq. 1 per head with d_k = head_dim; grouped-query attention
 *     shares KV head h / (H_q / H_kv) among consecutive query heads;
 *   - a class-token replica is an ordinary full-precision local row placed
 *     first; it is not encoded;
 *   - (Sec. 4.5 "Non-Ideal Network Conditions", App. E: packet loss without retransmission; the paper does not
 *     say what the receiver does) a non-local token whose codes never arrived is
 *     dropped from the key/value set of every local query: the *_valid variants.
 *
 * Parity pins live in tests/ (brute force, closed forms, library routines,
 * invariants).  The numerical outputs of the authors' trained models are
 * "parity unpinned": the paper prints no worked code or attention value.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Grouped VQ encode.  x [T, D], codebook [G, K, D/G], codes [T, G].
 * gap (nullable) [T, G] = (second-best - best) / best squared distance, the
 * quantity the near-tie report is defined on.  Returns 0, or -1 on bad shape. */
int oracle_vq_encode(const float* x, int64_t T, int D, int G, int K,
                     const float* codebook, int32_t* codes, double* gap) {
    if (T < 0 || D <= 0 || G <= 0 || K <= 0 || D % G != 0) return -1;
    const int dg = D / G;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int g = 0; g < G; ++g) {
            const float* z = x + t * (int64_t)D + (int64_t)g * dg;
            double best = INFINITY, second = INFINITY;
            int arg = -1;
            for (int k = 0; k < K; ++k) {
                const float* e = codebook + ((int64_t)g * K + k) * dg;
                double dist = 0.0;
                for (int j = 0; j < dg; ++j) {
                    const double diff = (double)e[j] - (double)z[j];
                    dist += diff * diff;
                }
                if (dist < best) {          /* strict: equal distance keeps the lower index */
                    second = best;
                    best = dist;
                    arg = k;
                } else if (dist < second) {
                    second = dist;
                }
            }
            codes[t * (int64_t)G + g] = arg;
            if (gap) {
                const double den = best > DBL_MIN ? best : DBL_MIN;
                gap[t * (int64_t)G + g] = (K > 1) ? (second - best) / den : INFINITY;
            }
        }
    }
    return 0;
}

/* Codebook lookup.  codes [T, G] -> x_hat [T, D]; values are copied, never
 * recomputed.  Returns -2 if a code is outside [0, K). */
int oracle_vq_decode(const int32_t* codes, int64_t T, int D, int G, int K,
                     const float* codebook, float* x_hat) {
    if (T < 0 || D <= 0 || G <= 0 || K <= 0 || D % G != 0) return -1;
    const int dg = D / G;
    for (int64_t i = 0; i < T * (int64_t)G; ++i)
        if (codes[i] < 0 || codes[i] >= K) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int g = 0; g < G; ++g) {
            const float* e = codebook + ((int64_t)g * K + codes[t * (int64_t)G + g]) * dg;
            memcpy(x_hat + t * (int64_t)D + (int64_t)g * dg, e, sizeof(float) * dg);
        }
    return 0;
}

/* out[t, o] = sum_i x[t, i] * w[i, o] + bias[o].  w is [D_in, D_out] as in
 * Q = X W_q; bias nullable. */
int oracle_linear(const double* x, int64_t T, int d_in, int d_out,
                  const float* w, const float* bias, double* out) {
    if (T < 0 || d_in <= 0 || d_out <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        double* o = out + t * (int64_t)d_out;
        for (int c = 0; c < d_out; ++c) o[c] = 0.0;
        for (int i = 0; i < d_in; ++i) {
            const double xi = x[t * (int64_t)d_in + i];
            const float* wr = w + (int64_t)i * d_out;
            for (int c = 0; c < d_out; ++c) o[c] += xi * (double)wr[c];
        }
        if (bias)
            for (int c = 0; c < d_out; ++c) o[c] += (double)bias[c];
    }
    return 0;
}

/* Eq. 1 for the T_q = n_cls + n_local local rows of one device.
 *   q            [T_q, H_q, dh]
 *   k_loc, v_loc [T_q, H_kv, dh]   full-precision local keys / values
 *   k_hat, v_hat [T_n, H_kv, dh]   keys / values projected from decoded tokens
 *   out          [T_q, H_q, dh]
 *   lse (nullable)   [H_q, T_q]    log of the softmax denominator (natural log, incl. the max)
 *   probs (nullable) [H_q, T_q, T_q + T_n]  the softmax row, local keys first as in [K | K-hat];
 *                                            excluded pairs hold 0
 * Allowed keys of local row i: not causal -> every local and non-local row;
 * causal -> local rows j <= i and non-local rows t < n_before. */
int oracle_mixed_attention_valid(const double* q, const double* k_loc, const double* v_loc,
                                 const double* k_hat, const double* v_hat, const uint8_t* valid_hat,
                                 int n_q_heads, int n_kv_heads, int head_dim,
                                 int n_cls, int n_local, int n_nonlocal,
                                 int causal, int n_before, double scale,
                                 double* out, double* lse, double* probs) {
    if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0 || head_dim <= 0) return -1;
    if (n_cls < 0 || n_local < 0 || n_nonlocal < 0) return -1;
    if (causal && (n_cls != 0 || n_before < 0 || n_before > n_nonlocal)) return -1;
    const int Tq = n_cls + n_local, Tn = n_nonlocal, Tk = Tq + Tn;
    const int rep = n_q_heads / n_kv_heads;
    if (scale == 0.0) scale = 1.0 / sqrt((double)head_dim);
    const int64_t rows = (int64_t)n_q_heads * Tq;
#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (Tk > 0 ? Tk : 1));
        char* allowed = (char*)malloc(Tk > 0 ? Tk : 1);
#pragma omp for schedule(dynamic, 8)
        for (int64_t r = 0; r < rows; ++r) {
            const int h = (int)(r / Tq), i = (int)(r % Tq);
            const int hk = h / rep;
            const double* qi = q + ((int64_t)i * n_q_heads + h) * head_dim;
            /* logits over the concatenation [K | K-hat] */
            double smax = -INFINITY;
            for (int j = 0; j < Tk; ++j) {
                const int is_local = j < Tq;
                const int jj = is_local ? j : j - Tq;
                allowed[j] = !causal ? 1 : (is_local ? (jj <= i) : (jj < n_before));
                if (!is_local && valid_hat && !valid_hat[jj]) allowed[j] = 0;      /* code never arrived: the key is dropped */
                if (!allowed[j]) continue;
                const double* kj = (is_local ? k_loc : k_hat) + ((int64_t)jj * n_kv_heads + hk) * head_dim;
                double dot = 0.0;
                for (int d = 0; d < head_dim; ++d) dot += qi[d] * kj[d];
                s[j] = dot * scale;
                if (s[j] > smax) smax = s[j];
            }
            double denom = 0.0;
            for (int j = 0; j < Tk; ++j)
                if (allowed[j]) { s[j] = exp(s[j] - smax); denom += s[j]; }
            double* o = out + ((int64_t)i * n_q_heads + h) * head_dim;
            for (int d = 0; d < head_dim; ++d) o[d] = 0.0;
            for (int j = 0; j < Tk; ++j) {
                const double p = allowed[j] ? s[j] / denom : 0.0;
                if (probs) probs[((int64_t)h * Tq + i) * Tk + j] = p;
                if (!allowed[j]) continue;
                const int is_local = j < Tq;
                const int jj = is_local ? j : j - Tq;
                const double* vj = (is_local ? v_loc : v_hat) + ((int64_t)jj * n_kv_heads + hk) * head_dim;
                for (int d = 0; d < head_dim; ++d) o[d] += p * vj[d];
            }
            if (lse) lse[(int64_t)h * Tq + i] = smax + log(denom);
        }
        free(s);
        free(allowed);
    }
    return 0;
}

/* Eq. 1 with every non-local code present. */
int oracle_mixed_attention(const double* q, const double* k_loc, const double* v_loc,
                           const double* k_hat, const double* v_hat,
                           int n_q_heads, int n_kv_heads, int head_dim,
                           int n_cls, int n_local, int n_nonlocal,
                           int causal, int n_before, double scale,
                           double* out, double* lse, double* probs) {
    return oracle_mixed_attention_valid(q, k_loc, v_loc, k_hat, v_hat, NULL, n_q_heads, n_kv_heads, head_dim,
                                        n_cls, n_local, n_nonlocal, causal, n_before, scale, out, lse, probs);
}

/* Rotary position embedding (not part of the paper, which never says how its Llama-shaped model encodes positions; the
 * published definition of Su et al., "RoFormer", Sec. 3.2.2, Eq. 34, in its original interleaved pairing): every head's
 * vector x of head_dim values at sequence position m is rotated pair by pair,
 *     (x[2i], x[2i+1]) -> (x[2i] cos(m t_i) - x[2i+1] sin(m t_i),  x[2i] sin(m t_i) + x[2i+1] cos(m t_i)),   t_i = base^(-2i / head_dim).
 * mat [rows, n_heads * head_dim] in place; pos[r] = position of row r, a negative value leaves the row as it is. */
int oracle_rope(double* mat, int64_t rows, int n_heads, int head_dim, const int64_t* pos, double base) {
    if (head_dim <= 0 || head_dim % 2 != 0 || n_heads <= 0 || !(base > 0.0)) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        if (pos[r] < 0) continue;
        for (int h = 0; h < n_heads; ++h) {
            double* x = mat + (r * n_heads + h) * head_dim;
            for (int i = 0; i < head_dim / 2; ++i) {
                const double theta = pow(base, -2.0 * (double)i / (double)head_dim);
                const double a = (double)pos[r] * theta;
                const double c = cos(a), sn = sin(a);
                const double x0 = x[2 * i], x1 = x[2 * i + 1];
                x[2 * i] = x0 * c - x1 * sn;
                x[2 * i + 1] = x0 * sn + x1 * c;
            }
        }
    }
    return 0;
}

/* One Astra attention layer on one device (Sec. 3.1):
 *   codes_local = encode(content rows of x_local)        -> what this device transmits
 *   X-hat       = decode(codes_nonlocal)                  -> what it rebuilds from its peers
 *   Q, K, V     = x_local W_q, x_local W_k, x_local W_v   (full precision)
 *   K-hat,V-hat = X-hat W_k, X-hat W_v                     (same weights)
 *   Y           = Attn(Q, K, K-hat, V, V-hat) W_o
 * x_local [T_q, D] with the class row (if any) first; weights [D_in, D_out];
 * biases nullable.  y [T_q, D] double, codes_local [n_local, G], gap nullable.
 * rope_base > 0 (optional, outside the paper): Q, K and K-hat are rotated by oracle_rope before the attention, every row
 * at its position in the whole sequence: local content row i at n_before + i, non-local row j at j when it precedes the
 * local chunk (j < n_before) and at j + n_local otherwise; a class row has no position and is not rotated. */
int oracle_layer_forward_rope(const float* x_local, const int32_t* codes_nonlocal, const uint8_t* valid_nonlocal,
                              const float* codebook, int D, int G, int K,
                              const float* wq, const float* wk, const float* wv, const float* wo,
                              const float* bq, const float* bk, const float* bv, const float* bo,
                              int n_q_heads, int n_kv_heads, int head_dim,
                              int n_cls, int n_local, int n_nonlocal,
                              int causal, int n_before, double scale, double rope_base,
                              double* y, int32_t* codes_local, double* gap_local) {
    const int Tq = n_cls + n_local, Tn = n_nonlocal;
    const int dq = n_q_heads * head_dim, dkv = n_kv_heads * head_dim;
    int rc = oracle_vq_encode(x_local + (int64_t)n_cls * D, n_local, D, G, K, codebook,
                              codes_local, gap_local);
    if (rc) return rc;

    float* x_hat = (float*)malloc(sizeof(float) * ((int64_t)Tn * D + 1));
    if (!valid_nonlocal) {
        rc = oracle_vq_decode(codes_nonlocal, Tn, D, G, K, codebook, x_hat);
    } else {
        /* a row whose codes never arrived is not looked up (whatever sits in its slot is ignored); it is left
         * zero and excluded from the attention below */
        for (int64_t t = 0; t < Tn && !rc; ++t) {
            if (valid_nonlocal[t]) rc = oracle_vq_decode(codes_nonlocal + t * G, 1, D, G, K, codebook, x_hat + t * (int64_t)D);
            else memset(x_hat + t * (int64_t)D, 0, sizeof(float) * D);
        }
    }
    if (rc) { free(x_hat); return rc; }

    double* xl = (double*)malloc(sizeof(double) * ((int64_t)Tq * D + 1));
    double* xh = (double*)malloc(sizeof(double) * ((int64_t)Tn * D + 1));
    for (int64_t i = 0; i < (int64_t)Tq * D; ++i) xl[i] = (double)x_local[i];
    for (int64_t i = 0; i < (int64_t)Tn * D; ++i) xh[i] = (double)x_hat[i];
    double* Q = (double*)malloc(sizeof(double) * ((int64_t)Tq * dq + 1));
    double* Kl = (double*)malloc(sizeof(double) * ((int64_t)Tq * dkv + 1));
    double* Vl = (double*)malloc(sizeof(double) * ((int64_t)Tq * dkv + 1));
    double* Kh = (double*)malloc(sizeof(double) * ((int64_t)Tn * dkv + 1));
    double* Vh = (double*)malloc(sizeof(double) * ((int64_t)Tn * dkv + 1));
    double* O = (double*)malloc(sizeof(double) * ((int64_t)Tq * dq + 1));
    oracle_linear(xl, Tq, D, dq, wq, bq, Q);
    oracle_linear(xl, Tq, D, dkv, wk, bk, Kl);
    oracle_linear(xl, Tq, D, dkv, wv, bv, Vl);
    oracle_linear(xh, Tn, D, dkv, wk, bk, Kh);
    oracle_linear(xh, Tn, D, dkv, wv, bv, Vh);
    if (rope_base > 0.0) {
        int64_t* pos = (int64_t*)malloc(sizeof(int64_t) * ((int64_t)Tq + Tn + 1));
        for (int i = 0; i < Tq; ++i) pos[i] = i < n_cls ? -1 : (int64_t)n_before + (i - n_cls);
        for (int j = 0; j < Tn; ++j) pos[Tq + j] = j < n_before ? j : (int64_t)j + n_local;
        rc = oracle_rope(Q, Tq, n_q_heads, head_dim, pos, rope_base);
        if (!rc) rc = oracle_rope(Kl, Tq, n_kv_heads, head_dim, pos, rope_base);
        if (!rc) rc = oracle_rope(Kh, Tn, n_kv_heads, head_dim, pos + Tq, rope_base);
        free(pos);
    }
    if (!rc)
        rc = oracle_mixed_attention_valid(Q, Kl, Vl, Kh, Vh, valid_nonlocal, n_q_heads, n_kv_heads, head_dim,
                                          n_cls, n_local, n_nonlocal, causal, n_before, scale,
                                          O, NULL, NULL);
    if (!rc) oracle_linear(O, Tq, dq, D, wo, bo, y);
    free(x_hat); free(xl); free(xh); free(Q); free(Kl); free(Vl); free(Kh); free(Vh); free(O);
    return rc;
}

/* The layer as the paper states it (no positional rotation). */
int oracle_layer_forward_valid(const float* x_local, const int32_t* codes_nonlocal, const uint8_t* valid_nonlocal,
                               const float* codebook, int D, int G, int K,
                         const float* wq, const float* wk, const float* wv, const float* wo,
                         const float* bq, const float* bk, const float* bv, const float* bo,
                         int n_q_heads, int n_kv_heads, int head_dim,
                         int n_cls, int n_local, int n_nonlocal,
                         int causal, int n_before, double scale,
                         double* y, int32_t* codes_local, double* gap_local) {
    return oracle_layer_forward_rope(x_local, codes_nonlocal, valid_nonlocal, codebook, D, G, K, wq, wk, wv, wo, bq, bk, bv, bo,
                                     n_q_heads, n_kv_heads, head_dim, n_cls, n_local, n_nonlocal, causal, n_before, scale, 0.0,
                                     y, codes_local, gap_local);
}

/* The layer with every non-local code present. */
int oracle_layer_forward(const float* x_local, const int32_t* codes_nonlocal,
                         const float* codebook, int D, int G, int K,
                         const float* wq, const float* wk, const float* wv, const float* wo,
                         const float* bq, const float* bk, const float* bv, const float* bo,
                         int n_q_heads, int n_kv_heads, int head_dim,
                         int n_cls, int n_local, int n_nonlocal,
                         int causal, int n_before, double scale,
                         double* y, int32_t* codes_local, double* gap_local) {
    return oracle_layer_forward_valid(x_local, codes_nonlocal, NULL, codebook, D, G, K, wq, wk, wv, wo, bq, bk, bv, bo,
                                      n_q_heads, n_kv_heads, head_dim, n_cls, n_local, n_nonlocal, causal, n_before,
                                      scale, y, codes_local, gap_local);
}

/* ------------------------------------------------------------------------------------------------
 * One whole Transformer block on one device (Sec. 3.1: "Within each Transformer block ..." — local
 * quantisation, exchange of indices, mixed-precision attention, then the position-wise MLP, "executed
 * locally on each device without communication").  The paper uses the stock ViT / GPT-2 / Llama blocks
 * and does not restate them; the pre-norm residual form of those models is taken:
 *     h   = norm1(x)                      the tensor that feeds the projections is the one quantised
 *     r   = x + layer(h)                  layer = oracle_layer_forward (Eq. 1 and W_o)
 *     out = r + mlp(norm2(r))
 * norm_kind 0: LayerNorm  (x - mean) / sqrt(var + eps) * gain + bias   (biased variance over the row)
 *           1: RMSNorm    x / sqrt(mean(x^2) + eps) * gain
 * mlp_kind  0: fc2(gelu_tanh(fc1(h)))   gelu_tanh(a) = a/2 (1 + tanh(sqrt(2/pi) (a + 0.044715 a^3)))   (GPT-2)
 *           1: fc2(gelu_erf(fc1(h)))    gelu_erf(a)  = a/2 (1 + erf(a / sqrt 2))                        (ViT)
 *           2: down(silu(gate(h)) * up(h)),  silu(a) = a / (1 + exp(-a)); w1 = [W_gate | W_up] as
 *              [D, 2 d_ff] (gate columns first), no biases needed                                      (Llama)
 * No rotary or learned positional encoding is applied.
 * ------------------------------------------------------------------------------------------------ */
int oracle_norm(const double* x, int64_t T, int D, int norm_kind, double eps,
                const float* gain, const float* bias, double* out) {
    if (T < 0 || D <= 0 || (norm_kind != 0 && norm_kind != 1)) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double* r = x + t * (int64_t)D;
        double* o = out + t * (int64_t)D;
        double mean = 0.0;
        if (norm_kind == 0) {
            for (int i = 0; i < D; ++i) mean += r[i];
            mean /= D;
        }
        double var = 0.0;
        for (int i = 0; i < D; ++i) var += (r[i] - mean) * (r[i] - mean);
        var /= D;
        const double inv = 1.0 / sqrt(var + eps);
        for (int i = 0; i < D; ++i) {
            double v = (r[i] - mean) * inv;
            if (gain) v *= (double)gain[i];
            if (norm_kind == 0 && bias) v += (double)bias[i];
            o[i] = v;
        }
    }
    return 0;
}

static double act_gelu_tanh(double a) { return 0.5 * a * (1.0 + tanh(0.7978845608028654 * (a + 0.044715 * a * a * a))); }
static double act_gelu_erf(double a) { return 0.5 * a * (1.0 + erf(a * 0.7071067811865476)); }
static double act_silu(double a) { return a / (1.0 + exp(-a)); }

/* h [T, D] -> out [T, D].  w1 [D, d_ff] (kinds 0, 1) or [D, 2 d_ff] (kind 2); w2 [d_ff, D]. */
int oracle_mlp(const double* h, int64_t T, int D, int d_ff, int mlp_kind,
               const float* w1, const float* b1, const float* w2, const float* b2, double* out) {
    if (T < 0 || D <= 0 || d_ff <= 0 || mlp_kind < 0 || mlp_kind > 2) return -1;
    const int n1 = mlp_kind == 2 ? 2 * d_ff : d_ff;
    double* a = (double*)malloc(sizeof(double) * ((int64_t)T * n1 + 1));
    double* g = (double*)malloc(sizeof(double) * ((int64_t)T * d_ff + 1));
    int rc = oracle_linear(h, T, D, n1, w1, b1, a);
    if (!rc) {
        for (int64_t t = 0; t < T; ++t)
            for (int j = 0; j < d_ff; ++j) {
                const double v = a[t * (int64_t)n1 + j];
                double r;
                if (mlp_kind == 0) r = act_gelu_tanh(v);
                else if (mlp_kind == 1) r = act_gelu_erf(v);
                else r = act_silu(v) * a[t * (int64_t)n1 + d_ff + j];
                g[t * (int64_t)d_ff + j] = r;
            }
        rc = oracle_linear(g, T, d_ff, D, w2, b2, out);
    }
    free(a);
    free(g);
    return rc;
}

/* x [T_q, D] fp64 residual stream in, x_out [T_q, D] out.  The normalised tensor h = norm1(x) is rounded to the
 * element type the layer's inputs have (h_is_bf16: bf16, round to nearest even; else fp32) before it enters the
 * layer: an argmin is decided on it, and both sides must take that decision on the same values.  h_out (nullable)
 * returns that tensor, which is what this device's peers would receive the codes of. */
int oracle_block_forward_rope(const double* x, const int32_t* codes_nonlocal, const uint8_t* valid_nonlocal,
                              const float* codebook, int D, int G, int K,
                              int norm_kind, double eps, const float* g1, const float* be1, const float* g2, const float* be2,
                              const float* wq, const float* wk, const float* wv, const float* wo,
                              const float* bq, const float* bk, const float* bv, const float* bo,
                              int mlp_kind, int d_ff, const float* w1, const float* b1, const float* w2, const float* b2,
                              int n_q_heads, int n_kv_heads, int head_dim,
                              int n_cls, int n_local, int n_nonlocal, int causal, int n_before, double scale,
                              int h_is_bf16, double rope_base,
                              double* x_out, int32_t* codes_local, double* gap_local, float* h_out) {
    const int Tq = n_cls + n_local;
    const int64_t n = (int64_t)Tq * D;
    double* h = (double*)malloc(sizeof(double) * (n + 1));
    float* hf = (float*)malloc(sizeof(float) * (n + 1));
    double* y = (double*)malloc(sizeof(double) * (n + 1));
    double* r = (double*)malloc(sizeof(double) * (n + 1));
    double* m = (double*)malloc(sizeof(double) * (n + 1));
    int rc = oracle_norm(x, Tq, D, norm_kind, eps, g1, be1, h);
    if (!rc) {
        /* the layer takes its input in the device's element type */
        for (int64_t i = 0; i < n; ++i) {
            float f = (float)h[i];
            if (h_is_bf16) {
                uint32_t u;
                memcpy(&u, &f, 4);
                if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);      /* round to nearest even */
                u &= 0xffff0000u;
                memcpy(&f, &u, 4);
            }
            hf[i] = f;
        }
        if (h_out) memcpy(h_out, hf, sizeof(float) * n);
        rc = oracle_layer_forward_rope(hf, codes_nonlocal, valid_nonlocal, codebook, D, G, K, wq, wk, wv, wo, bq, bk, bv, bo,
                                       n_q_heads, n_kv_heads, head_dim, n_cls, n_local, n_nonlocal, causal, n_before,
                                       scale, rope_base, y, codes_local, gap_local);
    }
    if (!rc) {
        for (int64_t i = 0; i < n; ++i) r[i] = x[i] + y[i];
        rc = oracle_norm(r, Tq, D, norm_kind, eps, g2, be2, h);
    }
    if (!rc) rc = oracle_mlp(h, Tq, D, d_ff, mlp_kind, w1, b1, w2, b2, m);
    if (!rc)
        for (int64_t i = 0; i < n; ++i) x_out[i] = r[i] + m[i];
    free(h); free(hf); free(y); free(r); free(m);
    return rc;
}

/* The block as the paper states it (no positional rotation inside the layer). */
int oracle_block_forward(const double* x, const int32_t* codes_nonlocal, const uint8_t* valid_nonlocal,
                         const float* codebook, int D, int G, int K,
                         int norm_kind, double eps, const float* g1, const float* be1, const float* g2, const float* be2,
                         const float* wq, const float* wk, const float* wv, const float* wo,
                         const float* bq, const float* bk, const float* bv, const float* bo,
                         int mlp_kind, int d_ff, const float* w1, const float* b1, const float* w2, const float* b2,
                         int n_q_heads, int n_kv_heads, int head_dim,
                         int n_cls, int n_local, int n_nonlocal, int causal, int n_before, double scale,
                         int h_is_bf16,
                         double* x_out, int32_t* codes_local, double* gap_local, float* h_out) {
    return oracle_block_forward_rope(x, codes_nonlocal, valid_nonlocal, codebook, D, G, K, norm_kind, eps, g1, be1, g2, be2,
                                     wq, wk, wv, wo, bq, bk, bv, bo, mlp_kind, d_ff, w1, b1, w2, b2, n_q_heads, n_kv_heads, head_dim,
                                     n_cls, n_local, n_nonlocal, causal, n_before, scale, h_is_bf16, 0.0,
                                     x_out, codes_local, gap_local, h_out);
}

/* ------------------------------------------------------------------------------------------------
 * The layer with keys and values quantised AFTER projection (App. "Memory Cost Analysis": Llama-3-8B uses
 * C = 2 codebooks per layer of hidden dimension d = 1024 = H_kv * dh, which is also what the 640 = 32 * 2 * 10
 * bits per token of the Llama results imply; the main text's Sec. 3.2 quantises the embeddings instead — the two
 * are different variants and both are kept).  On one device:
 *   Q, K, V        = x_local W_q, x_local W_k, x_local W_v          K, V stored in the element type
 *   codes_k_local  = encode(content rows of K; K codebook)  \   what this device transmits, and what a KV cache
 *   codes_v_local  = encode(content rows of V; V codebook)  /   keeps of it on the other devices
 *   K-hat, V-hat   = decode(codes_k_nonlocal), decode(codes_v_nonlocal)     no projection of rebuilt rows
 *   Y              = Attn(Q, K, K-hat, V, V-hat) W_o                        (Eq. 1 unchanged)
 * codebook_k, codebook_v [G, K, dkv / G].  kv_is_bf16: K and V are rounded to bf16 (nearest even) before they are
 * quantised and attended to, as the device stores them; else to fp32.  k_out, v_out (nullable, [T_q, dkv] fp32)
 * return those stored tensors.
 * ------------------------------------------------------------------------------------------------ */
static float round_elem(double v, int to_bf16) {
    float f = (float)v;
    if (to_bf16) {
        uint32_t u;
        memcpy(&u, &f, 4);
        if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);
        u &= 0xffff0000u;
        memcpy(&f, &u, 4);
    }
    return f;
}

int oracle_layer_forward_kv(const float* x_local, const int32_t* codes_k_nonlocal, const int32_t* codes_v_nonlocal,
                            const uint8_t* valid_nonlocal, const float* codebook_k, const float* codebook_v,
                            int D, int G, int K,
                            const float* wq, const float* wk, const float* wv, const float* wo,
                            const float* bq, const float* bk, const float* bv, const float* bo,
                            int n_q_heads, int n_kv_heads, int head_dim,
                            int n_cls, int n_local, int n_nonlocal, int causal, int n_before, double scale,
                            int kv_is_bf16,
                            double* y, int32_t* codes_k_local, int32_t* codes_v_local, double* gap_k, double* gap_v,
                            float* k_out, float* v_out) {
    const int Tq = n_cls + n_local, Tn = n_nonlocal;
    const int dq = n_q_heads * head_dim, dkv = n_kv_heads * head_dim;
    if (G <= 0 || dkv % G != 0) return -1;
    double* xl = (double*)malloc(sizeof(double) * ((int64_t)Tq * D + 1));
    for (int64_t i = 0; i < (int64_t)Tq * D; ++i) xl[i] = (double)x_local[i];
    double* Q = (double*)malloc(sizeof(double) * ((int64_t)Tq * dq + 1));
    double* Kl = (double*)malloc(sizeof(double) * ((int64_t)Tq * dkv + 1));
    double* Vl = (double*)malloc(sizeof(double) * ((int64_t)Tq * dkv + 1));
    float* Kf = (float*)malloc(sizeof(float) * ((int64_t)Tq * dkv + 1));
    float* Vf = (float*)malloc(sizeof(float) * ((int64_t)Tq * dkv + 1));
    float* Khf = (float*)calloc((int64_t)Tn * dkv + 1, sizeof(float));
    float* Vhf = (float*)calloc((int64_t)Tn * dkv + 1, sizeof(float));
    double* Kh = (double*)malloc(sizeof(double) * ((int64_t)Tn * dkv + 1));
    double* Vh = (double*)malloc(sizeof(double) * ((int64_t)Tn * dkv + 1));
    double* O = (double*)malloc(sizeof(double) * ((int64_t)Tq * dq + 1));
    oracle_linear(xl, Tq, D, dq, wq, bq, Q);
    oracle_linear(xl, Tq, D, dkv, wk, bk, Kl);
    oracle_linear(xl, Tq, D, dkv, wv, bv, Vl);
    /* K and V as the device stores them: that is what gets quantised and what the local attention uses */
    for (int64_t i = 0; i < (int64_t)Tq * dkv; ++i) {
        Kf[i] = round_elem(Kl[i], kv_is_bf16);
        Vf[i] = round_elem(Vl[i], kv_is_bf16);
        Kl[i] = (double)Kf[i];
        Vl[i] = (double)Vf[i];
    }
    if (k_out) memcpy(k_out, Kf, sizeof(float) * (int64_t)Tq * dkv);
    if (v_out) memcpy(v_out, Vf, sizeof(float) * (int64_t)Tq * dkv);
    int rc = oracle_vq_encode(Kf + (int64_t)n_cls * dkv, n_local, dkv, G, K, codebook_k, codes_k_local, gap_k);
    if (!rc) rc = oracle_vq_encode(Vf + (int64_t)n_cls * dkv, n_local, dkv, G, K, codebook_v, codes_v_local, gap_v);
    /* rows whose codes never arrived are not looked up; they stay zero and are excluded from the attention */
    for (int64_t t = 0; t < Tn && !rc; ++t) {
        if (valid_nonlocal && !valid_nonlocal[t]) continue;
        rc = oracle_vq_decode(codes_k_nonlocal + t * G, 1, dkv, G, K, codebook_k, Khf + t * (int64_t)dkv);
        if (!rc) rc = oracle_vq_decode(codes_v_nonlocal + t * G, 1, dkv, G, K, codebook_v, Vhf + t * (int64_t)dkv);
    }
    for (int64_t i = 0; i < (int64_t)Tn * dkv; ++i) {
        Kh[i] = (double)Khf[i];
        Vh[i] = (double)Vhf[i];
    }
    if (!rc)
        rc = oracle_mixed_attention_valid(Q, Kl, Vl, Kh, Vh, valid_nonlocal, n_q_heads, n_kv_heads, head_dim, n_cls, n_local,
                                          n_nonlocal, causal, n_before, scale, O, NULL, NULL);
    if (!rc) oracle_linear(O, Tq, dq, D, wo, bo, y);
    free(xl); free(Q); free(Kl); free(Vl); free(Kf); free(Vf); free(Khf); free(Vhf); free(Kh); free(Vh); free(O);
    return rc;
}

/* ------------------------------------------------------------------------------------------------
 * One decoding step over a KV cache whose non-local part is kept as VQ indices (App. "Memory Cost Analysis": each
 * device keeps its local tokens' keys and values at full precision and the non-local ones as one index per group per
 * token; Sec. 3.1: after the parallel encoding, autoregressive decoding proceeds on the single device that holds the
 * most recent token).  The new token's query attends to every cached token (all of them precede it):
 *   K-hat, V-hat = decode(codes_k), decode(codes_v)                      two codebooks, as in oracle_layer_forward_kv
 *   out[h]       = softmax_t( q[h] . [K_loc | K-hat][t, h / rep] * scale ) [V_loc | V-hat]
 * q [H_q, dh]; k_loc, v_loc [n_local, H_kv, dh] (the new token's own row included by the caller);
 * codes_k, codes_v [n_nonlocal, G]; valid (nullable) marks non-local tokens whose codes exist; out [H_q, dh];
 * lse (nullable) [H_q].  scale 0 means 1/sqrt(dh).
 * ------------------------------------------------------------------------------------------------ */
int oracle_decode_attention(const double* q, const double* k_loc, const double* v_loc,
                            const int32_t* codes_k, const int32_t* codes_v, const uint8_t* valid,
                            const float* codebook_k, const float* codebook_v, int G, int K,
                            int n_q_heads, int n_kv_heads, int head_dim, int n_local, int n_nonlocal, double scale,
                            double* out, double* lse) {
    const int dkv = n_kv_heads * head_dim;
    if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0 || G <= 0 || dkv % G != 0) return -1;
    const int rep = n_q_heads / n_kv_heads;
    const int T = n_local + n_nonlocal;
    if (scale == 0.0) scale = 1.0 / sqrt((double)head_dim);
    float* khf = (float*)calloc((int64_t)n_nonlocal * dkv + 1, sizeof(float));
    float* vhf = (float*)calloc((int64_t)n_nonlocal * dkv + 1, sizeof(float));
    int rc = 0;
    for (int64_t t = 0; t < n_nonlocal && !rc; ++t) {
        if (valid && !valid[t]) continue;
        rc = oracle_vq_decode(codes_k + t * G, 1, dkv, G, K, codebook_k, khf + t * (int64_t)dkv);
        if (!rc) rc = oracle_vq_decode(codes_v + t * G, 1, dkv, G, K, codebook_v, vhf + t * (int64_t)dkv);
    }
    double* s = (double*)malloc(sizeof(double) * (T + 1));
    for (int h = 0; h < n_q_heads && !rc; ++h) {
        const int j = h / rep;
        const double* qh = q + (int64_t)h * head_dim;
        double m = -INFINITY;
        for (int t = 0; t < T; ++t) {
            double acc = 0.0;
            if (t < n_local) {
                const double* kr = k_loc + ((int64_t)t * n_kv_heads + j) * head_dim;
                for (int c = 0; c < head_dim; ++c) acc += qh[c] * kr[c];
            } else if (!valid || valid[t - n_local]) {
                const float* kr = khf + ((int64_t)(t - n_local) * n_kv_heads + j) * head_dim;
                for (int c = 0; c < head_dim; ++c) acc += qh[c] * (double)kr[c];
            } else {
                s[t] = -INFINITY;
                continue;
            }
            s[t] = acc * scale;
            if (s[t] > m) m = s[t];
        }
        double l = 0.0;
        double* oh = out + (int64_t)h * head_dim;
        for (int c = 0; c < head_dim; ++c) oh[c] = 0.0;
        if (m == -INFINITY) {                    /* nothing to attend to */
            if (lse) lse[h] = -INFINITY;
            continue;
        }
        for (int t = 0; t < T; ++t) {
            if (s[t] == -INFINITY) continue;
            const double p = exp(s[t] - m);
            l += p;
            if (t < n_local) {
                const double* vr = v_loc + ((int64_t)t * n_kv_heads + j) * head_dim;
                for (int c = 0; c < head_dim; ++c) oh[c] += p * vr[c];
            } else {
                const float* vr = vhf + ((int64_t)(t - n_local) * n_kv_heads + j) * head_dim;
                for (int c = 0; c < head_dim; ++c) oh[c] += p * (double)vr[c];
            }
        }
        for (int c = 0; c < head_dim; ++c) oh[c] /= l;
        if (lse) lse[h] = m + log(l);
    }
    free(khf); free(vhf); free(s);
    return rc;
}

/* ------------------------------------------------------------------------------------------------
 * Training-side operations of the VQ module (Sec. 3.2 "The VQ module is jointly trained ...": K-means
 * initialisation over token embeddings, exponential-moving-average updates during fine-tuning, the commitment
 * term of Eq. 2; Sec. 3.3 NAVQ).  Forward arithmetic only; gradients are outside this build.
 * ------------------------------------------------------------------------------------------------ */

/* Per-codeword statistics of an assignment: counts[g,k] = number of tokens with codes[t,g] = k,
 * sums[g,k,:] = sum of their slices x[t, g*dg:(g+1)*dg], sqerr[g] = sum_t ||x[t, slice g] - codebook[g, codes[t,g], :]||^2
 * (the commitment term of Eq. 2 is beta times the sum of sqerr over the groups: ||X - sg(X-hat)||_2^2 written out;
 * the stop-gradient has no effect on the value).  K-means and the EMA update are built on counts and sums. */
int oracle_codebook_stats(const float* x, const int32_t* codes, const float* codebook, int64_t T, int D, int G, int K,
                          int64_t* counts, double* sums, double* sqerr) {
    if (T < 0 || D <= 0 || G <= 0 || K <= 0 || D % G != 0) return -1;
    const int dg = D / G;
    memset(counts, 0, sizeof(int64_t) * (size_t)G * K);
    for (int64_t i = 0; i < (int64_t)G * K * dg; ++i) sums[i] = 0.0;
    for (int g = 0; g < G; ++g) sqerr[g] = 0.0;
    for (int64_t t = 0; t < T; ++t)
        for (int g = 0; g < G; ++g) {
            const int32_t k = codes[t * G + g];
            if (k < 0 || k >= K) return -2;
            const float* xs = x + t * (int64_t)D + (int64_t)g * dg;
            const float* c = codebook + ((int64_t)g * K + k) * dg;
            double* s = sums + ((int64_t)g * K + k) * dg;
            counts[(int64_t)g * K + k] += 1;
            for (int j = 0; j < dg; ++j) {
                s[j] += (double)xs[j];
                const double d = (double)xs[j] - (double)c[j];
                sqerr[g] += d * d;
            }
        }
    return 0;
}

/* Codebook update from statistics.  EMA (gamma in [0, 1)):  N' = gamma N + (1 - gamma) counts,
 * M' = gamma M + (1 - gamma) sums, codeword = M' / N' where N' > 0, else the old codeword.  gamma = 0 is one
 * K-means (Lloyd) centroid step: codeword = sums / counts, an empty cluster keeps its codeword.
 * ema_n [G,K], ema_m [G,K,dg] are updated in place (both may be NULL when gamma == 0). */
int oracle_codebook_update(const int64_t* counts, const double* sums, double gamma, double* ema_n, double* ema_m,
                           const float* codebook_old, int G, int K, int dg, double* codebook_new) {
    if (G <= 0 || K <= 0 || dg <= 0 || !(gamma >= 0.0 && gamma < 1.0)) return -1;
    if (gamma > 0.0 && (!ema_n || !ema_m)) return -1;
    for (int64_t i = 0; i < (int64_t)G * K; ++i) {
        double n = (double)counts[i];
        if (ema_n) { n = gamma * ema_n[i] + (1.0 - gamma) * (double)counts[i]; ema_n[i] = n; }
        for (int j = 0; j < dg; ++j) {
            double m = sums[i * dg + j];
            if (ema_m) { m = gamma * ema_m[i * dg + j] + (1.0 - gamma) * sums[i * dg + j]; ema_m[i * dg + j] = m; }
            codebook_new[i * dg + j] = n > 0.0 ? m / n : (double)codebook_old[i * dg + j];
        }
    }
    return 0;
}

/* NAVQ (Sec. 3.3): X-tilde = X-hat + lambda * xi, xi ~ N(mu, Sigma) fitted to the quantisation residuals.  With
 * Sigma = L L^T and standard normal draws z [T, D] passed in (the method's random numbers are inputs):
 * xi[t] = mu + L z[t].  l_factor [D, D] row-major (any factor with L L^T = Sigma; the lower Cholesky factor in the
 * tests).  x_tilde [T, D]. */
int oracle_navq(const int32_t* codes, const float* codebook, int64_t T, int D, int G, int K,
                const float* mu, const float* l_factor, const float* z, double lambda, double* x_tilde) {
    float* xh = (float*)malloc(sizeof(float) * ((size_t)T * D + 1));
    int rc = oracle_vq_decode(codes, T, D, G, K, codebook, xh);
    for (int64_t t = 0; t < T && !rc; ++t)
        for (int i = 0; i < D; ++i) {
            double xi = (double)mu[i];
            for (int j = 0; j < D; ++j) xi += (double)l_factor[(int64_t)i * D + j] * (double)z[t * (int64_t)D + j];
            x_tilde[t * (int64_t)D + i] = (double)xh[t * (int64_t)D + i] + lambda * xi;
        }
    free(xh);
    return rc;
}
