// C ABI of the library: argument checking and the per-layer orchestration (paper Sec. 3.1).

#include "common.h"
#include "vq_encode_body.h"

namespace astra {

int check_vq_desc(const astra_vq_desc* d) {
    if (!d) return ASTRA_ERR_NULL;
    if (d->dtype != ASTRA_F32 && d->dtype != ASTRA_BF16) return ASTRA_ERR_DTYPE;
    if (d->code_type != ASTRA_CODE_U8 && d->code_type != ASTRA_CODE_U16) return ASTRA_ERR_DTYPE;
    if (d->d_model <= 0 || d->n_groups <= 0 || d->codebook_size <= 0) return ASTRA_ERR_SHAPE;
    if (d->d_model % d->n_groups != 0) return ASTRA_ERR_SHAPE;
    if (d->codebook_size > 65536) return ASTRA_ERR_SHAPE;
    if (d->code_type == ASTRA_CODE_U8 && d->codebook_size > 256) return ASTRA_ERR_DTYPE;
    return ASTRA_OK;
}

int check_attn_desc(const astra_attn_desc* d) {
    if (!d) return ASTRA_ERR_NULL;
    if (d->dtype != ASTRA_F32 && d->dtype != ASTRA_BF16) return ASTRA_ERR_DTYPE;
    if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0) return ASTRA_ERR_SHAPE;
    if (d->n_q_heads % d->n_kv_heads != 0 || d->n_q_heads > 65535) return ASTRA_ERR_SHAPE;
    if (d->n_cls < 0 || d->n_cls > 1 || d->n_local < 0 || d->n_nonlocal < 0) return ASTRA_ERR_SHAPE;
    if (d->causal != 0 && d->causal != 1) return ASTRA_ERR_SHAPE;
    if (d->causal && (d->n_cls != 0 || d->n_nonlocal_before < 0 || d->n_nonlocal_before > d->n_nonlocal)) return ASTRA_ERR_SHAPE;
    if (!(d->scale >= 0.f)) return ASTRA_ERR_SHAPE;
    if ((int64_t)d->n_cls + d->n_local > (1 << 30) || d->n_nonlocal > (1 << 30)) return ASTRA_ERR_SHAPE;
    if (d->dtype == ASTRA_BF16) {
        if (d->head_dim != 64 && d->head_dim != 128) return ASTRA_ERR_UNSUPPORTED;
    } else {
        if (d->head_dim > 256) return ASTRA_ERR_UNSUPPORTED;
    }
    return ASTRA_OK;
}

static AttnParams attn_params(const astra_attn_desc& d, const void* q, const void* k_local, const void* v_local,
                              const void* k_hat, const void* v_hat, void* out, float* lse) {
    AttnParams p{};
    p.q = q; p.k_loc = k_local; p.v_loc = v_local; p.k_hat = k_hat; p.v_hat = v_hat;
    p.out = out; p.lse = lse;
    p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.Tq = d.n_cls + d.n_local;
    p.Tn_vis = d.causal ? d.n_nonlocal_before : d.n_nonlocal;
    p.causal = d.causal;
    p.scale = d.scale != 0.f ? d.scale : 1.f / sqrtf((float)d.head_dim);
    return p;
}

struct LayerPlan {
    int Tq, Tn, Tn_vis, D, dq, dkv;
    bool need_xhat;
    bool wide_enc;           // wide groups: the encode runs as score products + an argmin pass over scores kept in the workspace
    bool vt;                 // V, V-hat kept transposed for the attention kernel (bf16)
    int ldv_loc, ldv_hat;    // padded token counts of the transposed V buffers
    size_t off_q, off_k, off_v, off_kh, off_vh, off_o, off_xhat, off_scores, total;
};

static int make_plan(const astra_layer_desc* desc, LayerPlan* pl) {
    if (!desc) return ASTRA_ERR_NULL;
    int rc = check_vq_desc(&desc->vq);
    if (rc) return rc;
    rc = check_attn_desc(&desc->attn);
    if (rc) return rc;
    if (desc->vq.dtype != desc->attn.dtype) return ASTRA_ERR_DTYPE;
    const astra_attn_desc& a = desc->attn;
    const int eb = elem_bytes(desc->vq.dtype);
    pl->Tq = a.n_cls + a.n_local;
    pl->Tn = a.n_nonlocal;
    pl->Tn_vis = a.causal ? a.n_nonlocal_before : a.n_nonlocal;
    pl->D = desc->vq.d_model;
    pl->dq = a.n_q_heads * a.head_dim;
    pl->dkv = a.n_kv_heads * a.head_dim;
    const int dg = pl->D / desc->vq.n_groups;
    if (desc->vq.dtype == ASTRA_BF16 && (pl->D % 8 != 0)) return ASTRA_ERR_UNSUPPORTED;
    pl->need_xhat = desc->vq.dtype == ASTRA_BF16 && (dg % 8 != 0);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    pl->off_q = take((size_t)pl->Tq * pl->dq * eb);
    pl->off_k = take((size_t)pl->Tq * pl->dkv * eb);
    pl->vt = desc->vq.dtype == ASTRA_BF16;
    pl->ldv_loc = (int)align_up((size_t)pl->Tq, 64);
    pl->ldv_hat = (int)align_up((size_t)pl->Tn_vis, 64);
    pl->off_v = take((size_t)(pl->vt ? pl->ldv_loc : pl->Tq) * pl->dkv * eb);
    pl->off_kh = take((size_t)pl->Tn_vis * pl->dkv * eb);
    pl->off_vh = take((size_t)(pl->vt ? pl->ldv_hat : pl->Tn_vis) * pl->dkv * eb);
    pl->off_o = take((size_t)pl->Tq * pl->dq * eb);
    pl->off_xhat = take(pl->need_xhat ? (size_t)pl->Tn_vis * pl->D * eb : 0);
    // scores [T_l, G, K] fp32 of the wide-group encode (few groups: the buffer is T_l * G * K * 4 bytes, capped at 256 MiB)
    // (with one group the product rides in the projection launch for free; with more it is launches of its own, which pay once
    // a group's codebook has 2^17 elements or more: below that the kernel that streams the codebook per 32 tokens is faster)
    pl->wide_enc = desc->vq.dtype == ASTRA_BF16 && vq_encode_wide_ok(desc->vq.codebook_size, dg, pl->D) && a.n_local > 0 &&
                   desc->vq.codebook_size % 8 == 0 &&
                   (desc->vq.n_groups == 1 || (int64_t)desc->vq.codebook_size * dg >= (1 << 17)) &&
                   (size_t)a.n_local * desc->vq.n_groups * desc->vq.codebook_size * 4 <= ((size_t)256 << 20);
    pl->off_scores = take(pl->wide_enc ? (size_t)a.n_local * desc->vq.n_groups * desc->vq.codebook_size * 4 : 0);
    pl->total = off > 0 ? off : 256;
    return ASTRA_OK;
}

struct KvPlan {
    int Tq, Tn, Tn_vis, D, dq, dkv;
    bool vt;
    int ldv_loc, ldv_hat;
    size_t off_q, off_k, off_v, off_vt, off_kh, off_vh, off_o, total;
};

static int make_kv_plan(const astra_layer_kv_desc* desc, KvPlan* pl) {
    if (!desc) return ASTRA_ERR_NULL;
    int rc = check_vq_desc(&desc->vq);
    if (rc) return rc;
    rc = check_attn_desc(&desc->attn);
    if (rc) return rc;
    if (desc->vq.dtype != desc->attn.dtype) return ASTRA_ERR_DTYPE;
    const astra_attn_desc& a = desc->attn;
    if (desc->d_model <= 0 || desc->vq.d_model != a.n_kv_heads * a.head_dim) return ASTRA_ERR_SHAPE;
    const int dtype = desc->vq.dtype, eb = elem_bytes(dtype);
    pl->Tq = a.n_cls + a.n_local;
    pl->Tn = a.n_nonlocal;
    pl->Tn_vis = a.causal ? a.n_nonlocal_before : a.n_nonlocal;
    pl->D = desc->d_model;
    pl->dq = a.n_q_heads * a.head_dim;
    pl->dkv = a.n_kv_heads * a.head_dim;
    pl->vt = dtype == ASTRA_BF16;
    if (pl->vt && ((pl->dkv / desc->vq.n_groups) % 8 != 0 || pl->D % 64 != 0)) return ASTRA_ERR_UNSUPPORTED;
    pl->ldv_loc = (int)align_up((size_t)pl->Tq, 64);
    pl->ldv_hat = (int)align_up((size_t)pl->Tn_vis, 64);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    pl->off_q = take((size_t)pl->Tq * pl->dq * eb);
    pl->off_k = take((size_t)pl->Tq * pl->dkv * eb);
    pl->off_v = take((size_t)pl->Tq * pl->dkv * eb);
    pl->off_vt = take(pl->vt ? (size_t)pl->ldv_loc * pl->dkv * eb : 0);
    pl->off_kh = take((size_t)pl->Tn_vis * pl->dkv * eb);
    pl->off_vh = take((size_t)(pl->vt ? pl->ldv_hat : pl->Tn_vis) * pl->dkv * eb);
    pl->off_o = take((size_t)pl->Tq * pl->dq * eb);
    pl->total = off > 0 ? off : 256;
    return ASTRA_OK;
}

struct BlockPlan {
    LayerPlan layer;
    int d_ff;
    size_t off_h, off_a, off_a2, off_split, split_bytes, total;     // after the layer's own workspace: normalised rows, MLP hidden
                                                                    // rows, partial sums of the second MLP product
};

static int make_block_plan(const astra_block_desc* desc, BlockPlan* bp) {
    if (!desc) return ASTRA_ERR_NULL;
    int rc = make_plan(&desc->layer, &bp->layer);
    if (rc) return rc;
    if (desc->norm_kind != ASTRA_NORM_LAYER && desc->norm_kind != ASTRA_NORM_RMS) return ASTRA_ERR_SHAPE;
    if (desc->mlp_kind != ASTRA_MLP_GELU_TANH && desc->mlp_kind != ASTRA_MLP_GELU_ERF && desc->mlp_kind != ASTRA_MLP_SWIGLU)
        return ASTRA_ERR_SHAPE;
    if (desc->d_ff <= 0 || desc->d_ff > (1 << 24) || !(desc->eps >= 0.f)) return ASTRA_ERR_SHAPE;
    if (!(desc->rope_base >= 0.f) || desc->rope_base > 1e30f) return ASTRA_ERR_SHAPE;
    // rotary positions need every row's place in the sequence: given for causal layers (contiguous chunks, n_before)
    if (desc->rope_base > 0.f && (!desc->layer.attn.causal || desc->layer.attn.head_dim % 2 != 0)) return ASTRA_ERR_UNSUPPORTED;
    const int dtype = desc->layer.vq.dtype;
    if (dtype == ASTRA_BF16 && desc->d_ff % 64 != 0) return ASTRA_ERR_UNSUPPORTED;     // d_ff is a contraction length
    const int eb = elem_bytes(dtype);
    const LayerPlan& pl = bp->layer;
    bp->d_ff = desc->d_ff;
    size_t off = pl.total;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    bp->off_h = take((size_t)pl.Tq * pl.D * eb);
    bp->off_a = take((size_t)pl.Tq * desc->d_ff * eb);
    // fp32 has no fused gate: the first GEMM leaves [T_q, 2 d_ff], a second kernel forms the product
    bp->off_a2 = take(dtype != ASTRA_BF16 && desc->mlp_kind == ASTRA_MLP_SWIGLU ? (size_t)pl.Tq * 2 * desc->d_ff * eb : 0);
    bp->split_bytes = gemm_split_workspace_bytes(dtype, pl.Tq, pl.D, desc->d_ff);
    bp->off_split = take(bp->split_bytes);
    bp->total = off;
    return ASTRA_OK;
}

}  // namespace astra

using namespace astra;

extern "C" {

int astra_version(void) { return 100; }

const char* astra_status_string(int status) {
    switch (status) {
        case ASTRA_OK: return "ok";
        case ASTRA_ERR_NULL: return "required pointer is NULL";
        case ASTRA_ERR_SHAPE: return "inconsistent or out-of-range sizes";
        case ASTRA_ERR_DTYPE: return "bad element or code type";
        case ASTRA_ERR_WORKSPACE: return "workspace missing or too small";
        case ASTRA_ERR_UNSUPPORTED: return "no kernel for this configuration";
        case ASTRA_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int astra_vq_prepare(const astra_vq_desc* desc, const void* codebook, float* cnorm_out, void* stream) {
    int rc = check_vq_desc(desc);
    if (rc) return rc;
    if (!codebook || !cnorm_out) return ASTRA_ERR_NULL;
    return launch_vq_prepare(*desc, codebook, cnorm_out, (hipStream_t)stream);
}

int astra_vq_encode(const astra_vq_desc* desc, const void* x, int64_t n_tokens, const void* codebook,
                    const float* cnorm, void* codes_out, void* stream) {
    int rc = check_vq_desc(desc);
    if (rc) return rc;
    if (n_tokens < 0) return ASTRA_ERR_SHAPE;
    if (n_tokens == 0) return ASTRA_OK;
    if (!x || !codebook || !cnorm || !codes_out) return ASTRA_ERR_NULL;
    return launch_vq_encode(*desc, x, desc->d_model, n_tokens, codebook, cnorm, codes_out, (hipStream_t)stream);
}

// wide groups with a workspace: score products (up to six groups per launch) + one argmin pass
static bool encode_ws_applies(const astra_vq_desc& d, int64_t n_tokens) {
    const int dg = d.d_model / d.n_groups;
    // the products pay once a group's codebook has 2^17 elements or more; below that the kernel that streams it per 32 tokens wins
    return d.dtype == ASTRA_BF16 && vq_encode_wide_ok(d.codebook_size, dg, d.d_model) && d.codebook_size % 8 == 0 && n_tokens > 0 &&
           n_tokens <= 0x7fffffff && (int64_t)d.codebook_size * dg >= (1 << 17);
}

size_t astra_vq_encode_workspace_bytes(const astra_vq_desc* desc, int64_t n_tokens) {
    if (check_vq_desc(desc) != ASTRA_OK || n_tokens < 0) return 0;
    if (!encode_ws_applies(*desc, n_tokens)) return 256;
    return align_up((size_t)n_tokens * desc->n_groups * desc->codebook_size * sizeof(float), 256);
}

int astra_vq_encode_ws(const astra_vq_desc* desc, const void* x, int64_t n_tokens, const void* codebook, const float* cnorm,
                       void* codes_out, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_vq_desc(desc);
    if (rc) return rc;
    if (n_tokens < 0) return ASTRA_ERR_SHAPE;
    if (n_tokens == 0) return ASTRA_OK;
    if (!x || !codebook || !cnorm || !codes_out) return ASTRA_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (!encode_ws_applies(*desc, n_tokens)) return launch_vq_encode(*desc, x, desc->d_model, n_tokens, codebook, cnorm, codes_out, s);
    if (!workspace || workspace_bytes < astra_vq_encode_workspace_bytes(desc, n_tokens)) return ASTRA_ERR_WORKSPACE;
    const int G = desc->n_groups, K = desc->codebook_size, D = desc->d_model, dg = D / G;
    float* scores = (float*)workspace;
    for (int pass = 0; pass < 2; ++pass) {           // every launch is validated before the first one runs
        for (int g0 = 0; g0 < G; g0 += kMaxGemmProblems) {
            GemmProblem sp[kMaxGemmProblems] = {};
            const int n = G - g0 < kMaxGemmProblems ? G - g0 : kMaxGemmProblems;
            for (int i = 0; i < n; ++i) {
                const int g = g0 + i;
                sp[i].a = (const char*)x + (size_t)g * dg * 2; sp[i].lda = D;
                sp[i].b = (const char*)codebook + (size_t)g * K * dg * 2; sp[i].ldb = dg;
                sp[i].c = scores + (size_t)g * K; sp[i].ldc = G * K;
                sp[i].M = (int)n_tokens; sp[i].N = K; sp[i].K = dg; sp[i].c_mode = kCF32;
            }
            rc = launch_gemm_batch(desc->dtype, sp, n, s, nullptr, nullptr, pass == 0, nullptr, 0, false);
            if (rc) return rc;
        }
    }
    return launch_vq_argmin_scores(*desc, scores, cnorm, n_tokens, codes_out, s);
}

int astra_vq_decode(const astra_vq_desc* desc, const void* codes, int64_t n_tokens, const void* codebook,
                    void* x_hat_out, void* stream) {
    int rc = check_vq_desc(desc);
    if (rc) return rc;
    if (n_tokens < 0) return ASTRA_ERR_SHAPE;
    if (n_tokens == 0) return ASTRA_OK;
    if (!codes || !codebook || !x_hat_out) return ASTRA_ERR_NULL;
    return launch_vq_decode(*desc, codes, n_tokens, codebook, x_hat_out, (hipStream_t)stream);
}

int astra_mixed_attention(const astra_attn_desc* desc, const void* q, const void* k_local, const void* v_local,
                          const void* k_hat, const void* v_hat, void* out, float* lse_out, void* stream) {
    return astra_mixed_attention_valid(desc, q, k_local, v_local, k_hat, v_hat, nullptr, out, lse_out, stream);
}

int astra_mixed_attention_valid(const astra_attn_desc* desc, const void* q, const void* k_local, const void* v_local,
                                const void* k_hat, const void* v_hat, const uint64_t* valid_bits, void* out, float* lse_out,
                                void* stream) {
    int rc = check_attn_desc(desc);
    if (rc) return rc;
    if (desc->n_cls + desc->n_local == 0) return ASTRA_OK;
    if (!q || !k_local || !v_local || !out) return ASTRA_ERR_NULL;
    const int vis = desc->causal ? desc->n_nonlocal_before : desc->n_nonlocal;
    if (vis > 0 && (!k_hat || !v_hat)) return ASTRA_ERR_NULL;
    AttnParams ap = attn_params(*desc, q, k_local, v_local, k_hat, v_hat, out, lse_out);
    ap.valid_bits = (const unsigned long long*)valid_bits;
    return launch_attention(desc->dtype, ap, desc->head_dim, (hipStream_t)stream);
}

size_t astra_layer_workspace_bytes(const astra_layer_desc* desc) {
    LayerPlan pl;
    if (make_plan(desc, &pl) != ASTRA_OK) return 0;
    return pl.total;
}

static int layer_forward_impl(const astra_layer_desc* desc, const void* x_local, const void* codes_nonlocal,
                              const void* codebook, const float* cnorm,
                              const void* wq, const void* wk, const void* wv, const void* wo,
                              const void* bq, const void* bk, const void* bv, const void* bo,
                              void* y_out, void* codes_local_out, void* workspace, size_t workspace_bytes, void* stream,
                              void* const* ev, int* plan_encode_fused = nullptr, const uint64_t* valid_bits = nullptr,
                              const float* residual = nullptr, const float* pre_k = nullptr, const float* pre_v = nullptr,
                              float rope_base = 0.f) {
    // plan_encode_fused: validate the shapes and report whether the projection launch would carry the encode;
    // nothing is launched and no pointer is dereferenced
    const bool plan_only = plan_encode_fused != nullptr;
    LayerPlan pl;
    int rc = make_plan(desc, &pl);
    if (rc) return rc;
    const astra_vq_desc& vq = desc->vq;
    const astra_attn_desc& at = desc->attn;
    if (plan_only) *plan_encode_fused = 0;
    if (pl.Tq == 0) return ASTRA_OK;
    if (!plan_only) {
        if (!x_local || !codebook || !cnorm || !wq || !wk || !wv || !wo || !y_out) return ASTRA_ERR_NULL;
        if (at.n_local > 0 && !codes_local_out) return ASTRA_ERR_NULL;
        if (pl.Tn_vis > 0 && !codes_nonlocal) return ASTRA_ERR_NULL;
        if (!workspace || workspace_bytes < pl.total) return ASTRA_ERR_WORKSPACE;
    } else {
        // shapes only: any non-null address marks the gathered operand
        x_local = &pl;
        codes_nonlocal = &pl;
        workspace = &pl;
    }
    hipStream_t s = (hipStream_t)stream;
    auto mark = [&](int i, hipStream_t on) { if (ev && ev[i]) (void)hipEventRecord((hipEvent_t)ev[i], on); };
    mark(0, s);
    const int eb = elem_bytes(vq.dtype);
    char* ws = (char*)workspace;
    void *Q = ws + pl.off_q, *K = ws + pl.off_k, *V = ws + pl.off_v, *Kh = ws + pl.off_kh, *Vh = ws + pl.off_vh,
         *O = ws + pl.off_o, *Xh = ws + pl.off_xhat;

    // 1. indices this device transmits: the encode of the content rows (the class row is not encoded) depends on
    //    nothing else in the layer and nothing in the layer depends on it.  It is offered to the projection launch,
    //    which runs it as extra workgroups on compute units its tiles leave idle; if that launch does not take it
    //    (other element type, tile count, group size), it runs as a kernel of its own on the same stream.
    EncodeJob ej{};
    ej.x = (const char*)x_local + (size_t)at.n_cls * pl.D * eb;
    ej.codebook = codebook; ej.cnorm = cnorm; ej.codes = codes_local_out; ej.ldx = pl.D;
    ej.n_tokens = at.n_local; ej.G = vq.n_groups; ej.K = vq.codebook_size; ej.dg = pl.D / vq.n_groups;
    ej.code_bytes = code_bytes(vq.code_type);
    const bool offer = vq.dtype == ASTRA_BF16 && at.n_local > 0 && pl.D % 8 == 0;
    bool enc_fused = false;

    // 2. projections: Q, K, V of local rows; K-hat, V-hat of the rows rebuilt from the peers' codes
    GemmProblem pr[kMaxGemmProblems] = {};
    int n_pr = 5;
    auto local = [&](GemmProblem& g, const void* w, const void* b, void* c, int n) {
        g.a = x_local; g.b = w; g.bias = b; g.c = c; g.M = pl.Tq; g.N = n; g.K = pl.D; g.lda = pl.D; g.ldc = n;
        g.c_mode = vq.dtype == ASTRA_BF16 ? kCBf16 : kCF32;
    };
    auto nonlocal_ = [&](GemmProblem& g, const void* w, const void* b, void* c, int n) {
        g.b = w; g.bias = b; g.c = c; g.M = pl.Tn_vis; g.N = n; g.K = pl.D; g.lda = pl.D; g.ldc = n;
        g.c_mode = vq.dtype == ASTRA_BF16 ? kCBf16 : kCF32;
        if (pl.need_xhat) { g.a = Xh; }
        else {
            g.codes = codes_nonlocal; g.codebook = codebook; g.G = vq.n_groups; g.Kc = vq.codebook_size;
            g.dg = pl.D / vq.n_groups; g.code_bytes = code_bytes(vq.code_type);
        }
    };
    local(pr[0], wq, bq, Q, pl.dq);
    local(pr[1], wk, bk, K, pl.dkv);
    local(pr[2], wv, bv, V, pl.dkv);
    if (pl.vt) { pr[2].c_mode = kCTransposedV; pr[2].ldc = pl.ldv_loc; }
    const bool preprojected = pre_k != nullptr;       // K-hat, V-hat come from pre-projected codebooks: no product of rebuilt rows
    nonlocal_(pr[3], wk, bk, Kh, pl.dkv);
    nonlocal_(pr[4], wv, bv, Vh, pl.dkv);
    if (pl.vt) { pr[4].c_mode = kCTransposedV; pr[4].ldc = pl.ldv_hat; }
    if (preprojected) {
        if (pl.dkv % 8 != 0 || (pl.vt && pl.dkv % 64 != 0)) return ASTRA_ERR_UNSUPPORTED;
        pr[3].M = pr[4].M = 0;
    }
    // Wide groups (few groups of 128 values or more, down to the paper's G = 1): the distance matrix of a group is a product of
    // its own, scores[t, g, k] = x[t, slice g] . codebook[g, k, :] (fp32, workspace), followed by one argmin pass over
    // ||c||^2 - 2 score.  With one group the product rides in the projection launch as a sixth problem (its tiles land on compute
    // units the projections leave idle); with more it is launched on its own, up to six groups at a time.
    float* scores = (float*)(ws + pl.off_scores);
    const int Kc = vq.codebook_size, dg_ = pl.D / vq.n_groups;
    auto score_problem = [&](GemmProblem& g, int grp) {
        g = GemmProblem{};
        g.a = (const char*)ej.x + (size_t)grp * dg_ * eb; g.lda = pl.D;
        g.b = (const char*)codebook + (size_t)grp * Kc * dg_ * eb; g.ldb = dg_;
        g.c = scores + (size_t)grp * Kc; g.ldc = vq.n_groups * Kc;
        g.M = at.n_local; g.N = Kc; g.K = dg_; g.c_mode = kCF32;
    };
    const bool scores_in_projection_launch = pl.wide_enc && vq.n_groups == 1;
    if (scores_in_projection_launch) score_problem(pr[n_pr++], 0);
    const bool offer_fused = offer && !pl.wide_enc;

    AttnParams ap = attn_params(at, Q, K, V, Kh, Vh, O, nullptr);
    ap.v_transposed = pl.vt ? 1 : 0;
    ap.valid_bits = (const unsigned long long*)valid_bits;
    ap.ldv_loc = pl.ldv_loc;
    ap.ldv_hat = pl.ldv_hat;
    GemmProblem po = {};
    po.a = O; po.b = wo; po.bias = bo; po.c = y_out; po.M = pl.Tq; po.N = pl.D; po.K = pl.dq; po.lda = pl.dq; po.ldc = pl.D;
    po.c_mode = kCF32;      // y leaves the layer as the fp32 accumulator, for both element types
    po.residual = residual; // inside a block: y_out = residual + layer output

    // every launch of the layer is validated before the first one runs: an error leaves all outputs untouched
    rc = launch_gemm_batch(vq.dtype, pr, n_pr, s, offer_fused ? &ej : nullptr, offer_fused ? &enc_fused : nullptr, true);
    if (rc == ASTRA_OK && pl.wide_enc && !scores_in_projection_launch) {
        for (int g0 = 0; g0 < vq.n_groups && rc == ASTRA_OK; g0 += kMaxGemmProblems) {
            GemmProblem sp[kMaxGemmProblems];
            const int n = vq.n_groups - g0 < kMaxGemmProblems ? vq.n_groups - g0 : kMaxGemmProblems;
            for (int i = 0; i < n; ++i) score_problem(sp[i], g0 + i);
            rc = launch_gemm_batch(vq.dtype, sp, n, s, nullptr, nullptr, true, nullptr, 0, false);
        }
    }
    if (rc == ASTRA_OK) rc = launch_attention(vq.dtype, ap, at.head_dim, s, true);
    if (rc == ASTRA_OK) rc = launch_gemm_batch(vq.dtype, &po, 1, s, nullptr, nullptr, true);
    if (plan_only) {
        *plan_encode_fused = enc_fused ? 1 : 0;
        return rc;
    }
    if (rc) return rc;

    if (pl.need_xhat && pl.Tn_vis > 0 && !preprojected) {
        rc = launch_vq_decode(vq, codes_nonlocal, pl.Tn_vis, codebook, Xh, s);
        if (rc) return rc;
    }
    rc = launch_gemm_batch(vq.dtype, pr, n_pr, s, offer_fused ? &ej : nullptr, offer_fused ? &enc_fused : nullptr, false);
    if (rc) return rc;
    if (preprojected && pl.Tn_vis > 0) {
        rc = launch_preproj_gather(vq.dtype, vq.code_type, codes_nonlocal, pre_k, bk, pl.Tn_vis, vq.n_groups, vq.codebook_size, pl.dkv,
                                   Kh, pl.dkv, false, s);
        if (rc) return rc;
        rc = launch_preproj_gather(vq.dtype, vq.code_type, codes_nonlocal, pre_v, bv, pl.Tn_vis, vq.n_groups, vq.codebook_size, pl.dkv,
                                   Vh, pl.vt ? pl.ldv_hat : pl.dkv, pl.vt, s);
        if (rc) return rc;
    }
    mark(1, s);
    mark(5, s);
    if (pl.wide_enc) {
        if (!scores_in_projection_launch) {
            for (int g0 = 0; g0 < vq.n_groups; g0 += kMaxGemmProblems) {
                GemmProblem sp[kMaxGemmProblems];
                const int n = vq.n_groups - g0 < kMaxGemmProblems ? vq.n_groups - g0 : kMaxGemmProblems;
                for (int i = 0; i < n; ++i) score_problem(sp[i], g0 + i);
                rc = launch_gemm_batch(vq.dtype, sp, n, s, nullptr, nullptr, false, nullptr, 0, false);
                if (rc) return rc;
            }
        }
        rc = launch_vq_argmin_scores(vq, scores, cnorm, at.n_local, codes_local_out, s);
        if (rc) return rc;
    }
    // an encode the projection launch did not take is offered to the attention launch (extra workgroups in its tail); if
    // that does not take it either, it runs as a kernel of its own
    const bool enc_pending = !pl.wide_enc && !enc_fused && at.n_local > 0;
    bool enc_in_attention = false;
    mark(6, s);

    // optional rotary positions (a block's choice, outside the paper): Q and K of the local rows (content row i at n_before + i,
    // class rows untouched) and K-hat of the visible non-local rows (row j at j; the layer is causal, so they all precede the chunk)
    if (rope_base > 0.f) {
        rc = launch_rope(vq.dtype, Q, pl.dq, pl.Tq, at.n_q_heads, at.head_dim, at.n_cls, 0, 0, at.n_nonlocal_before - at.n_cls, rope_base, s);
        if (rc == ASTRA_OK) rc = launch_rope(vq.dtype, K, pl.dkv, pl.Tq, at.n_kv_heads, at.head_dim, at.n_cls, 0, 0, at.n_nonlocal_before - at.n_cls, rope_base, s);
        if (rc == ASTRA_OK) rc = launch_rope(vq.dtype, Kh, pl.dkv, pl.Tn_vis, at.n_kv_heads, at.head_dim, 0, at.n_nonlocal_before, 0, at.n_local, rope_base, s);
        if (rc) return rc;
    }

    // 3. mixed-precision attention (Eq. 1)
    rc = launch_attention(vq.dtype, ap, at.head_dim, s, false, enc_pending && offer ? &ej : nullptr, enc_pending && offer ? 1 : 0,
                          enc_pending && offer ? &enc_in_attention : nullptr);
    if (rc) return rc;
    if (enc_pending && !enc_in_attention) {
        rc = launch_vq_encode(vq, ej.x, pl.D, at.n_local, codebook, cnorm, codes_local_out, s);
        if (rc) return rc;
    }
    mark(2, s);

    // 4. output projection
    rc = launch_gemm_batch(vq.dtype, &po, 1, s);
    mark(3, s);
    mark(4, s);
    return rc;
}

int astra_vq_project_codebook(const astra_vq_desc* desc, const void* codebook, const void* w, int32_t n_out, float* p_out,
                              void* stream) {
    int rc = check_vq_desc(desc);
    if (rc) return rc;
    if (n_out <= 0 || n_out % 8 != 0) return ASTRA_ERR_SHAPE;
    if (!codebook || !w || !p_out) return ASTRA_ERR_NULL;
    const int G = desc->n_groups, K = desc->codebook_size, D = desc->d_model, dg = D / G;
    const int eb = elem_bytes(desc->dtype);
    // one product per group: P_g [K, n_out] = C_g [K, dg] . (w[:, g*dg:(g+1)*dg])^T, the weight slice read in place through
    // its row stride D; fp32 out.  All launches are validated before the first.
    for (int pass = 0; pass < 2; ++pass) {
        for (int g0 = 0; g0 < G; g0 += kMaxGemmProblems) {
            GemmProblem pr[kMaxGemmProblems] = {};
            const int n = G - g0 < kMaxGemmProblems ? G - g0 : kMaxGemmProblems;
            for (int i = 0; i < n; ++i) {
                const int g = g0 + i;
                pr[i].a = (const char*)codebook + (size_t)g * K * dg * eb;
                pr[i].b = (const char*)w + (size_t)g * dg * eb;
                pr[i].c = p_out + (size_t)g * K * n_out;
                pr[i].M = K; pr[i].N = n_out; pr[i].K = dg; pr[i].lda = dg; pr[i].ldb = D; pr[i].ldc = n_out;
                pr[i].c_mode = kCF32;
            }
            rc = launch_gemm_batch(desc->dtype, pr, n, (hipStream_t)stream, nullptr, nullptr, pass == 0, nullptr, 0, false);
            if (rc) return rc;
        }
    }
    return ASTRA_OK;
}

int astra_layer_forward_preprojected(const astra_layer_desc* desc, const void* x_local, const void* codes_nonlocal,
                                     const uint64_t* valid_nonlocal_bits, const void* codebook, const float* cnorm,
                                     const float* p_k, const float* p_v,
                                     const void* wq, const void* wk, const void* wv, const void* wo,
                                     const void* bq, const void* bk, const void* bv, const void* bo,
                                     void* y_out, void* codes_local_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (!p_k || !p_v) return ASTRA_ERR_NULL;
    return layer_forward_impl(desc, x_local, codes_nonlocal, codebook, cnorm, wq, wk, wv, wo, bq, bk, bv, bo, y_out, codes_local_out,
                              workspace, workspace_bytes, stream, nullptr, nullptr, valid_nonlocal_bits, nullptr, p_k, p_v);
}

int astra_probe_mfma_bf16(float* out, int n_blocks, int iters, void* stream) {
    if (!out) return ASTRA_ERR_NULL;
    return launch_mfma_probe(out, n_blocks, iters, (hipStream_t)stream);
}

int astra_layer_encode_fused(const astra_layer_desc* desc) {
    int fused = 0;
    const int rc = layer_forward_impl(desc, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                      nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr, &fused);
    return rc ? rc : fused;
}

int astra_layer_forward(const astra_layer_desc* desc, const void* x_local, const void* codes_nonlocal,
                        const void* codebook, const float* cnorm,
                        const void* wq, const void* wk, const void* wv, const void* wo,
                        const void* bq, const void* bk, const void* bv, const void* bo,
                        void* y_out, void* codes_local_out, void* workspace, size_t workspace_bytes, void* stream) {
    return layer_forward_impl(desc, x_local, codes_nonlocal, codebook, cnorm, wq, wk, wv, wo, bq, bk, bv, bo, y_out,
                              codes_local_out, workspace, workspace_bytes, stream, nullptr);
}

int astra_layer_forward_valid(const astra_layer_desc* desc, const void* x_local, const void* codes_nonlocal,
                              const uint64_t* valid_nonlocal_bits, const void* codebook, const float* cnorm,
                              const void* wq, const void* wk, const void* wv, const void* wo,
                              const void* bq, const void* bk, const void* bv, const void* bo,
                              void* y_out, void* codes_local_out, void* workspace, size_t workspace_bytes, void* stream) {
    return layer_forward_impl(desc, x_local, codes_nonlocal, codebook, cnorm, wq, wk, wv, wo, bq, bk, bv, bo, y_out,
                              codes_local_out, workspace, workspace_bytes, stream, nullptr, nullptr, valid_nonlocal_bits);
}

size_t astra_layer_kv_workspace_bytes(const astra_layer_kv_desc* desc) {
    KvPlan pl;
    if (make_kv_plan(desc, &pl) != ASTRA_OK) return 0;
    return pl.total;
}

int astra_layer_forward_kv(const astra_layer_kv_desc* desc, const void* x_local, const void* codes_k_nonlocal,
                           const void* codes_v_nonlocal, const uint64_t* valid_nonlocal_bits, const void* codebook_k,
                           const float* cnorm_k, const void* codebook_v, const float* cnorm_v, const void* wq, const void* wk,
                           const void* wv, const void* wo, const void* bq, const void* bk, const void* bv, const void* bo,
                           void* y_out, void* codes_k_local_out, void* codes_v_local_out, void* k_out, void* v_out,
                           void* workspace, size_t workspace_bytes, void* stream) {
    KvPlan pl;
    int rc = make_kv_plan(desc, &pl);
    if (rc) return rc;
    if (pl.Tq == 0) return ASTRA_OK;
    const astra_vq_desc& vq = desc->vq;
    const astra_attn_desc& at = desc->attn;
    if (!x_local || !codebook_k || !cnorm_k || !codebook_v || !cnorm_v || !wq || !wk || !wv || !wo || !y_out) return ASTRA_ERR_NULL;
    if (at.n_local > 0 && (!codes_k_local_out || !codes_v_local_out)) return ASTRA_ERR_NULL;
    if (pl.Tn_vis > 0 && (!codes_k_nonlocal || !codes_v_nonlocal)) return ASTRA_ERR_NULL;
    if (!workspace || workspace_bytes < pl.total) return ASTRA_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int dtype = vq.dtype, eb = elem_bytes(dtype);
    char* ws = (char*)workspace;
    void *Q = ws + pl.off_q, *K = k_out ? k_out : ws + pl.off_k, *V = v_out ? v_out : ws + pl.off_v, *Vt = ws + pl.off_vt,
         *Kh = ws + pl.off_kh, *Vh = ws + pl.off_vh, *O = ws + pl.off_o;

    // 1. projections of the local rows only; K and V row-major, as they are quantised and cached
    GemmProblem pr[3] = {};
    auto local = [&](GemmProblem& g, const void* w, const void* b, void* c, int n) {
        g.a = x_local; g.b = w; g.bias = b; g.c = c; g.M = pl.Tq; g.N = n; g.K = pl.D; g.lda = pl.D; g.ldc = n;
        g.c_mode = dtype == ASTRA_BF16 ? kCBf16 : kCF32;
    };
    local(pr[0], wq, bq, Q, pl.dq);
    local(pr[1], wk, bk, K, pl.dkv);
    local(pr[2], wv, bv, V, pl.dkv);
    GemmProblem po = {};
    po.a = O; po.b = wo; po.bias = bo; po.c = y_out; po.M = pl.Tq; po.N = pl.D; po.K = pl.dq; po.lda = pl.dq; po.ldc = pl.D;
    po.c_mode = kCF32;
    rc = launch_gemm_batch(dtype, pr, 3, s, nullptr, nullptr, true);      // both GEMM launches validated before anything runs
    if (rc) return rc;
    rc = launch_gemm_batch(dtype, &po, 1, s, nullptr, nullptr, true);
    if (rc) return rc;
    rc = launch_gemm_batch(dtype, pr, 3, s);
    if (rc) return rc;

    // 2. what this device transmits: codes of the content rows of K and of V (the class row is not sent).  Nothing else in
    //    the layer depends on them: they are offered to the attention launch, which runs them as extra workgroups on the
    //    compute units its light query blocks leave early; if it does not take them they run as kernels of their own.
    EncodeJob ej[2] = {};
    const void* enc_x[2] = {(const char*)K + (size_t)at.n_cls * pl.dkv * eb, (const char*)V + (size_t)at.n_cls * pl.dkv * eb};
    const void* enc_cb[2] = {codebook_k, codebook_v};
    const float* enc_cn[2] = {cnorm_k, cnorm_v};
    void* enc_out[2] = {codes_k_local_out, codes_v_local_out};
    for (int j = 0; j < 2; ++j) {
        ej[j].x = enc_x[j]; ej[j].codebook = enc_cb[j]; ej[j].cnorm = enc_cn[j]; ej[j].codes = enc_out[j]; ej[j].ldx = pl.dkv;
        ej[j].n_tokens = at.n_local; ej[j].G = vq.n_groups; ej[j].K = vq.codebook_size; ej[j].dg = pl.dkv / vq.n_groups;
        ej[j].code_bytes = code_bytes(vq.code_type);
    }
    const bool offer = dtype == ASTRA_BF16 && at.n_local > 0;
    bool enc_fused = false;

    // 3. the peers' keys and values, looked up from their codes; values go straight into the attention's layout
    if (pl.vt) {
        // bf16: the three gathers are one launch
        rc = launch_kv_pack(vq, codes_k_nonlocal, codes_v_nonlocal, codebook_k, codebook_v, V, pl.Tn_vis, pl.Tq, pl.dkv, Kh, Vh, pl.ldv_hat,
                            Vt, pl.ldv_loc, s);
        if (rc) return rc;
    } else if (pl.Tn_vis > 0) {
        rc = launch_vq_decode(vq, codes_k_nonlocal, pl.Tn_vis, codebook_k, Kh, s);
        if (rc) return rc;
        rc = launch_vq_decode(vq, codes_v_nonlocal, pl.Tn_vis, codebook_v, Vh, s);
        if (rc) return rc;
    }

    // 4. mixed-precision attention (Eq. 1) and the output projection
    AttnParams ap = attn_params(at, Q, K, pl.vt ? Vt : V, Kh, Vh, O, nullptr);
    ap.v_transposed = pl.vt ? 1 : 0;
    ap.valid_bits = (const unsigned long long*)valid_nonlocal_bits;
    ap.ldv_loc = pl.ldv_loc;
    ap.ldv_hat = pl.ldv_hat;
    rc = launch_attention(dtype, ap, at.head_dim, s, false, offer ? ej : nullptr, offer ? 2 : 0, offer ? &enc_fused : nullptr);
    if (rc) return rc;
    if (!enc_fused && at.n_local > 0) {
        for (int j = 0; j < 2; ++j) {
            rc = launch_vq_encode(vq, enc_x[j], pl.dkv, at.n_local, enc_cb[j], enc_cn[j], enc_out[j], s);
            if (rc) return rc;
        }
    }
    return launch_gemm_batch(dtype, &po, 1, s);
}

size_t astra_block_workspace_bytes(const astra_block_desc* desc) {
    BlockPlan bp;
    if (make_block_plan(desc, &bp) != ASTRA_OK) return 0;
    return bp.total;
}

// validate_only: every check of the call, no launch
static int block_forward_impl(const astra_block_desc* desc, const astra_block_weights* w, const float* x, const void* codes_nonlocal,
                              const uint64_t* valid_nonlocal_bits, float* x_out, void* codes_local_out, void* h_out,
                              void* workspace, size_t workspace_bytes, void* stream, bool validate_only) {
    BlockPlan bp;
    int rc = make_block_plan(desc, &bp);
    if (rc) return rc;
    const LayerPlan& pl = bp.layer;
    if (pl.Tq == 0) return ASTRA_OK;
    if (!w || !x || !x_out) return ASTRA_ERR_NULL;
    if (!w->codebook || !w->cnorm || !w->wq || !w->wk || !w->wv || !w->wo || !w->w1 || !w->w2) return ASTRA_ERR_NULL;
    if (desc->layer.attn.n_local > 0 && !codes_local_out) return ASTRA_ERR_NULL;
    if (pl.Tn_vis > 0 && !codes_nonlocal) return ASTRA_ERR_NULL;
    if (!workspace || workspace_bytes < bp.total) return ASTRA_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int dtype = desc->layer.vq.dtype;
    char* ws = (char*)workspace;
    void* h = h_out ? h_out : (void*)(ws + bp.off_h);
    void* a = ws + bp.off_a;
    const int F = bp.d_ff;
    // every launch of the block is validated before the first one is made
    int fused = 0;
    rc = layer_forward_impl(&desc->layer, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                            nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr, &fused);
    if (rc) return rc;

    // x_out = r + mlp(h2), h2 = norm2(r) in the slot of the normalised rows of the first half (dead by then, unless
    // the caller asked for them in h_out)
    void* h2 = ws + bp.off_h;
    GemmProblem g1 = {};
    g1.a = h2; g1.b = w->w1; g1.bias = w->b1; g1.c = a; g1.M = pl.Tq; g1.K = pl.D; g1.lda = pl.D;
    if (desc->mlp_kind == ASTRA_MLP_SWIGLU) {
        g1.N = 2 * F;
        if (dtype == ASTRA_BF16) { g1.c_mode = kCSwiGLU; g1.ldc = F; }
        else { g1.c = ws + bp.off_a2; g1.c_mode = kCF32; g1.ldc = 2 * F; }
    } else {
        g1.N = F; g1.ldc = F;
        g1.c_mode = dtype == ASTRA_BF16 ? kCBf16 : kCF32;
        g1.act = desc->mlp_kind == ASTRA_MLP_GELU_TANH ? kActGeluTanh : kActGeluErf;
    }
    GemmProblem g2 = {};
    g2.a = a; g2.b = w->w2; g2.bias = w->b2; g2.c = x_out; g2.M = pl.Tq; g2.N = pl.D; g2.K = F; g2.lda = F; g2.ldc = pl.D;
    g2.c_mode = kCF32;
    g2.residual = x_out;
    rc = launch_gemm_batch(dtype, &g1, 1, s, nullptr, nullptr, true);
    if (rc) return rc;
    rc = launch_gemm_batch(dtype, &g2, 1, s, nullptr, nullptr, true);
    if (rc) return rc;
    if (validate_only) return ASTRA_OK;

    // h = norm1(x) in the layer's element type: the tensor that is quantised and projected
    rc = launch_norm(dtype, desc->norm_kind, x, pl.Tq, pl.D, desc->eps, w->norm1_gain, w->norm1_bias, h, s);
    if (rc) return rc;
    // r = x + layer(h), written to x_out by the output projection's epilogue
    rc = layer_forward_impl(&desc->layer, h, codes_nonlocal, w->codebook, w->cnorm, w->wq, w->wk, w->wv, w->wo, w->bq, w->bk, w->bv,
                            w->bo, x_out, codes_local_out, workspace, pl.total, stream, nullptr, nullptr, valid_nonlocal_bits, x,
                            nullptr, nullptr, desc->rope_base);
    if (rc) return rc;
    rc = launch_norm(dtype, desc->norm_kind, x_out, pl.Tq, pl.D, desc->eps, w->norm2_gain, w->norm2_bias, h2, s);
    if (rc) return rc;
    rc = launch_gemm_batch(dtype, &g1, 1, s);
    if (rc) return rc;
    if (desc->mlp_kind == ASTRA_MLP_SWIGLU && dtype != ASTRA_BF16) {
        rc = launch_swiglu_f32((const float*)(ws + bp.off_a2), pl.Tq, F, (float*)a, s);
        if (rc) return rc;
    }
    return launch_gemm_batch(dtype, &g2, 1, s, nullptr, nullptr, false, ws + bp.off_split, bp.split_bytes);
}

int astra_block_forward(const astra_block_desc* desc, const astra_block_weights* w, const float* x, const void* codes_nonlocal,
                        const uint64_t* valid_nonlocal_bits, float* x_out, void* codes_local_out, void* h_out,
                        void* workspace, size_t workspace_bytes, void* stream) {
    return block_forward_impl(desc, w, x, codes_nonlocal, valid_nonlocal_bits, x_out, codes_local_out, h_out, workspace,
                              workspace_bytes, stream, false);
}

int astra_stack_forward(const astra_block_desc* desc, int32_t n_layers, const astra_block_weights* weights, const float* x,
                        const void* const* codes_nonlocal, const uint64_t* const* valid_nonlocal_bits, float* x_out,
                        void* const* codes_local_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (n_layers < 0) return ASTRA_ERR_SHAPE;
    if (!desc) return ASTRA_ERR_NULL;
    if (n_layers == 0) return ASTRA_OK;
    if (!weights || !codes_nonlocal || !codes_local_out) return ASTRA_ERR_NULL;
    // two passes: validate every block, then launch them; block 0 reads x, the others continue in place on x_out
    for (int pass = 0; pass < 2; ++pass)
        for (int l = 0; l < n_layers; ++l) {
            const int rc = block_forward_impl(desc, &weights[l], l == 0 ? x : x_out, codes_nonlocal[l],
                                              valid_nonlocal_bits ? valid_nonlocal_bits[l] : nullptr, x_out, codes_local_out[l],
                                              nullptr, workspace, workspace_bytes, stream, pass == 0);
            if (rc) return rc;
        }
    return ASTRA_OK;
}

int astra_layer_forward_profiled(const astra_layer_desc* desc, const void* x_local, const void* codes_nonlocal,
                                 const void* codebook, const float* cnorm,
                                 const void* wq, const void* wk, const void* wv, const void* wo,
                                 const void* bq, const void* bk, const void* bv, const void* bo,
                                 void* y_out, void* codes_local_out, void* workspace, size_t workspace_bytes, void* stream,
                                 void* const* stage_events) {
    if (!stage_events) return ASTRA_ERR_NULL;
    return layer_forward_impl(desc, x_local, codes_nonlocal, codebook, cnorm, wq, wk, wv, wo, bq, bk, bv, bo, y_out,
                              codes_local_out, workspace, workspace_bytes, stream, stage_events);
}

}  // extern "C"
