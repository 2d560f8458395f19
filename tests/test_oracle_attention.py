"""Pins for the CPU oracle's projections, mixed-precision attention (Eq. 1) and layer (Sec. 3.1).
Checks use library routines (numpy matmul, torch SDPA on CPU in fp64, scipy logsumexp), the
single-device masked formulation of the same attention written independently below, special
cases that reduce to plain attention, and invariants."""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp

import oracle


def sdpa(q, k, v, causal=False, scale=None):
    """Library attention on [T, H, dh] arrays (fp64, CPU)."""
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).permute(1, 0, 2)[None] for a in (q, k, v))
    if tk.shape[1] != tq.shape[1]:
        rep = tq.shape[1] // tk.shape[1]
        tk, tv = tk.repeat_interleave(rep, dim=1), tv.repeat_interleave(rep, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


def rand_qkv(rng, tq, tn, hq, hkv, dh):
    f = lambda *s: rng.standard_normal(s)
    return f(tq, hq, dh), f(tq, hkv, dh), f(tq, hkv, dh), f(tn, hkv, dh), f(tn, hkv, dh)


def test_linear_is_matmul_plus_bias():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 5))
    w = rng.standard_normal((5, 3)).astype(np.float32)      # non-square: a transposed read cannot pass
    b = rng.standard_normal(3).astype(np.float32)
    np.testing.assert_allclose(oracle.linear(x, w, b), x @ w.astype(np.float64) + b, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.linear(x, w), x @ w.astype(np.float64), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2)])
def test_all_local_is_plain_attention(hq, hkv):
    rng = np.random.default_rng(1)
    q, k, v, kh, vh = rand_qkv(rng, 19, 0, hq, hkv, 16)
    out = oracle.mixed_attention(q, k, v, kh, vh)
    np.testing.assert_allclose(out, sdpa(q, k, v), rtol=1e-10, atol=1e-12)
    # first device of a causal model: nothing precedes it -> plain causal attention on its chunk
    out_c = oracle.mixed_attention(q, k, v, kh, vh, causal=True, n_before=0)
    np.testing.assert_allclose(out_c, sdpa(q, k, v, causal=True), rtol=1e-10, atol=1e-12)


def test_causal_hides_following_chunks_entirely():
    rng = np.random.default_rng(2)
    q, k, v, kh, vh = rand_qkv(rng, 9, 12, 2, 2, 8)
    a = oracle.mixed_attention(q, k, v, kh, vh, causal=True, n_before=5)
    b = oracle.mixed_attention(q, k, v, kh[:5], vh[:5], causal=True, n_before=5)
    np.testing.assert_allclose(a, b, rtol=0, atol=0)
    # and equals library causal attention over [preceding non-local | local] in global order
    kk, vv = np.concatenate([kh[:5], k]), np.concatenate([vh[:5], v])
    qq = np.concatenate([np.zeros((5, 2, 8)), q])
    np.testing.assert_allclose(a, sdpa(qq, kk, vv, causal=True)[5:], rtol=1e-10, atol=1e-12)


def test_noncausal_equals_library_attention_over_concatenation():
    rng = np.random.default_rng(3)
    q, k, v, kh, vh = rand_qkv(rng, 6, 10, 4, 2, 8)
    out, lse, probs = oracle.mixed_attention(q, k, v, kh, vh, return_lse=True, return_probs=True)
    kk, vv = np.concatenate([k, kh]), np.concatenate([v, vh])
    tq = q.shape[0]
    # library SDPA needs as many query rows as it likes; keys are the concatenation
    tq_t = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk_t = torch.from_numpy(kk).permute(1, 0, 2)[None].repeat_interleave(2, dim=1)
    tv_t = torch.from_numpy(vv).permute(1, 0, 2)[None].repeat_interleave(2, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq_t, tk_t, tv_t)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(probs.sum(axis=-1), 1.0, rtol=1e-12)        # softmax rows sum to 1
    logits = np.einsum("ihd,jhd->hij", q, np.repeat(kk, 2, axis=1)) / np.sqrt(8)
    np.testing.assert_allclose(lse, logsumexp(logits, axis=-1), rtol=1e-12)
    assert probs.shape == (4, tq, tq + 10)


def test_causal_probabilities_are_zero_on_excluded_pairs_and_sum_to_one():
    rng = np.random.default_rng(4)
    q, k, v, kh, vh = rand_qkv(rng, 7, 9, 2, 1, 4)
    _, probs = oracle.mixed_attention(q, k, v, kh, vh, causal=True, n_before=4, return_probs=True)
    np.testing.assert_allclose(probs.sum(axis=-1), 1.0, rtol=1e-12)
    for i in range(7):
        assert np.all(probs[:, i, i + 1:7] == 0) and np.all(probs[:, i, :i + 1] > 0)   # local part of [K | K-hat]
        assert np.all(probs[:, i, 7:7 + 4] > 0) and np.all(probs[:, i, 7 + 4:] == 0)   # non-local part


def test_scale_argument_and_default():
    rng = np.random.default_rng(5)
    q, k, v, kh, vh = rand_qkv(rng, 5, 3, 2, 2, 16)
    a = oracle.mixed_attention(q, k, v, kh, vh)
    b = oracle.mixed_attention(q, k, v, kh, vh, scale=0.25)              # 1/sqrt(16)
    np.testing.assert_allclose(a, b, rtol=1e-14)
    c = oracle.mixed_attention(q, k, v, kh, vh, scale=0.5)
    np.testing.assert_allclose(c, oracle.mixed_attention(2 * q, k, v, kh, vh, scale=0.25), rtol=1e-12)


def test_nonlocal_permutation_invariance():
    rng = np.random.default_rng(6)
    q, k, v, kh, vh = rand_qkv(rng, 5, 11, 3, 3, 8)
    perm = rng.permutation(11)
    np.testing.assert_allclose(oracle.mixed_attention(q, k, v, kh, vh),
                               oracle.mixed_attention(q, k, v, kh[perm], vh[perm]), rtol=1e-12, atol=1e-14)


def test_gqa_equals_mha_with_replicated_kv_heads():
    rng = np.random.default_rng(7)
    q, k, v, kh, vh = rand_qkv(rng, 6, 7, 8, 2, 8)
    rep = lambda a: np.repeat(a, 4, axis=1)       # consecutive query heads share a KV head
    np.testing.assert_allclose(oracle.mixed_attention(q, k, v, kh, vh),
                               oracle.mixed_attention(q, rep(k), rep(v), rep(kh), rep(vh)), rtol=1e-13)


def test_equal_values_give_that_value():
    rng = np.random.default_rng(8)
    q, k, v, kh, vh = rand_qkv(rng, 4, 6, 2, 2, 8)
    row = rng.standard_normal((1, 2, 8))
    out = oracle.mixed_attention(q, k, np.repeat(row, 4, 0), kh, np.repeat(row, 6, 0))
    np.testing.assert_allclose(out, np.repeat(row, 4, 0), rtol=1e-12)


def test_class_row_is_an_ordinary_local_row():
    rng = np.random.default_rng(9)
    q, k, v, kh, vh = rand_qkv(rng, 6, 5, 2, 2, 8)
    a = oracle.mixed_attention(q, k, v, kh, vh, n_cls=1)
    b = oracle.mixed_attention(q, k, v, kh, vh, n_cls=0)
    np.testing.assert_array_equal(a, b)
    # moving the class row to the end of the local block only moves its output row
    roll = lambda t: np.concatenate([t[1:], t[:1]])
    c = oracle.mixed_attention(roll(q), roll(k), roll(v), kh, vh)
    np.testing.assert_allclose(roll(a), c, rtol=1e-12, atol=1e-14)
    with pytest.raises(ValueError):
        oracle.mixed_attention(q, k, v, kh, vh, n_cls=1, causal=True)


# ---- layer level -------------------------------------------------------------------------

def make_layer(rng, n, d, hq, hkv, dh):
    x = rng.standard_normal((n, d)).astype(np.float32)
    w = lambda a, b: (rng.standard_normal((a, b)) / np.sqrt(a)).astype(np.float32)
    return x, w(d, hq * dh), w(d, hkv * dh), w(d, hkv * dh), w(hq * dh, d)


def full_attention_layer(x, wq, wk, wv, wo, hq, hkv, dh, causal):
    """Single-device, unquantised attention layer through library routines."""
    x64 = x.astype(np.float64)
    q = (x64 @ wq.astype(np.float64)).reshape(-1, hq, dh)
    k = (x64 @ wk.astype(np.float64)).reshape(-1, hkv, dh)
    v = (x64 @ wv.astype(np.float64)).reshape(-1, hkv, dh)
    return sdpa(q, k, v, causal=causal).reshape(x.shape[0], hq * dh) @ wo.astype(np.float64)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("rank", [0, 1, 3])
def test_lossless_codebook_recovers_single_device_attention(causal, rank):
    """If every non-local token is itself a codeword (G = 1), X-hat = X and the device's output
    must be the corresponding rows of ordinary attention over the whole sequence.  With
    causal=True this also fixes what n_before means (global positions, contiguous chunks)."""
    rng = np.random.default_rng(20 + rank)
    n, n_dev, d, hq, hkv, dh = 32, 4, 12, 4, 2, 6
    x, wq, wk, wv, wo = make_layer(rng, n, d, hq, hkv, dh)
    tl = n // n_dev
    lo, hi = rank * tl, (rank + 1) * tl
    x_nonlocal = np.concatenate([x[:lo], x[hi:]])
    codebook = x_nonlocal[None]                               # [1, K = T_n, D]
    codes_nonlocal = oracle.vq_encode(x_nonlocal, codebook)
    assert np.array_equal(codes_nonlocal[:, 0], np.arange(n - tl))
    y, codes_local = oracle.layer_forward(x[lo:hi], codes_nonlocal, codebook, wq, wk, wv, wo,
                                          n_q_heads=hq, n_kv_heads=hkv, causal=causal, n_before=lo)
    ref = full_attention_layer(x, wq, wk, wv, wo, hq, hkv, dh, causal)[lo:hi]
    np.testing.assert_allclose(y, ref, rtol=1e-9, atol=1e-11)
    assert np.array_equal(codes_local, oracle.vq_encode(x[lo:hi], codebook))


def global_masked_formulation(x, x_hat, owner, wq, wk, wv, wo, hq, hkv, dh, causal):
    """The training-time statement of Eq. 1: all devices at once on one machine; a (query, key)
    pair uses the full-precision key/value when both tokens sit on the same device and the
    quantised one otherwise.  Written with dense [N, N] selections, no per-device concatenation."""
    n = x.shape[0]
    x64, xh64 = x.astype(np.float64), x_hat.astype(np.float64)
    W = [w.astype(np.float64) for w in (wq, wk, wv, wo)]
    q = (x64 @ W[0]).reshape(n, hq, dh)
    kf, vf = (x64 @ W[1]).reshape(n, hkv, dh), (x64 @ W[2]).reshape(n, hkv, dh)
    kq, vq = (xh64 @ W[1]).reshape(n, hkv, dh), (xh64 @ W[2]).reshape(n, hkv, dh)
    same = owner[:, None] == owner[None, :]
    visible = np.tril(np.ones((n, n), dtype=bool)) if causal else np.ones((n, n), dtype=bool)
    out = np.zeros((n, hq, dh))
    for h in range(hq):
        hk = h // (hq // hkv)
        s_full = q[:, h] @ kf[:, hk].T
        s_quant = q[:, h] @ kq[:, hk].T
        s = np.where(same, s_full, s_quant) / np.sqrt(dh)
        s = np.where(visible, s, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        out[:, h] = (p * same) @ vf[:, hk] + (p * ~same) @ vq[:, hk]
    return out.reshape(n, hq * dh) @ W[3]


@pytest.mark.parametrize("causal", [False, True])
def test_per_device_concatenation_equals_global_masked_formulation(causal):
    rng = np.random.default_rng(30)
    n, n_dev, d, hq, hkv, dh, G, K = 24, 3, 8, 4, 2, 4, 2, 8
    x, wq, wk, wv, wo = make_layer(rng, n, d, hq, hkv, dh)
    codebook = rng.standard_normal((G, K, d // G)).astype(np.float32)
    codes = oracle.vq_encode(x, codebook)
    x_hat = oracle.vq_decode(codes, codebook)
    tl = n // n_dev
    owner = np.arange(n) // tl
    ref = global_masked_formulation(x, x_hat, owner, wq, wk, wv, wo, hq, hkv, dh, causal)
    for r in range(n_dev):
        lo, hi = r * tl, (r + 1) * tl
        codes_nl = np.concatenate([codes[:lo], codes[hi:]])
        y, cl = oracle.layer_forward(x[lo:hi], codes_nl, codebook, wq, wk, wv, wo,
                                     n_q_heads=hq, n_kv_heads=hkv, causal=causal, n_before=lo)
        np.testing.assert_allclose(y, ref[lo:hi], rtol=1e-9, atol=1e-11)
        assert np.array_equal(cl, codes[lo:hi])


def test_layer_class_row_first_not_encoded_and_biases():
    rng = np.random.default_rng(31)
    d, hq, hkv, dh, G, K = 8, 2, 2, 4, 2, 4
    x, wq, wk, wv, wo = make_layer(rng, 5, d, hq, hkv, dh)      # row 0 = class replica
    codebook = rng.standard_normal((G, K, d // G)).astype(np.float32)
    codes_nl = rng.integers(0, K, size=(6, G)).astype(np.int32)
    bq, bk, bv, bo = (rng.standard_normal(s).astype(np.float32) for s in (hq * dh, hkv * dh, hkv * dh, d))
    y, cl = oracle.layer_forward(x, codes_nl, codebook, wq, wk, wv, wo, n_q_heads=hq, n_kv_heads=hkv,
                                 n_cls=1, bq=bq, bk=bk, bv=bv, bo=bo)
    assert cl.shape == (4, G) and np.array_equal(cl, oracle.vq_encode(x[1:], codebook))
    # same thing assembled from library pieces
    x_hat = np.stack([codebook[g, codes_nl[:, g]] for g in range(G)], axis=1).reshape(6, d).astype(np.float64)
    x64 = x.astype(np.float64)
    q = (x64 @ wq + bq).reshape(5, hq, dh)
    k = np.concatenate([x64 @ wk + bk, x_hat @ wk + bk]).reshape(11, hkv, dh)
    v = np.concatenate([x64 @ wv + bv, x_hat @ wv + bv]).reshape(11, hkv, dh)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    o = torch.nn.functional.scaled_dot_product_attention(
        tq, torch.from_numpy(k).permute(1, 0, 2)[None], torch.from_numpy(v).permute(1, 0, 2)[None])
    ref = o[0].permute(1, 0, 2).reshape(5, hq * dh).numpy() @ wo.astype(np.float64) + bo
    np.testing.assert_allclose(y, ref, rtol=1e-9, atol=1e-11)
