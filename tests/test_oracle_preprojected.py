"""Pins for the oracle's pre-projected-codebook functions.  A rebuilt row is a concatenation of codewords (Sec. 3.2), so
its projection with the shared weights (text under Eq. 1) splits into per-group terms: project_codebook tabulates the
terms, gather_sum adds the ones a token's codes select.  Pinned to the separately pinned decode + linear (the identity the
method relies on), to numpy's matmul for one group, to a hand-worked example, and by cases that catch a shifted weight
slice, a bias added once per group, a swapped group or a transposed table."""
import numpy as np
import pytest

import oracle


def make(rng, G=3, K=7, dg=4, n=5, T=9):
    f32 = lambda a: np.asarray(a, dtype=np.float32)
    return (f32(rng.standard_normal((G, K, dg))), f32(rng.standard_normal((G * dg, n))), f32(rng.standard_normal(n)),
            rng.integers(0, K, (T, G)).astype(np.int32))


@pytest.mark.parametrize("G,K,dg,n,T", [(1, 5, 6, 4, 8), (2, 7, 3, 5, 9), (4, 16, 2, 3, 33), (8, 3, 1, 2, 5)])
def test_gather_sum_of_the_table_is_the_projection_of_the_rebuilt_rows(G, K, dg, n, T):
    cb, w, b, codes = make(np.random.default_rng(5 + G), G, K, dg, n, T)
    p = oracle.project_codebook(cb, w)
    assert p.shape == (G, K, n)
    want = oracle.linear(oracle.vq_decode(codes, cb), w, b)
    got = oracle.gather_sum(codes, p, b)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    # without a bias too (a bias added once per group would pass the G = 1 case only)
    np.testing.assert_allclose(oracle.gather_sum(codes, p), oracle.linear(oracle.vq_decode(codes, cb), w), rtol=0, atol=1e-12)


def test_one_group_is_a_plain_matrix_product_and_a_plain_lookup():
    cb, w, b, codes = make(np.random.default_rng(1), G=1, K=6, dg=5, n=4, T=7)
    p = oracle.project_codebook(cb, w)
    np.testing.assert_allclose(p[0], cb[0].astype(np.float64) @ w.astype(np.float64), rtol=0, atol=1e-13)
    np.testing.assert_array_equal(oracle.gather_sum(codes, p), p[0][codes[:, 0]])


def test_hand_worked_example():
    # two groups of width 1, two codewords each; w = [[1, 10], [100, 1000]]
    cb = np.array([[[1.0], [2.0]], [[3.0], [4.0]]], dtype=np.float32)
    w = np.array([[1.0, 10.0], [100.0, 1000.0]], dtype=np.float32)
    p = oracle.project_codebook(cb, w)
    np.testing.assert_array_equal(p, [[[1, 10], [2, 20]], [[300, 3000], [400, 4000]]])
    codes = np.array([[0, 0], [1, 0], [0, 1], [1, 1]], dtype=np.int32)
    np.testing.assert_array_equal(oracle.gather_sum(codes, p, np.array([0.5, 0.25], dtype=np.float32)),
                                  [[301.5, 3010.25], [302.5, 3020.25], [401.5, 4010.25], [402.5, 4020.25]])


def test_each_group_uses_its_own_weight_slice_and_its_own_codes():
    cb, w, _, codes = make(np.random.default_rng(2), G=3, K=5, dg=2, n=4, T=6)
    p = oracle.project_codebook(cb, w)
    # changing the weight rows of slice 1 changes table 1 only
    w2 = w.copy()
    w2[2:4] += 1.0
    p2 = oracle.project_codebook(cb, w2)
    np.testing.assert_array_equal(p2[0], p[0])
    np.testing.assert_array_equal(p2[2], p[2])
    assert np.abs(p2[1] - p[1]).max() > 0.1
    # changing the codes of group 2 changes the result by exactly the difference of the two table rows
    c2 = codes.copy()
    c2[:, 2] = (c2[:, 2] + 1) % 5
    d = oracle.gather_sum(c2, p) - oracle.gather_sum(codes, p)
    np.testing.assert_allclose(d, p[2][c2[:, 2]] - p[2][codes[:, 2]], rtol=0, atol=1e-12)


def test_the_layer_on_preprojected_tables_is_the_layer():
    """K-hat, V-hat from the tables fed to the attention give the layer's output: what the GPU's pre-projected path
    must reproduce is therefore oracle.layer_forward itself."""
    rng = np.random.default_rng(3)
    f32 = lambda a: np.asarray(a, dtype=np.float32)
    D, hq, hkv, dh, tl, tn, G, K = 12, 4, 2, 3, 5, 9, 2, 8
    x, cb = f32(rng.standard_normal((tl, D))), f32(rng.standard_normal((G, K, D // G)))
    wq, wk, wv, wo = (f32(0.4 * rng.standard_normal(s)) for s in ((D, hq * dh), (D, hkv * dh), (D, hkv * dh), (hq * dh, D)))
    bk, bv = f32(rng.standard_normal(hkv * dh)), f32(rng.standard_normal(hkv * dh))
    codes = rng.integers(0, K, (tn, G)).astype(np.int32)
    y_ref, _ = oracle.layer_forward(x, codes, cb, wq, wk, wv, wo, n_q_heads=hq, n_kv_heads=hkv, bk=bk, bv=bv)
    kh = oracle.gather_sum(codes, oracle.project_codebook(cb, wk), bk).reshape(tn, hkv, dh)
    vh = oracle.gather_sum(codes, oracle.project_codebook(cb, wv), bv).reshape(tn, hkv, dh)
    q = oracle.linear(x, wq).reshape(tl, hq, dh)
    k = oracle.linear(x, wk, bk).reshape(tl, hkv, dh)
    v = oracle.linear(x, wv, bv).reshape(tl, hkv, dh)
    o = oracle.mixed_attention(q, k, v, kh, vh)
    np.testing.assert_allclose(oracle.linear(o.reshape(tl, hq * dh), wo), y_ref, rtol=0, atol=1e-12)
