"""Pins for the oracle's lost-code variants (Sec. 4.5 "Non-Ideal Network Conditions" / App. E: packet loss
without retransmission; reading: a non-local token whose codes never arrived is dropped from the key/value
set).  The variant is pinned to the already pinned full path: dropping rows must equal physically removing
them, an all-ones mask must change nothing, an all-zero mask must equal having no non-local tokens."""
import numpy as np
import pytest

import oracle


def rand_qkv(rng, tq, tn, hq, hkv, dh):
    f = lambda *s: rng.standard_normal(s)
    return f(tq, hq, dh), f(tq, hkv, dh), f(tq, hkv, dh), f(tn, hkv, dh), f(tn, hkv, dh)


@pytest.mark.parametrize("causal,n_before", [(False, 0), (True, 23), (True, 0), (True, 37)])
def test_dropping_rows_equals_removing_them(causal, n_before):
    rng = np.random.default_rng(5)
    q, k, v, kh, vh = rand_qkv(rng, 13, 37, 6, 3, 8)
    valid = rng.random(37) > 0.3
    valid[[0, 36]] = [False, True]
    out, lse = oracle.mixed_attention(q, k, v, kh, vh, causal=causal, n_before=n_before, valid_hat=valid, return_lse=True)
    # the same attention with the lost rows physically removed; under causal masking the count of rows before the chunk shrinks with them
    nb = int(valid[:n_before].sum()) if causal else 0
    ref, lse_ref = oracle.mixed_attention(q, k, v, kh[valid], vh[valid], causal=causal, n_before=nb, return_lse=True)
    np.testing.assert_allclose(out, ref, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(lse, lse_ref, rtol=1e-13, atol=1e-13)
    # and the dropped rows matter: the unmasked result differs
    if valid[: (n_before if causal else 37)].sum() < (n_before if causal else 37):
        full = oracle.mixed_attention(q, k, v, kh, vh, causal=causal, n_before=n_before)
        assert np.abs(full - out).max() > 1e-6


def test_all_valid_changes_nothing_and_all_lost_equals_no_nonlocal_tokens():
    rng = np.random.default_rng(6)
    q, k, v, kh, vh = rand_qkv(rng, 9, 20, 4, 4, 16)
    base = oracle.mixed_attention(q, k, v, kh, vh)
    np.testing.assert_array_equal(oracle.mixed_attention(q, k, v, kh, vh, valid_hat=np.ones(20)), base)
    none = oracle.mixed_attention(q, k, v, kh[:0], vh[:0])
    np.testing.assert_allclose(oracle.mixed_attention(q, k, v, kh, vh, valid_hat=np.zeros(20)), none, rtol=1e-13, atol=1e-13)


def test_probabilities_of_lost_rows_are_zero_and_rows_sum_to_one():
    rng = np.random.default_rng(7)
    q, k, v, kh, vh = rand_qkv(rng, 5, 11, 2, 2, 4)
    valid = np.array([1, 0, 1, 1, 0, 0, 1, 1, 1, 0, 1])
    _, probs = oracle.mixed_attention(q, k, v, kh, vh, valid_hat=valid, return_probs=True)
    assert np.all(probs[:, :, 5:][:, :, valid == 0] == 0.0)
    np.testing.assert_allclose(probs.sum(-1), 1.0, rtol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_layer_with_lost_rows_equals_layer_without_those_rows(causal):
    """Whole layer: whatever sits in the slot of a lost row (here: out-of-range garbage) is never looked up."""
    rng = np.random.default_rng(8)
    D, G, K, hq, hkv, dh, tl, tn = 24, 4, 8, 4, 2, 6, 7, 15
    x = rng.standard_normal((tl, D)).astype(np.float32)
    cb = rng.standard_normal((G, K, D // G)).astype(np.float32)
    w = [(0.3 * rng.standard_normal(s)).astype(np.float32) for s in ((D, hq * dh), (D, hkv * dh), (D, hkv * dh), (hq * dh, D))]
    codes = rng.integers(0, K, (tn, G)).astype(np.int32)
    valid = rng.random(tn) > 0.35
    valid[3] = False
    garbage = codes.copy()
    garbage[~valid] = 10_000                      # an index no codebook has
    n_before = 9 if causal else 0
    y, c = oracle.layer_forward(x, garbage, cb, *w, n_q_heads=hq, n_kv_heads=hkv, causal=causal, n_before=n_before,
                                valid_nonlocal=valid)
    nb = int(valid[:n_before].sum()) if causal else 0
    y_ref, c_ref = oracle.layer_forward(x, codes[valid], cb, *w, n_q_heads=hq, n_kv_heads=hkv, causal=causal, n_before=nb)
    np.testing.assert_allclose(y, y_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(c, c_ref)
    with pytest.raises(ValueError):               # without the mask the garbage index is an error
        oracle.layer_forward(x, garbage, cb, *w, n_q_heads=hq, n_kv_heads=hkv, causal=causal, n_before=n_before)
