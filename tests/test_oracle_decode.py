"""Pins for the oracle's decoding step over an index KV cache (App. "Memory Cost Analysis": local keys and values at
full precision, non-local ones as one index per group per token; Sec. 3.1: decoding proceeds on the device that holds
the most recent token).  Pinned to torch's attention routine on the looked-up rows, to the prefill oracle (the last
row of a causal layer sees exactly this cache), and by special cases."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle


def t64(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def make(rng, hq=6, hkv=3, dh=8, tl=9, tn=14, G=4, K=16):
    dkv = hkv * dh
    return dict(q=rng.standard_normal((hq, dh)), k=rng.standard_normal((tl, hkv, dh)), v=rng.standard_normal((tl, hkv, dh)),
                ck=rng.integers(0, K, (tn, G)).astype(np.int32), cv=rng.integers(0, K, (tn, G)).astype(np.int32),
                cbk=rng.standard_normal((G, K, dkv // G)).astype(np.float32), cbv=rng.standard_normal((G, K, dkv // G)).astype(np.float32))


@pytest.mark.parametrize("G", [1, 4, 6])       # 6 groups of 4 over 3 heads of 8: groups line up with heads; 4 groups of 6 straddle them
def test_equals_library_attention_on_the_looked_up_rows(G):
    rng = np.random.default_rng(70 + G)
    p = make(rng, G=G)
    out, lse = oracle.decode_attention(p["q"], p["k"], p["v"], p["ck"], p["cv"], p["cbk"], p["cbv"], return_lse=True)
    kh = oracle.vq_decode(p["ck"], p["cbk"]).reshape(14, 3, 8)
    vh = oracle.vq_decode(p["cv"], p["cbv"]).reshape(14, 3, 8)
    k_all = torch.cat([t64(p["k"]), t64(kh)]).repeat_interleave(2, dim=1).transpose(0, 1)      # [H_q, T, dh]
    v_all = torch.cat([t64(p["v"]), t64(vh)]).repeat_interleave(2, dim=1).transpose(0, 1)
    ref = F.scaled_dot_product_attention(t64(p["q"])[:, None, :], k_all, v_all)[:, 0, :]
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-12, atol=1e-12)
    s = torch.einsum("hc,htc->ht", t64(p["q"]), k_all) / np.sqrt(8.0)
    np.testing.assert_allclose(lse, torch.logsumexp(s, dim=-1).numpy(), rtol=1e-12)


def test_last_row_of_a_causal_prefill_sees_exactly_this_cache():
    """The decode step for the newest token equals Eq. 1 for the last local row of a causal chunk that follows all
    non-local rows: same keys, same values, same result."""
    rng = np.random.default_rng(75)
    p = make(rng)
    qs = rng.standard_normal((9, 6, 8))
    qs[-1] = p["q"]
    kh = oracle.vq_decode(p["ck"], p["cbk"]).reshape(14, 3, 8)
    vh = oracle.vq_decode(p["cv"], p["cbv"]).reshape(14, 3, 8)
    full = oracle.mixed_attention(qs, p["k"], p["v"], kh, vh, causal=True, n_before=14)
    out = oracle.decode_attention(p["q"], p["k"], p["v"], p["ck"], p["cv"], p["cbk"], p["cbv"])
    np.testing.assert_allclose(out, full[-1], rtol=1e-12, atol=1e-12)


def test_special_cases():
    rng = np.random.default_rng(76)
    p = make(rng)
    base = oracle.decode_attention(p["q"], p["k"], p["v"], p["ck"], p["cv"], p["cbk"], p["cbv"])
    # no non-local tokens: plain attention over the local cache; no local tokens: attention over looked-up rows only
    a = oracle.decode_attention(p["q"], p["k"], p["v"], p["ck"][:0], p["cv"][:0], p["cbk"], p["cbv"])
    ref = F.scaled_dot_product_attention(t64(p["q"])[:, None, :], t64(p["k"]).repeat_interleave(2, dim=1).transpose(0, 1),
                                         t64(p["v"]).repeat_interleave(2, dim=1).transpose(0, 1))[:, 0, :]
    np.testing.assert_allclose(a, ref.numpy(), rtol=1e-12, atol=1e-12)
    # a single cached token: the output is its value row, whatever the query
    one = oracle.decode_attention(p["q"], p["k"][:1], p["v"][:1], p["ck"][:0], p["cv"][:0], p["cbk"], p["cbv"])
    np.testing.assert_allclose(one, np.repeat(p["v"][0], 2, axis=0), rtol=1e-14)
    # lost tokens equal removed tokens; key and value streams and codebooks are not interchangeable
    valid = rng.random(14) > 0.4
    lost = oracle.decode_attention(p["q"], p["k"], p["v"], p["ck"], p["cv"], p["cbk"], p["cbv"], valid=valid)
    removed = oracle.decode_attention(p["q"], p["k"], p["v"], p["ck"][valid], p["cv"][valid], p["cbk"], p["cbv"])
    np.testing.assert_allclose(lost, removed, rtol=1e-12, atol=1e-12)
    swapped = oracle.decode_attention(p["q"], p["k"], p["v"], p["cv"], p["ck"], p["cbk"], p["cbv"])
    assert np.abs(swapped - base).max() > 1e-3
    # scale: an explicit 1/sqrt(dh) is the default
    np.testing.assert_array_equal(oracle.decode_attention(p["q"], p["k"], p["v"], p["ck"], p["cv"], p["cbk"], p["cbv"],
                                                          scale=1 / np.sqrt(8.0)), base)
