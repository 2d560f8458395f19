"""Pins for the oracle's KV-space layer (App. "Memory Cost Analysis": C = 2 codebooks per layer of dimension
H_kv * dh; keys and values are quantised after projection and the receivers look them up without projecting).
Pinned to torch's attention routine through lossless codebooks, to the separately pinned encode / linear functions
for what is sent, and by special cases that tell the two codebooks and the two code streams apart."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2505_19342_amd import workloads as wl


def t64(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def make(rng, D=20, hq=4, hkv=2, dh=6, tl=7, tn=11, G=3, K=16):
    f32 = lambda a: np.asarray(a, dtype=np.float32)
    dkv = hkv * dh
    return dict(x=f32(rng.standard_normal((tl, D))), xn=f32(rng.standard_normal((tn, D))),
                wq=f32(0.4 * rng.standard_normal((D, hq * dh))), wk=f32(0.4 * rng.standard_normal((D, dkv))),
                wv=f32(0.4 * rng.standard_normal((D, dkv))), wo=f32(0.4 * rng.standard_normal((hq * dh, D))),
                bq=f32(rng.standard_normal(hq * dh)), bk=f32(rng.standard_normal(dkv)), bv=f32(rng.standard_normal(dkv)),
                bo=f32(rng.standard_normal(D)),
                cbk=f32(rng.standard_normal((G, K, dkv // G))), cbv=f32(rng.standard_normal((G, K, dkv // G))),
                ck=rng.integers(0, K, (tn, G)).astype(np.int32), cv=rng.integers(0, K, (tn, G)).astype(np.int32))


@pytest.mark.parametrize("causal", [False, True])
def test_lossless_codebooks_give_full_attention_over_the_whole_sequence(causal):
    """G = 1 and the K (V) codebook lists the peers' exact K (V) rows: the layer must equal ordinary attention of
    the local queries over the whole sequence, computed by torch (grouped-query heads expanded by hand)."""
    rng = np.random.default_rng(61)
    hq, hkv, dh, D, tl, tn, nb = 4, 2, 6, 20, 7, 11, 5
    p = make(rng, D=D, hq=hq, hkv=hkv, dh=dh, tl=tl, tn=tn)
    kn = (t64(p["xn"]) @ t64(p["wk"]) + t64(p["bk"])).to(torch.float32)
    vn = (t64(p["xn"]) @ t64(p["wv"]) + t64(p["bv"])).to(torch.float32)
    ids = np.arange(tn, dtype=np.int32)[:, None]
    got = oracle.layer_forward_kv(p["x"], ids, ids, kn.numpy()[None], vn.numpy()[None], p["wq"], p["wk"], p["wv"], p["wo"],
                                  n_q_heads=hq, n_kv_heads=hkv, causal=causal, n_before=nb,
                                  bq=p["bq"], bk=p["bk"], bv=p["bv"], bo=p["bo"])
    # the whole sequence in order: non-local rows before the chunk, the chunk, the rows after it
    xl = t64(p["x"])
    q = (xl @ t64(p["wq"]) + t64(p["bq"])).view(tl, hq, dh)
    kl = (xl @ t64(p["wk"]) + t64(p["bk"])).to(torch.float32).to(torch.float64)
    vl = (xl @ t64(p["wv"]) + t64(p["bv"])).to(torch.float32).to(torch.float64)
    k_all = torch.cat([kn[:nb].double(), kl, kn[nb:].double()]).view(tl + tn, hkv, dh).repeat_interleave(hq // hkv, dim=1)
    v_all = torch.cat([vn[:nb].double(), vl, vn[nb:].double()]).view(tl + tn, hkv, dh).repeat_interleave(hq // hkv, dim=1)
    mask = torch.ones(tl, tl + tn, dtype=torch.bool)
    if causal:
        pos_q = torch.arange(nb, nb + tl)[:, None]
        mask = torch.arange(tl + tn)[None, :] <= pos_q
    o = F.scaled_dot_product_attention(q.transpose(0, 1), k_all.transpose(0, 1), v_all.transpose(0, 1), attn_mask=mask)
    ref = o.transpose(0, 1).reshape(tl, hq * dh) @ t64(p["wo"]) + t64(p["bo"])
    np.testing.assert_allclose(got["y"], ref.numpy(), rtol=1e-10, atol=1e-10)


def test_what_is_sent_is_the_encode_of_the_stored_k_and_v_rows():
    rng = np.random.default_rng(62)
    p = make(rng)
    for bf16 in (False, True):
        got = oracle.layer_forward_kv(np.concatenate([p["x"][:1], p["x"]]), p["ck"], p["cv"], p["cbk"], p["cbv"], p["wq"], p["wk"],
                                      p["wv"], p["wo"], n_q_heads=4, n_kv_heads=2, n_cls=1, bk=p["bk"], bv=p["bv"], kv_is_bf16=bf16)
        xl = np.concatenate([p["x"][:1], p["x"]])
        k = oracle.linear(xl, p["wk"], p["bk"]).astype(np.float32)
        v = oracle.linear(xl, p["wv"], p["bv"]).astype(np.float32)
        if bf16:
            k, v = wl.round_to_bf16(k), wl.round_to_bf16(v)
            assert not np.any(got["k"].view(np.uint32) & 0xFFFF)
        np.testing.assert_array_equal(got["k"], k)
        np.testing.assert_array_equal(got["v"], v)
        # the class row is not sent; K rows go through the K codebook, V rows through the V codebook
        np.testing.assert_array_equal(got["codes_k"], oracle.vq_encode(k[1:], p["cbk"]))
        np.testing.assert_array_equal(got["codes_v"], oracle.vq_encode(v[1:], p["cbv"]))
        assert got["codes_k"].shape == (7, 3)
        assert np.any(got["codes_k"] != oracle.vq_encode(k[1:], p["cbv"]))


def test_equals_mixed_attention_on_the_looked_up_rows_and_keeps_the_streams_apart():
    rng = np.random.default_rng(63)
    p = make(rng)
    kw = dict(n_q_heads=4, n_kv_heads=2, causal=True, n_before=6)
    got = oracle.layer_forward_kv(p["x"], p["ck"], p["cv"], p["cbk"], p["cbv"], p["wq"], p["wk"], p["wv"], p["wo"], **kw)
    q = oracle.linear(p["x"], p["wq"]).reshape(7, 4, 6)
    k = got["k"].astype(np.float64).reshape(7, 2, 6)
    v = got["v"].astype(np.float64).reshape(7, 2, 6)
    kh = oracle.vq_decode(p["ck"], p["cbk"]).reshape(11, 2, 6)
    vh = oracle.vq_decode(p["cv"], p["cbv"]).reshape(11, 2, 6)
    o = oracle.mixed_attention(q, k, v, kh, vh, causal=True, n_before=6)
    np.testing.assert_allclose(got["y"], oracle.linear(o.reshape(7, 24), p["wo"]), rtol=1e-12, atol=1e-12)
    # swapping the two code streams, or the two codebooks, is a different computation
    a = oracle.layer_forward_kv(p["x"], p["cv"], p["ck"], p["cbk"], p["cbv"], p["wq"], p["wk"], p["wv"], p["wo"], **kw)["y"]
    b = oracle.layer_forward_kv(p["x"], p["ck"], p["cv"], p["cbv"], p["cbk"], p["wq"], p["wk"], p["wv"], p["wo"], **kw)["y"]
    assert np.abs(a - got["y"]).max() > 1e-3 and np.abs(b - got["y"]).max() > 1e-3


def test_lost_rows_equal_removed_rows():
    rng = np.random.default_rng(64)
    p = make(rng)
    valid = rng.random(11) > 0.4
    kw = dict(n_q_heads=4, n_kv_heads=2)
    a = oracle.layer_forward_kv(p["x"], p["ck"], p["cv"], p["cbk"], p["cbv"], p["wq"], p["wk"], p["wv"], p["wo"], valid_nonlocal=valid, **kw)
    b = oracle.layer_forward_kv(p["x"], p["ck"][valid], p["cv"][valid], p["cbk"], p["cbv"], p["wq"], p["wk"], p["wv"], p["wo"], **kw)
    np.testing.assert_allclose(a["y"], b["y"], rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(a["codes_k"], b["codes_k"])
