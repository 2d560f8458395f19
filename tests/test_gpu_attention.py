"""GPU parity: mixed-precision attention (Eq. 1) through the C ABI against the CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_2505_19342_amd import workloads as wl

pytestmark = pytest.mark.gpu

# Tolerances on attention outputs whose magnitude is O(1): bf16 rounds the probabilities and the output
# (relative 2^-9 each) and the inputs are already bf16, fp32 only reorders sums.
TOL = {"bf16": 2e-2, "f32": 2e-5}


def rand_case(seed, Tq, Tn, Hq, Hkv, dh, dtype, sigma=1.0):
    rng = np.random.default_rng(seed)
    f = lambda *s: (sigma * rng.standard_normal(s)).astype(np.float32)
    arrs = [f(Tq, Hq, dh), f(Tq, Hkv, dh), f(Tq, Hkv, dh), f(Tn, Hkv, dh), f(Tn, Hkv, dh)]
    if dtype == "bf16":
        arrs = [wl.round_to_bf16(a) for a in arrs]
    return arrs


CASES = [
    # Tq, Tn, Hq, Hkv, dh, dtype, n_cls, causal, n_before
    (64, 192, 3, 3, 64, "f32", 0, False, 0),          # tiny ViT
    (50, 70, 4, 2, 32, "f32", 1, False, 0),           # fp32, GQA, class row, ragged
    (40, 90, 2, 2, 128, "f32", 0, True, 37),          # fp32 causal, middle rank
    (257, 768, 12, 12, 64, "bf16", 1, False, 0),      # ViT-Base with class row (ragged 257)
    (256, 768, 12, 12, 64, "bf16", 0, True, 768),     # GPT-2 small, last rank
    (256, 768, 12, 12, 64, "bf16", 0, True, 256),     # GPT-2 small, rank 1
    (256, 768, 12, 12, 64, "bf16", 0, True, 0),       # GPT-2 small, rank 0 == plain causal
    (300, 0, 4, 4, 64, "bf16", 0, False, 0),          # all tokens local
    (300, 0, 8, 2, 128, "bf16", 0, True, 0),
    (1, 5, 2, 1, 128, "bf16", 0, False, 0),           # single query row
    (130, 333, 8, 2, 128, "bf16", 0, False, 0),       # GQA, ragged everywhere
    (200, 450, 8, 2, 128, "bf16", 0, True, 333),      # GQA causal, ragged, some non-local rows hidden
    # 64-wide heads run on 64-row query blocks with four tile parities while 128-row blocks would fill at most half of the
    # chip (every case above); beyond that on 128-row blocks with two:
    (1500, 600, 12, 12, 64, "bf16", 1, False, 0),     # 144 blocks of 128 rows: two parities, class row, ragged
    (1400, 650, 12, 4, 64, "bf16", 0, True, 650),     # the same kernel causal with grouped queries
    (70, 131, 12, 12, 64, "bf16", 0, True, 131),      # four parities, three tiles + a key: dummy tiles in the last iteration
    (1, 5, 2, 1, 64, "bf16", 0, False, 0),            # four parities, a single query row and a single tile
    (65, 1, 4, 2, 64, "bf16", 1, False, 0),           # a second query block of one row; one non-local key; class row
    (129, 260, 4, 4, 64, "bf16", 0, True, 100),       # causal with rows of the non-local set hidden, ragged blocks
]


@pytest.mark.parametrize("Tq,Tn,Hq,Hkv,dh,dtype,n_cls,causal,n_before", CASES)
def test_attention_matches_oracle(Tq, Tn, Hq, Hkv, dh, dtype, n_cls, causal, n_before):
    from gpu_util import gpu_mixed_attention
    q, k, v, kh, vh = rand_case(Tq * 7 + Tn, Tq, Tn, Hq, Hkv, dh, dtype)
    ref, ref_lse = oracle.mixed_attention(q, k, v, kh, vh, n_cls=n_cls, causal=causal, n_before=n_before, return_lse=True)
    got, lse = gpu_mixed_attention(q, k, v, kh, vh, dtype, n_cls=n_cls, causal=causal, n_before=n_before, want_lse=True)
    err = np.abs(got - ref).max()
    print(f"max abs err {err:.3e}")
    assert err <= TOL[dtype]
    np.testing.assert_allclose(lse, ref_lse, atol=2e-3 if dtype == "bf16" else 1e-4)


def test_llama_shape_attention_sampled_rows():
    """Full-size Llama-3-8B-shaped attention (last rank): every row is computed on the GPU, rows the
    oracle recomputes are a seeded sample spanning every 128-row block."""
    from gpu_util import gpu_mixed_attention
    Tq, Tn, Hq, Hkv, dh = 1024, 3072, 32, 8, 128
    q, k, v, kh, vh = rand_case(5, Tq, Tn, Hq, Hkv, dh, "bf16")
    got = gpu_mixed_attention(q, k, v, kh, vh, "bf16", causal=True, n_before=Tn)
    rows = np.unique(np.concatenate([np.arange(0, Tq, 128), np.arange(127, Tq, 128),
                                     np.random.default_rng(0).integers(0, Tq, 24)]))
    # causal row i depends on local rows <= i only: recompute just those rows with the oracle
    for i in rows:
        ref = oracle.mixed_attention(q[i:i + 1], k[i:i + 1], v[i:i + 1],
                                     np.concatenate([kh, k[:i]]), np.concatenate([vh, v[:i]]),
                                     causal=True, n_before=Tn + i)
        assert np.abs(got[i] - ref[0]).max() <= TOL["bf16"]


def test_scale_and_large_logits():
    from gpu_util import gpu_mixed_attention
    q, k, v, kh, vh = rand_case(11, 70, 100, 2, 2, 64, "bf16", sigma=3.0)     # logits of order +-70: softmax near one-hot
    ref = oracle.mixed_attention(q, k, v, kh, vh, scale=0.125)
    got = gpu_mixed_attention(q, k, v, kh, vh, "bf16", scale=0.125)
    assert np.abs(got - ref).max() <= 6e-2          # values are 3x larger here
    ref2 = oracle.mixed_attention(q, k, v, kh, vh, scale=0.01)
    got2 = gpu_mixed_attention(q, k, v, kh, vh, "bf16", scale=0.01)
    assert np.abs(got2 - ref2).max() <= TOL["bf16"]


def test_argument_errors():
    import torch
    from gpu_util import DEV
    from paper_2505_19342_amd import binding as B
    t = torch.zeros((4, 2, 64), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.AstraError):      # class row with causal masking
        B.astra_mixed_attention(B.AttnDesc(B.ASTRA_BF16, 2, 2, 64, 1, 3, 0, 1, 0, 0.0), t, t, t, None, None, t)
    with pytest.raises(B.AstraError):      # H_kv does not divide H_q
        B.astra_mixed_attention(B.AttnDesc(B.ASTRA_BF16, 3, 2, 64, 0, 4, 0, 0, 0, 0.0), t, t, t, None, None, t)
    with pytest.raises(B.AstraError):      # non-local rows announced but not given
        B.astra_mixed_attention(B.AttnDesc(B.ASTRA_BF16, 2, 2, 64, 0, 4, 8, 0, 0, 0.0), t, t, t, None, None, t)
    with pytest.raises(B.AstraError):      # head_dim without a bf16 kernel
        B.astra_mixed_attention(B.AttnDesc(B.ASTRA_BF16, 2, 2, 48, 0, 4, 0, 0, 0, 0.0), t, t, t, None, None, t)
