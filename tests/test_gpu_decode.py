"""GPU parity: one decoding step over a KV cache whose non-local part is VQ indices (App. "Memory Cost Analysis";
Sec. 3.1 hand-off to single-device decoding) through astra_decode_attention against the CPU oracle.
Bars: max-abs <= 1e-5 (fp32: same sums in another order) / 1e-2 (bf16: q, caches and codebooks are bf16 on both
sides, the arithmetic is fp32, only the output is rounded to bf16, 2^-9 relative); lse within 1e-4."""
import numpy as np
import pytest

import oracle
from paper_2505_19342_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}


def make_cache(cfg, n_local, n_nonlocal, seed, n_groups_kv=None, real_codes=True):
    """Seeded cache contents in the layer's element type: K, V rows of the local tokens (projections of seeded
    embeddings, as a prefill would have left them), the peers' code streams, the new token's query."""
    data = wl.generate_kv(cfg, n_groups_kv)
    rng = np.random.default_rng(seed)
    rnd = (lambda a: wl.round_to_bf16(a.astype(np.float32))) if cfg.dtype == "bf16" else (lambda a: a.astype(np.float32))
    hq, hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    G, K, _ = data["codebook_k"].shape
    x = rnd(rng.standard_normal((n_local + 1, cfg.d_model)))
    k = rnd(oracle.linear(x[:n_local], data["wk"])).reshape(n_local, hkv, dh)
    v = rnd(oracle.linear(x[:n_local], data["wv"])).reshape(n_local, hkv, dh)
    q = rnd(oracle.linear(x[n_local:], data["wq"])).reshape(hq, dh) * np.float32(2.0)      # sharper softmax than 0.02-scale weights give
    q = rnd(q)
    if real_codes and n_nonlocal > 0:
        xn = rnd(rng.standard_normal((n_nonlocal, cfg.d_model)))
        ck = oracle.vq_encode(rnd(oracle.linear(xn, data["wk"])), data["codebook_k"])
        cv = oracle.vq_encode(rnd(oracle.linear(xn, data["wv"])), data["codebook_v"])
    else:
        ck = rng.integers(0, K, (n_nonlocal, G)).astype(np.int32)
        cv = rng.integers(0, K, (n_nonlocal, G)).astype(np.int32)
    return data, q, k, v, ck, cv


def run_case(cfg, n_local, n_nonlocal, seed=0, valid=None, n_groups_kv=None, real_codes=True):
    import torch
    from gpu_util import to_dev, to_host, codes_to_dev, valid_bits_to_dev, empty_like_dtype, DEV
    from paper_2505_19342_amd import binding as B
    data, q, k, v, ck, cv = make_cache(cfg, n_local, n_nonlocal, seed, n_groups_kv, real_codes)
    ref, lse_ref = oracle.decode_attention(q, k, v, ck, cv, data["codebook_k"], data["codebook_v"], valid=valid, return_lse=True)
    dt = cfg.dtype
    G, K, _ = data["codebook_k"].shape
    desc = B.DecodeDesc(B.vq_desc(dt, cfg.n_kv_heads * cfg.head_dim, G, K), cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                        n_local, n_nonlocal, 0.0)
    out = empty_like_dtype((cfg.n_q_heads, cfg.head_dim), dt)
    lse = torch.empty(cfg.n_q_heads, dtype=torch.float32, device=DEV)
    ws = torch.empty(max(B.astra_decode_attention_workspace_bytes(desc), 256), dtype=torch.uint8, device=DEV)
    assert B.astra_decode_attention_workspace_bytes(desc) > 0
    d = lambda a: to_dev(a, dt) if a.shape[0] > 0 else None
    c = lambda a: codes_to_dev(a, K) if a.shape[0] > 0 else None
    args = (desc, to_dev(q, dt), d(k), d(v), c(ck), c(cv), None if valid is None else valid_bits_to_dev(valid),
            to_dev(data["codebook_k"], dt), to_dev(data["codebook_v"], dt), out, lse, ws)
    B.astra_decode_attention(*args)
    torch.cuda.synchronize()
    got, got_lse = to_host(out), lse.cpu().numpy()
    err = np.abs(got - ref).max()
    print(f"{cfg.name} n_local {n_local} n_nonlocal {n_nonlocal}: max abs err {err:.3e} (|out| max {np.abs(ref).max():.3f}), "
          f"lse err {np.abs(got_lse - lse_ref).max():.2e}")
    assert err <= TOL[dt]
    finite = np.isfinite(lse_ref)
    assert np.abs(got_lse - lse_ref)[finite].max(initial=0.0) <= 1e-4 and np.all(got_lse[~finite] == -np.inf)
    # a second call gives the same bits
    first = out.clone()
    B.astra_decode_attention(*args)
    torch.cuda.synchronize()
    assert torch.equal(first.view(torch.int16 if dt == "bf16" else torch.int32), out.view(torch.int16 if dt == "bf16" else torch.int32))
    return got


def test_tiny_vit_f32_groups_straddle_heads():
    run_case(wl.TINY_VIT, 64, 192)                 # dh 64, dg 48


def test_vit_base_bf16():
    run_case(wl.VIT_BASE, 256, 768)                # 12 heads of 64, dg 48


def test_gpt2_small_bf16():
    run_case(wl.GPT2_SMALL, 300, 777, seed=1)      # dg 24; ragged chunks


def test_llama3_8b_shape():
    run_case(wl.LLAMA3_8B, 1024, 3072, seed=2)     # grouped-query heads (4 per KV head), dh 128, dg 32, 16-bit codes


def test_llama_long_cache_takes_longer_chunks():
    run_case(wl.LLAMA3_8B, 3001, 37003, seed=3, real_codes=False)


@pytest.mark.parametrize("n_local,n_nonlocal", [(1, 0), (0, 5), (7, 1), (257, 255)])
def test_small_and_one_sided_caches(n_local, n_nonlocal):
    run_case(wl.GPT2_SMALL, n_local, n_nonlocal, seed=4)


def test_lost_tokens_and_an_empty_cache():
    rng = np.random.default_rng(9)
    valid = (rng.random(500) > 0.2).astype(np.uint8)
    a = run_case(wl.GPT2_SMALL, 100, 500, seed=5, valid=valid)
    b = run_case(wl.GPT2_SMALL, 100, 500, seed=5)
    assert np.abs(a - b).max() > 1e-4
    # every non-local token lost and no local token: nothing to attend to
    out = run_case(wl.GPT2_SMALL, 0, 70, seed=6, valid=np.zeros(70, dtype=np.uint8))
    assert np.all(out == 0.0)


def test_other_group_counts():
    run_case(wl.LLAMA3_8B, 200, 600, seed=7, n_groups_kv=8)        # one group per KV head
    run_case(wl.LLAMA3_8B, 200, 600, seed=8, n_groups_kv=64)       # eight groups per head
    run_case(wl.VIT_BASE, 100, 300, seed=9, n_groups_kv=1)         # one group across all heads
    run_case(wl.GPT2_SMALL, 100, 300, seed=10, n_groups_kv=64)     # groups of 12 channels: the two-channels-per-thread path
    run_case(wl.TINY_VIT, 33, 99, seed=11, n_groups_kv=16)         # the same in fp32


def test_code_widths_of_the_one_load_per_head_path():
    """A head's codes of a token are fetched as one aligned load when they fill 4 or 8 bytes: 16-bit codes of two groups
    (4 bytes) and of four groups (8 bytes) per 64-wide head; 8-bit codes of four groups are the GPT-2 cases above."""
    import dataclasses
    cfg = dataclasses.replace(wl.GPT2_SMALL, name="gpt2_k1024", codebook_size=1024, seed=21)
    run_case(cfg, 130, 700, seed=12, n_groups_kv=24, real_codes=False)      # dg 32: two groups per head
    run_case(cfg, 130, 1300, seed=13, n_groups_kv=48, real_codes=False)     # dg 16: four groups per head; passes of 512 with a ragged last one


def test_argument_errors():
    import torch
    from paper_2505_19342_amd import binding as B
    desc = B.DecodeDesc(B.vq_desc("bf16", 768, 32, 256), 12, 12, 64, 10, 10, 0.0)
    t = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(B.AstraError, match="workspace"):
        B.astra_decode_attention(desc, t, t, t, t, t, None, t, t, t, None, torch.zeros(16, dtype=torch.uint8, device="cuda:0"))
    with pytest.raises(B.AstraError, match="NULL"):
        B.astra_decode_attention(desc, t, None, t, t, t, None, t, t, t, None, t)
    bad = B.DecodeDesc(B.vq_desc("bf16", 700, 32, 256), 12, 12, 64, 10, 10, 0.0)
    assert B.astra_decode_attention_workspace_bytes(bad) == 0
    odd = B.DecodeDesc(B.vq_desc("bf16", 768, 256, 256), 12, 12, 64, 10, 10, 0.0)      # groups of 3 channels
    with pytest.raises(B.AstraError, match="no kernel"):
        B.astra_decode_attention(odd, t, t, t, t, t, None, t, t, t, None, t)
