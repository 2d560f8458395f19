"""GPU: astra_decode_attention_static (the decode step for callers that cannot allocate: its table and partial results
live in a scratch array inside the library's device image) against astra_decode_attention with a caller workspace.
Same kernels on the same inputs, so the outputs must agree bit for bit (the bar of the parity tests, 1e-2 bf16 /
1e-5 fp32 against the oracle, is met by the workspace entry point in test_gpu_decode.py); two calls in a row, the second
with a smaller input, so that what the first call left in the shared array cannot leak into the second."""
import numpy as np
import pytest

from paper_2505_19342_amd import workloads as wl

pytestmark = pytest.mark.gpu


def both_entry_points(cfg, n_local, n_nonlocal, seed, poison=None):
    import torch
    from gpu_util import to_dev, codes_to_dev, empty_like_dtype, DEV
    from test_gpu_decode import make_cache
    from paper_2505_19342_amd import binding as B
    data, q, k, v, ck, cv = make_cache(cfg, n_local, n_nonlocal, seed, real_codes=False)
    dt = cfg.dtype
    G, K, _ = data["codebook_k"].shape
    desc = B.DecodeDesc(B.vq_desc(dt, cfg.n_kv_heads * cfg.head_dim, G, K), cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                        n_local, n_nonlocal, 0.0)
    need = B.astra_decode_attention_workspace_bytes(desc)
    assert 0 < need <= B.astra_decode_attention_static_max_bytes()
    d = lambda a: to_dev(a, dt) if a.shape[0] > 0 else None
    c = lambda a: codes_to_dev(a, K) if a.shape[0] > 0 else None
    common = (desc, to_dev(q, dt), d(k), d(v), c(ck), c(cv), None, to_dev(data["codebook_k"], dt), to_dev(data["codebook_v"], dt))
    out_ws, out_st = empty_like_dtype((cfg.n_q_heads, cfg.head_dim), dt), empty_like_dtype((cfg.n_q_heads, cfg.head_dim), dt)
    lse_ws = torch.empty(cfg.n_q_heads, dtype=torch.float32, device=DEV)
    lse_st = torch.empty(cfg.n_q_heads, dtype=torch.float32, device=DEV)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    B.astra_decode_attention(*common, out_ws, lse_ws, ws)
    B.astra_decode_attention_static(*common, out_st, lse_st)
    torch.cuda.synchronize()
    as_bits = lambda t: t.view(torch.int16 if dt == "bf16" else torch.int32)
    assert torch.isfinite(out_st.float()).all()
    assert torch.equal(as_bits(out_ws), as_bits(out_st)), f"{cfg.name} {n_local}+{n_nonlocal}: outputs differ"
    assert torch.equal(lse_ws.view(torch.int32), lse_st.view(torch.int32))
    return out_st.float().cpu().numpy()


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    big = both_entry_points(wl.LLAMA3_8B, 1024, 3072, seed=21)
    small = both_entry_points(wl.LLAMA3_8B, 130, 200, seed=22)          # fewer chunks, shorter table use
    assert np.abs(big).max() > 0 and np.abs(small).max() > 0
    both_entry_points(wl.TINY_VIT, 64, 192, seed=23)                    # another element type and table shape, same array


def test_static_scratch_entry_point_rejects_shapes_beyond_its_array():
    import torch
    from paper_2505_19342_amd import binding as B
    # one KV head with eight query heads of 256 channels and two long caches: 1024 chunks x 8 heads x 258 floats of
    # partial results = 8.06 MiB, a shape the workspace entry point accepts
    desc = B.DecodeDesc(B.vq_desc("bf16", 256, 8, 256), 8, 1, 256, 65536, 65536, 0.0)
    assert B.astra_decode_attention_workspace_bytes(desc) > B.astra_decode_attention_static_max_bytes()
    t = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(B.AstraError, match="workspace"):
        B.astra_decode_attention_static(desc, t, t, t, t, t, None, t, t, t, None)
