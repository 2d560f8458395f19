"""GPU parity: one device's share of an L-block model through astra_stack_forward.  The CPU oracle simulates the
whole multi-device procedure of Sec. 3.1 (every device normalises and quantises its chunk, codes are exchanged,
every device runs its block, L times); the GPU gets one device's chunk and, per block, the codes that device
received in the simulation, and must reproduce that device's final stream.  Bars: the per-block bars of
tests/test_gpu_block.py added up over the blocks (fp32 1e-4 per block; bf16 2e-2 + 2^-6 rms of the block's update,
per block); block 0's codes under the near-tie rule; the stack call bit-identical (stream and every block's codes)
to the same blocks called one by one.  Codes of later blocks are outputs of streams that differ by rounding between
the two sides; they are covered by that bit-identity and the per-block parity tests."""
import numpy as np
import pytest

import oracle
from paper_2505_19342_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_stack(bcfg, n_layers, rank):
    from gpu_util import StackOnGpu
    cfg = bcfg.layer
    data = wl.generate_stack(bcfg, n_layers)
    sim = oracle.model_forward(data["x"], data["layers"], n_dev=cfg.n_dev, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
                               norm_kind=bcfg.norm_kind, eps=bcfg.eps, mlp_kind=bcfg.mlp_kind, causal=cfg.causal,
                               cls=data.get("cls"), h_is_bf16=cfg.dtype == "bf16")
    view = wl.device_view(cfg, data, rank)
    received = [sim["codes_nonlocal"][l][rank] for l in range(n_layers)]
    st = StackOnGpu(bcfg, data["layers"], view["x_local"], received, view["n_before"])
    st.run()
    out, codes = st.results()
    ref = sim["x"][rank]
    err = np.abs(out - ref).max()
    upd = float(np.sqrt(np.mean((ref - view["x_local"]) ** 2)))
    tol = n_layers * 1e-4 if cfg.dtype == "f32" else n_layers * 2e-2 + 2.0 ** -6 * upd * np.sqrt(n_layers)
    print(f"{bcfg.name} x{n_layers} rank {rank}: max abs err {err:.3e} (bar {tol:.3e}; |x| max {np.abs(ref).max():.2f}, rms update {upd:.3f})")
    assert err <= tol
    # block 0 quantises the same input on both sides
    d0 = codes[0] != sim["codes"][0][rank]
    assert d0.mean() <= 2e-3, f"{int(d0.sum())} of {d0.size} block-0 codes differ"
    # the stack call is the same launches as the blocks one by one
    st2 = StackOnGpu(bcfg, data["layers"], view["x_local"], received, view["n_before"])
    st2.run_block_by_block()
    out2, codes2 = st2.results()
    np.testing.assert_array_equal(out, out2)
    for a, b in zip(codes, codes2):
        np.testing.assert_array_equal(a, b)
    if cfg.n_cls:
        # the distributed class token: this device's replica is row 0; the pooled token is the mean over devices (Sec. 3.3)
        assert np.abs(out[0] - sim["x"][rank][0]).max() <= tol
    return err


@pytest.mark.parametrize("rank", [0, 2])
def test_tiny_vit_f32_three_blocks(rank):
    run_stack(wl.TINY_VIT_BLOCK, 3, rank)


def test_vit_base_bf16_two_blocks_with_class_row():
    run_stack(wl.VIT_BASE_BLOCK, 2, 1)


@pytest.mark.parametrize("rank", [0, 3])
def test_gpt2_small_bf16_two_blocks_causal(rank):
    run_stack(wl.GPT2_SMALL_BLOCK, 2, rank)


def test_stack_argument_errors_launch_nothing():
    import torch
    from gpu_util import StackOnGpu
    from paper_2505_19342_amd import binding as B
    bcfg = wl.TINY_VIT_BLOCK
    cfg = bcfg.layer
    data = wl.generate_stack(bcfg, 2)
    view = wl.device_view(cfg, data, 0)
    rng = np.random.default_rng(0)
    codes = [rng.integers(0, cfg.codebook_size, (cfg.n_nonlocal, cfg.n_groups)) for _ in range(2)]
    st = StackOnGpu(bcfg, data["layers"], view["x_local"], codes, view["n_before"])
    st.x_out.fill_(-3.0)
    # the second block lacks a matrix: nothing may run, not even the first block
    w_bad = B.block_weights(**{k: v for k, v in st.blocks[1].tensors.items() if k != "w1"})
    with pytest.raises(B.AstraError, match="NULL"):
        B.astra_stack_forward(st.desc, [st.blocks[0].weights, w_bad], st.x, [b.codes_nonlocal for b in st.blocks], None, st.x_out,
                              [b.codes_local for b in st.blocks], st.workspace)
    torch.cuda.synchronize()
    assert bool((st.x_out == -3.0).all())
    with pytest.raises(B.AstraError):
        B.astra_stack_forward(st.desc, [st.blocks[0].weights], st.x, [b.codes_nonlocal for b in st.blocks], None, st.x_out,
                              [b.codes_local for b in st.blocks], st.workspace)
