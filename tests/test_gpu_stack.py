"""GPU parity: one device's share of an L-block model through astra_stack_forward.  The CPU oracle simulates the
whole multi-device procedure of Sec. 3.1 (every device normalises and quantises its chunk, codes are exchanged,
every device runs its block, L times); the GPU gets one device's chunk and, per block, the codes that device
received in the simulation, and must reproduce that device's final stream.  Bars: the per-block bars of
tests/test_gpu_block.py added up over the blocks (fp32 1e-4 per block; bf16 2e-2 + 2^-6 rms of the block's update,
per block: block l+1 starts from a stream that already differs by block l's rounding, and a pre-norm residual block
passes such a difference on about unchanged, so the bars of the blocks add; the observed error is printed and stays
several times below).  Block 0 quantises the same input on both sides: its codes are held to the block test's rule
(bit-exact where the normalised rows agree, except near-ties with an oracle gap below 1e-5 relative; on the few group
slices whose bf16 rounding of h falls on the other side of a boundary, a codeword that the differing slice justifies).
The stack call must be bit-identical (stream and every block's codes) to the same blocks called one by one.  Codes of
later blocks are outputs of streams that differ by rounding between the two sides; they are covered by that
bit-identity and the per-block parity tests."""
import dataclasses

import numpy as np
import pytest

import oracle
from paper_2505_19342_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_stack(bcfg, n_layers, rank):
    from gpu_util import BlockOnGpu, StackOnGpu, check_h_and_codes
    cfg = bcfg.layer
    data = wl.generate_stack(bcfg, n_layers)
    sim = oracle.model_forward(data["x"], data["layers"], n_dev=cfg.n_dev, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
                               norm_kind=bcfg.norm_kind, eps=bcfg.eps, mlp_kind=bcfg.mlp_kind, causal=cfg.causal,
                               cls=data.get("cls"), h_is_bf16=cfg.dtype == "bf16", rope_base=bcfg.rope_base)
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
    # block 0 quantises the same input on both sides: the block test's rule for h and the codes
    p0 = data["layers"][0]
    names = ("bq", "bk", "bv", "bo", "b1", "b2")
    _, codes_ref, gap, h_ref = oracle.block_forward(
        view["x_local"], received[0], p0["codebook"], p0["wq"], p0["wk"], p0["wv"], p0["wo"], norm_kind=bcfg.norm_kind,
        eps=bcfg.eps, g1=p0["g1"], g2=p0["g2"], be1=p0.get("be1"), be2=p0.get("be2"), mlp_kind=bcfg.mlp_kind, w1=p0["w1"],
        w2=p0["w2"], n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, n_cls=cfg.n_cls, causal=cfg.causal,
        n_before=view["n_before"], h_is_bf16=cfg.dtype == "bf16", rope_base=bcfg.rope_base, **{n: p0.get(n) for n in names})
    np.testing.assert_array_equal(codes_ref, sim["codes"][0][rank])
    b0 = BlockOnGpu(bcfg, p0, view["x_local"], received[0], view["n_before"])
    b0.run()
    _, codes_b0, h = b0.results()
    np.testing.assert_array_equal(codes_b0, codes[0])          # the stack's first block is this block call
    n_tie, n_slices, n_other = check_h_and_codes(cfg.dtype, cfg.n_cls, h, h_ref, codes[0], codes_ref, gap, p0["codebook"])
    print(f"  block-0 codes: {n_tie}/{codes[0].size} near-ties, {n_slices} slices with a differing h ({n_other} chose another codeword)")
    assert n_tie <= max(2, codes[0].size // 2000)
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


def test_llama_width_four_blocks_rmsnorm_swiglu_grouped_query_heads():
    """Llama-3-8B widths (D 4096, 32 / 8 heads of 128, G 64, K 1024, 16-bit codes, RMSNorm, SwiGLU) with 287 local rows
    and a narrower MLP, four blocks deep, on a middle rank of the causal split."""
    layer = dataclasses.replace(wl.LLAMA3_8B, name="llama_stack", seq_len=1148, seed=61)
    run_stack(dataclasses.replace(wl.LLAMA3_8B_BLOCK, name="llama_stack_block", layer=layer, d_ff=1792), 4, 2)


def test_llama_width_three_blocks_with_rotary_positions():
    """The same widths with rotary positions inside every layer (optional, outside the paper), last rank of the causal split."""
    layer = dataclasses.replace(wl.LLAMA3_8B, name="llama_rope_stack", seq_len=1148, seed=62)
    run_stack(dataclasses.replace(wl.LLAMA3_8B_BLOCK, name="llama_rope_stack_block", layer=layer, d_ff=1792, rope_base=500000.0), 3, 3)


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
