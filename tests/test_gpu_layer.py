"""GPU parity: the whole per-device layer (encode + decode + projections + mixed-precision attention +
output projection) through astra_layer_forward against the CPU oracle, on the seeded workloads.
Bars: codes bit-exact except counted near-ties (oracle gap < 1e-5 relative); layer output max-abs
<= 1e-4 (fp32) / 2e-2 (bf16)."""
import dataclasses

import numpy as np
import pytest

import oracle
from paper_2505_19342_amd import workloads as wl

pytestmark = pytest.mark.gpu

Y_TOL = {"f32": 1e-4, "bf16": 2e-2}
NEAR_TIE = 1e-5


def run_case(cfg, rank, biases=False):
    from gpu_util import LayerOnGpu, compare_codes
    data = wl.generate(cfg)
    view = wl.device_view(cfg, data, rank)
    codes_nl = oracle.vq_encode(view["x_nonlocal"], data["codebook"])       # what the peers would have sent
    b = None
    if biases:
        rng = np.random.default_rng(99)
        dq, dkv = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
        b = [(0.1 * rng.standard_normal(n)).astype(np.float32) for n in (dq, dkv, dkv, cfg.d_model)]
        if cfg.dtype == "bf16":
            b = [wl.round_to_bf16(v) for v in b]
    kw = {} if b is None else dict(bq=b[0], bk=b[1], bv=b[2], bo=b[3])
    y_ref, codes_ref, gap = oracle.layer_forward(
        view["x_local"], codes_nl, data["codebook"], data["wq"], data["wk"], data["wv"], data["wo"],
        n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, n_cls=cfg.n_cls, causal=cfg.causal,
        n_before=view["n_before"], return_gap=True, **kw)
    layer = LayerOnGpu(cfg, data, view["x_local"], codes_nl, view["n_before"], biases=b)
    layer.run()
    y, codes = layer.results()
    n_tie = compare_codes(codes, codes_ref, gap, NEAR_TIE)
    err = np.abs(y - y_ref).max()
    print(f"{cfg.name} rank {rank}: max abs err {err:.3e} (|y| max {np.abs(y_ref).max():.3f}), near-tie codes {n_tie}/{codes.size}")
    assert err <= Y_TOL[cfg.dtype]
    assert n_tie <= max(2, codes.size // 2000)
    return err


@pytest.mark.parametrize("rank", [0, 1, 3])
def test_tiny_vit_f32(rank):
    run_case(wl.TINY_VIT, rank)


@pytest.mark.parametrize("rank", [0, 3])
def test_vit_base_bf16_with_class_row(rank):
    run_case(wl.VIT_BASE, rank)


@pytest.mark.parametrize("rank", [0, 2, 3])
def test_gpt2_small_bf16_causal(rank):
    run_case(wl.GPT2_SMALL, rank)


def test_biases_f32_and_bf16():
    run_case(wl.TINY_VIT, 1, biases=True)
    run_case(wl.VIT_BASE, 1, biases=True)


def test_f32_launches_of_large_and_small_tiles():
    """The fp32 product runs on 64 x 64 tiles once a launch has 128 of them and on 32 x 32 tiles below (the tiny shape): a
    longer sequence with ragged rows takes the large ones for the projections and, with two heads of 96, output values
    beyond the first 64 lanes in the attention."""
    cfg = dataclasses.replace(wl.TINY_VIT, name="f32_long", seq_len=1500, n_q_heads=2, n_kv_heads=2, head_dim=96, seed=17)
    run_case(cfg, 1, biases=True)


@pytest.mark.parametrize("i_dev", [0, 1, 2])
@pytest.mark.parametrize("i_k", [0, 1, 2])
@pytest.mark.parametrize("i_g", [0, 1, 2, 3])
def test_sweep_points(i_g, i_k, i_dev):
    """Every point of the sweep on the ViT-Base shape: G in {1, 4, 16, 64} x K in {16, 256, 1024} x {2, 4, 8} devices
    (group widths 768, 192, 48 and 12: the last is not a multiple of the 16-byte operand piece, so the peers' rows are
    rebuilt by the decode kernel instead of inside the projection's operand loader)."""
    cfg = wl.sweep_config(i_g, i_k, i_dev)
    run_case(cfg, cfg.n_dev - 1 if i_g == i_k else 1)


def test_uneven_split_and_ragged_shapes():
    # a device holding 100 of 420 tokens: nothing in the ABI assumes an even split
    from gpu_util import LayerOnGpu, compare_codes
    cfg = dataclasses.replace(wl.GPT2_SMALL, name="uneven", seq_len=420, seed=77)
    data = wl.generate(cfg)
    lo, hi = 130, 230
    x_local = data["x"][lo:hi]
    x_nl = np.concatenate([data["x"][:lo], data["x"][hi:]])
    codes_nl = oracle.vq_encode(x_nl, data["codebook"])
    y_ref, codes_ref, gap = oracle.layer_forward(x_local, codes_nl, data["codebook"], data["wq"], data["wk"], data["wv"],
                                                 data["wo"], n_q_heads=12, n_kv_heads=12, causal=True, n_before=lo,
                                                 return_gap=True)
    layer = LayerOnGpu(cfg, data, x_local, codes_nl, lo)
    layer.run()
    y, codes = layer.results()
    compare_codes(codes, codes_ref, gap, NEAR_TIE)
    assert np.abs(y - y_ref).max() <= Y_TOL["bf16"]


@pytest.mark.parametrize("rank", [3, 0])
def test_llama3_8b_shape_full_size(rank):
    """The benchmark workload at full size, same launch configuration as bench.py times."""
    run_case(wl.LLAMA3_8B, rank)


@pytest.mark.parametrize("seq_len,lo,fused", [(3917, 2917, True), (1000, 0, True), (1900, 900, False), (5100, 3070, False)])
def test_llama_dims_ragged_rows_in_every_projection_tile_shape(seq_len, lo, fused):
    """Llama-3-8B widths with row counts that are multiples of nothing: the last seq_len - lo tokens on this device,
    so the last tile of every projection and the last token block of the encode are ragged.  The cases take the
    launch shapes of the projections: 256x256 tiles with the encode on the units left over (the configuration
    bench.py times), 192 tiles of 128x256 with the encode on the units left over (no visible peers), 256 tiles of
    128x256 that fill the chip (the encode then runs as a kernel of its own), and 288 tiles of 256x256, which are dealt
    into two launches (one of 256x256 tiles that fills its round, one on 128x128 tiles)."""
    from gpu_util import LayerOnGpu, compare_codes
    from paper_2505_19342_amd import binding as B
    cfg = dataclasses.replace(wl.LLAMA3_8B, name="llama_ragged", seq_len=seq_len, seed=41)
    data = wl.generate(cfg)
    x_local, x_nl = data["x"][lo:], data["x"][:lo]
    codes_nl = oracle.vq_encode(x_nl, data["codebook"])
    y_ref, codes_ref, gap = oracle.layer_forward(x_local, codes_nl, data["codebook"], data["wq"], data["wk"], data["wv"],
                                                 data["wo"], n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, causal=True,
                                                 n_before=lo, return_gap=True)
    layer = LayerOnGpu(cfg, data, x_local, codes_nl, lo)
    assert B.astra_layer_encode_fused(layer.desc) == fused
    layer.run()
    y, codes = layer.results()
    n_tie = compare_codes(codes, codes_ref, gap, NEAR_TIE)
    err = np.abs(y - y_ref).max()
    print(f"llama dims, {seq_len - lo} local / {lo} non-local rows: max abs err {err:.3e}, near-tie codes {n_tie}/{codes.size}")
    assert err <= Y_TOL["bf16"]
    assert n_tie <= max(2, codes.size // 2000)


def test_fused_encode_equals_the_standalone_encode_and_calls_repeat_bit_exactly():
    """The encode inside the projection launch and astra_vq_encode run the same arithmetic in the same order: equal codes,
    bit for bit.  Two calls of the layer, and the call with stage events, give identical bits too."""
    import torch
    from gpu_util import LayerOnGpu, empty_codes
    from paper_2505_19342_amd import binding as B
    cfg = wl.LLAMA3_8B
    data = wl.generate(cfg)
    view = wl.device_view(cfg, data, 2)
    codes_nl = oracle.vq_encode(view["x_nonlocal"], data["codebook"])
    layer = LayerOnGpu(cfg, data, view["x_local"], codes_nl, view["n_before"])
    assert B.astra_layer_encode_fused(layer.desc)
    layer.run()
    torch.cuda.synchronize()
    y1, c1 = layer.y.clone(), layer.codes_local.clone()
    alone = empty_codes(cfg.n_local, cfg.n_groups, cfg.codebook_size)
    B.astra_vq_encode(layer.desc.vq, layer.x_local, cfg.n_local, layer.codebook, layer.cnorm, alone)
    torch.cuda.synchronize()
    assert torch.equal(alone, c1)
    layer.y.zero_()
    layer.codes_local.zero_()
    layer.run()
    torch.cuda.synchronize()
    assert torch.equal(layer.y, y1) and torch.equal(layer.codes_local, c1)
    layer.y.zero_()
    layer.codes_local.zero_()
    ev = B.HipEvents(7)
    B.astra_layer_forward_profiled(layer.desc, layer.x_local, layer.codes_nonlocal, layer.codebook, layer.cnorm, *layer.w,
                                   *layer.b, layer.y, layer.codes_local, layer.workspace, ev.handles)
    torch.cuda.synchronize()
    assert torch.equal(layer.y, y1) and torch.equal(layer.codes_local, c1)
    assert ev.elapsed_ms(0, 4) > 0


def test_workspace_too_small_is_an_error():
    import torch
    from gpu_util import DEV, LayerOnGpu
    from paper_2505_19342_amd import binding as B
    cfg = wl.TINY_VIT
    data = wl.generate(cfg)
    view = wl.device_view(cfg, data, 0)
    layer = LayerOnGpu(cfg, data, view["x_local"], np.zeros((cfg.n_nonlocal, cfg.n_groups), np.int32), 0)
    layer.workspace = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.AstraError):
        layer.run()
