"""The C-ABI library loads and exports every function include/astra.h declares (no GPU needed), and
the Python descriptors mirror the C structs."""
import ctypes
import os
import re

from paper_2505_19342_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "astra.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(astra_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = declared_functions()
    assert set(B.EXPORTS) == set(names)
    for n in names:
        assert getattr(lib, n) is not None


def test_loading_first_still_puts_torchs_hip_runtime_in_the_process():
    # a library opened before torch would bind to another HIP runtime than the one torch's streams belong to
    import subprocess
    import sys
    code = "from paper_2505_19342_amd import binding as B; import sys; assert 'torch' not in sys.modules; B.load(False); assert 'torch' in sys.modules"
    subprocess.run([sys.executable, "-c", code], cwd=ROOT, check=True, timeout=300)


def test_version_and_status_strings_run_without_a_gpu():
    lib = B.load()
    assert lib.astra_version() >= 100
    assert lib.astra_status_string(0) == b"ok"
    assert b"workspace" in lib.astra_status_string(-4)


def test_descriptor_layouts():
    assert ctypes.sizeof(B.VqDesc) == 20
    assert ctypes.sizeof(B.AttnDesc) == 40
    assert ctypes.sizeof(B.LayerDesc) == 60
    assert B.AttnDesc.scale.offset == 36


def test_host_side_argument_checks_need_no_gpu():
    lib = B.load()
    bad = B.LayerDesc(B.VqDesc(B.ASTRA_BF16, B.ASTRA_CODE_U8, 768, 5, 256),        # 5 does not divide 768
                      B.attn_desc("bf16", 12, 12, 64, 0, 256, 768, False))
    assert lib.astra_layer_workspace_bytes(ctypes.byref(bad)) == 0
    good = B.LayerDesc(B.vq_desc("bf16", 768, 16, 256), B.attn_desc("bf16", 12, 12, 64, 1, 256, 768, False))
    need = lib.astra_layer_workspace_bytes(ctypes.byref(good))
    # Q, O: 257 x 768; K, V: 257 x 768; K-hat, V-hat: 768 x 768, bf16, each rounded up to 256 bytes
    assert need >= 2 * (4 * 257 * 768 + 2 * 768 * 768)
    # NULL descriptor and NULL data pointers are reported, not dereferenced
    assert lib.astra_vq_prepare(None, None, None, None) == -1
    assert lib.astra_vq_encode(ctypes.byref(good.vq), None, 5, None, None, None, None) == -1
    assert lib.astra_vq_encode(ctypes.byref(good.vq), None, 0, None, None, None, None) == 0
    assert lib.astra_vq_encode(ctypes.byref(good.vq), None, -1, None, None, None, None) == -2
    # the measurement probes check their arguments before anything is launched
    assert lib.astra_probe_mfma_bf16(None, 1, 1, None) == -1


def test_encode_fusion_plan_is_host_only():
    """astra_layer_encode_fused decides from the shapes alone: the projection launch carries the encode when
    its tiles leave compute units idle in the last round (Llama-3-8B shape: 192 tiles of 128x256 on the first
    rank, 160 and 192 tiles of 256x256 on the last two; the second rank's 256 tiles of 128x256 fill the chip),
    never for fp32; an invalid descriptor is an error, not a crash."""
    from paper_2505_19342_amd import workloads as wl

    def desc(cfg, rank):
        tn = (cfg.n_dev - 1) * cfg.n_local
        return B.LayerDesc(B.vq_desc(cfg.dtype, cfg.d_model, cfg.n_groups, cfg.codebook_size),
                           B.attn_desc(cfg.dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n_cls, cfg.n_local, tn,
                                       cfg.causal, rank * cfg.n_local))

    llama = wl.CONFIGS["llama3_8b_bf16"]
    assert [B.astra_layer_encode_fused(desc(llama, r)) for r in range(llama.n_dev)] == [True, False, True, True]
    # the small bf16 shapes run their projections as a single partial round of 128x128 tiles: the idle units take the encode too
    for name, want in (("tiny_vit_f32", False), ("vit_base_bf16", True), ("gpt2_small_bf16", True)):
        cfg = wl.CONFIGS[name]
        assert B.astra_layer_encode_fused(desc(cfg, cfg.n_dev - 1)) == want
    bad = desc(llama, 3)
    bad.vq.n_groups = 7          # 4096 is not a multiple of 7
    assert B.load().astra_layer_encode_fused(ctypes.byref(bad)) < 0


def test_block_kv_and_decode_planning_is_host_only():
    """Workspace sizes and argument checks of the entry points around the layer are decided on the host: the sizes
    cover the buffers the calls need, invalid descriptors give 0 / an error code, NULL pointers are reported."""
    lib = B.load()
    assert ctypes.sizeof(B.BlockDesc) == 80 and ctypes.sizeof(B.LayerKvDesc) == 64 and ctypes.sizeof(B.DecodeDesc) == 44
    assert ctypes.sizeof(B.BlockWeights) == 18 * ctypes.sizeof(ctypes.c_void_p)
    layer = B.LayerDesc(B.vq_desc("bf16", 4096, 64, 1024), B.attn_desc("bf16", 32, 8, 128, 0, 1024, 3072, True, 3072))
    blk = B.block_desc(layer, "rmsnorm", "swiglu", 14336, 1e-5)
    need = B.astra_block_workspace_bytes(blk)
    lay = B.astra_layer_workspace_bytes(layer)
    # layer workspace + normalised rows + hidden rows + four fp32 slices of the split second MLP product
    assert need >= lay + 1024 * 4096 * 2 + 1024 * 14336 * 2 + 4 * 1024 * 4096 * 4
    assert B.astra_block_workspace_bytes(B.block_desc(layer, "rmsnorm", "swiglu", 14336 + 8, 1e-5)) == 0      # d_ff % 64 for bf16
    assert B.astra_block_workspace_bytes(B.block_desc(layer, "rmsnorm", "swiglu", 0, 1e-5)) == 0
    bad = B.block_desc(layer, "rmsnorm", "swiglu", 14336, 1e-5)
    bad.norm_kind = 5
    assert B.astra_block_workspace_bytes(bad) == 0
    assert lib.astra_block_forward(ctypes.byref(blk), None, None, None, None, None, None, None, None, 0, None) == -1
    assert lib.astra_stack_forward(ctypes.byref(blk), -1, None, None, None, None, None, None, None, 0, None) == -2
    assert lib.astra_stack_forward(ctypes.byref(blk), 0, None, None, None, None, None, None, None, 0, None) == 0
    assert lib.astra_stack_forward(ctypes.byref(blk), 2, None, None, None, None, None, None, None, 0, None) == -1

    kv = B.LayerKvDesc(B.vq_desc("bf16", 1024, 32, 1024), layer.attn, 4096)
    need = B.astra_layer_kv_workspace_bytes(kv)
    # Q, O: 1024 x 4096; K, V, V^T: 1024 x 1024; K-hat, V-hat^T: 3072 x 1024 (bf16)
    assert need >= 2 * (2 * 1024 * 4096 + 3 * 1024 * 1024 + 2 * 3072 * 1024)
    kv.vq.d_model = 4096                        # the codebooks must span H_kv * dh
    assert B.astra_layer_kv_workspace_bytes(kv) == 0

    dec = B.DecodeDesc(B.vq_desc("bf16", 1024, 32, 1024), 32, 8, 128, 1025, 3072, 0.0)
    need = B.astra_decode_attention_workspace_bytes(dec)
    assert need >= 32 * 4 * 1024 * 4            # the table: 32 query heads x 4 groups per head x 1024 entries, fp32
    assert lib.astra_decode_attention(ctypes.byref(dec), None, None, None, None, None, None, None, None, None, None, None, 0, None) == -1
    for field, value in (("n_q_heads", 12), ("head_dim", 100), ("n_local", -1)):      # 12 % 8; 8 * 100 != 1024; negative
        d = B.DecodeDesc(B.vq_desc("bf16", 1024, 32, 1024), 32, 8, 128, 1025, 3072, 0.0)
        setattr(d, field, value)
        assert B.astra_decode_attention_workspace_bytes(d) == 0
    three = B.DecodeDesc(B.vq_desc("bf16", 1024, 32, 1024), 24, 8, 128, 10, 10, 0.0)  # 3 query heads per KV head: no kernel
    assert B.astra_decode_attention_workspace_bytes(three) == 0
    empty = B.DecodeDesc(B.vq_desc("bf16", 1024, 32, 1024), 32, 8, 128, 0, 0, 0.0)
    assert B.astra_decode_attention_workspace_bytes(empty) > 0
