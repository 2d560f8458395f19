"""Seeded synthetic inputs for the Astra attention-layer workloads.

This module only draws random numbers and arranges them; it performs none of
the method's arithmetic (no distance, no projection, no softmax).  Both the
tests (which hand the same arrays to the CPU checker and to the HIP library)
and the benchmark use it.  It needs numpy only.

The workloads stand in for the paper's ViT-Base, GPT2 and Llama-3-8B
experiments (Sec. 4.1), whose data, weights and learned codebooks are not
available: shapes follow those models, values follow the stated
distributions.  Everything is generated in fp32; for bf16 workloads every
tensor is then rounded to the nearest bf16 (ties to even) so that the bits
given to every consumer are identical.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    name: str
    dtype: str            # "f32" | "bf16"
    d_model: int          # D
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int          # N content tokens over all simulated devices
    n_dev: int
    n_groups: int         # G
    codebook_size: int    # K
    n_cls: int = 0        # one full-precision class-token replica per device
    causal: bool = False
    seed: int = 0
    dist: str = "normal"  # "normal" | "normal_shift" | "student_t5" | "rms_normal"

    @property
    def n_local(self) -> int:
        return self.seq_len // self.n_dev

    @property
    def n_nonlocal(self) -> int:
        return self.seq_len - self.n_local

    @property
    def group_dim(self) -> int:
        return self.d_model // self.n_groups

    @property
    def code_dtype(self):
        return np.uint8 if self.codebook_size <= 256 else np.uint16


TINY_VIT = LayerConfig("tiny_vit_f32", "f32", 192, 3, 3, 64, 256, 4, 4, 256, seed=0, dist="normal")
VIT_BASE = LayerConfig("vit_base_bf16", "bf16", 768, 12, 12, 64, 1024, 4, 16, 256, n_cls=1, seed=1,
                       dist="normal_shift")
GPT2_SMALL = LayerConfig("gpt2_small_bf16", "bf16", 768, 12, 12, 64, 1024, 4, 32, 256, causal=True, seed=2,
                         dist="student_t5")
LLAMA3_8B = LayerConfig("llama3_8b_bf16", "bf16", 4096, 32, 8, 128, 4096, 4, 64, 1024, causal=True, seed=4,
                        dist="rms_normal")

CONFIGS = {c.name: c for c in (TINY_VIT, VIT_BASE, GPT2_SMALL, LLAMA3_8B)}

SWEEP_GROUPS = (1, 4, 16, 64)
SWEEP_CODEBOOK_SIZES = (16, 256, 1024)
SWEEP_DEVICES = (2, 4, 8)


def sweep_config(i_g: int, i_k: int, i_dev: int) -> LayerConfig:
    """One point of the ViT-Base-shaped G x K x devices sweep (no class row)."""
    g, k, n = SWEEP_GROUPS[i_g], SWEEP_CODEBOOK_SIZES[i_k], SWEEP_DEVICES[i_dev]
    return replace(VIT_BASE, name=f"sweep_G{g}_K{k}_dev{n}", n_groups=g, codebook_size=k, n_dev=n,
                   n_cls=0, seed=1000 + 100 * i_g + 10 * i_k + i_dev)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Nearest-even rounding of fp32 values to bf16, returned widened back to fp32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16-representable fp32 values."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _embeddings(rng, n, d, dist):
    if dist == "normal":
        return rng.standard_normal((n, d), dtype=np.float32)
    if dist == "normal_shift":      # per-token scalar mean shift, std 0.1
        x = rng.standard_normal((n, d), dtype=np.float32)
        return x + (0.1 * rng.standard_normal((n, 1))).astype(np.float32)
    if dist == "student_t5":        # heavy tails, scaled to unit variance (Var t_5 = 5/3)
        return (rng.standard_t(5, size=(n, d)) * np.sqrt(3.0 / 5.0)).astype(np.float32)
    if dist == "rms_normal":        # rows divided by their root mean square, no gain
        x = rng.standard_normal((n, d), dtype=np.float32)
        return x / np.sqrt(np.mean(x.astype(np.float64) ** 2, axis=1, keepdims=True)).astype(np.float32)
    raise ValueError(dist)


def generate(cfg: LayerConfig) -> dict:
    """All tensors of one layer call, in the paper's orientation (``Q = X W_q``,
    so ``wq`` is ``[D, H_q*dh]``).  Keys: x [N, D], cls [n_dev, D] (if n_cls),
    codebook [G, K, dg], wq, wk, wv, wo."""
    rng = np.random.default_rng(cfg.seed)
    d, dq, dkv = cfg.d_model, cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    out = {"x": _embeddings(rng, cfg.seq_len, d, cfg.dist)}
    if cfg.n_cls:
        out["cls"] = rng.standard_normal((cfg.n_dev, d), dtype=np.float32)
    out["codebook"] = rng.standard_normal((cfg.n_groups, cfg.codebook_size, cfg.group_dim), dtype=np.float32)
    for name, shape in (("wq", (d, dq)), ("wk", (d, dkv)), ("wv", (d, dkv)), ("wo", (dq, d))):
        out[name] = (0.02 * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
    if cfg.dtype == "bf16":
        out = {k: round_to_bf16(v) for k, v in out.items()}
    return out


def device_view(cfg: LayerConfig, data: dict, rank: int) -> dict:
    """What simulated device ``rank`` holds: its contiguous chunk (class row
    first when there is one) and, in global-position order, the full-precision
    embeddings of the other devices' tokens (the caller encodes these to obtain
    the codes that would have been received).  ``n_before`` is the number of
    non-local tokens that precede the local chunk."""
    tl = cfg.n_local
    lo, hi = rank * tl, (rank + 1) * tl
    x = data["x"]
    x_local = x[lo:hi]
    if cfg.n_cls:
        x_local = np.concatenate([data["cls"][rank:rank + 1], x_local], axis=0)
    x_nonlocal = np.concatenate([x[:lo], x[hi:]], axis=0)
    return {"x_local": np.ascontiguousarray(x_local), "x_nonlocal": np.ascontiguousarray(x_nonlocal),
            "n_before": lo, "rank": rank}


# ---- whole blocks (Sec. 3.1: the layer inside the stock pre-norm block of each model) ------------------------
@dataclass(frozen=True)
class BlockConfig:
    name: str
    layer: LayerConfig
    norm_kind: str        # "layernorm" | "rmsnorm"
    mlp_kind: str         # "gelu_tanh" | "gelu_erf" | "swiglu"
    d_ff: int
    eps: float
    biases: bool          # linear layers carry biases (ViT, GPT-2) or not (Llama)
    rope_base: float = 0.0  # > 0: rotary positions inside the layer (optional, causal layers; the paper names no positional encoding)


TINY_VIT_BLOCK = BlockConfig("tiny_vit_block_f32", TINY_VIT, "layernorm", "gelu_erf", 768, 1e-6, True)
VIT_BASE_BLOCK = BlockConfig("vit_base_block_bf16", VIT_BASE, "layernorm", "gelu_erf", 3072, 1e-6, True)
GPT2_SMALL_BLOCK = BlockConfig("gpt2_small_block_bf16", GPT2_SMALL, "layernorm", "gelu_tanh", 3072, 1e-5, True)
LLAMA3_8B_BLOCK = BlockConfig("llama3_8b_block_bf16", LLAMA3_8B, "rmsnorm", "swiglu", 14336, 1e-5, False)
BLOCK_CONFIGS = {c.name: c for c in (TINY_VIT_BLOCK, VIT_BASE_BLOCK, GPT2_SMALL_BLOCK, LLAMA3_8B_BLOCK)}


def generate_block(bcfg: BlockConfig) -> dict:
    """Tensors of one block call.  Everything generate() gives for the layer (codebook, wq..wo; its "x" and "cls"
    become the fp32 residual stream after a rescale and a per-channel offset, and are NOT rounded: the stream is fp32
    for both element types), plus norm parameters (fp32), MLP weights w1 [D, d_ff] or [D, 2 d_ff] (gate | up) and
    w2 [d_ff, D] in the paper's orientation, and biases when the model has them."""
    cfg = bcfg.layer
    out = generate(cfg)
    rng = np.random.default_rng(cfg.seed + 7919)
    d, f = cfg.d_model, bcfg.d_ff
    offset = (0.3 * rng.standard_normal(d)).astype(np.float32)
    stream_rng = np.random.default_rng(cfg.seed)            # the same draws as generate(), kept unrounded
    out["x"] = (1.7 * _embeddings(stream_rng, cfg.seq_len, d, cfg.dist) + offset).astype(np.float32)
    if cfg.n_cls:
        out["cls"] = (1.7 * stream_rng.standard_normal((cfg.n_dev, d), dtype=np.float32) + offset).astype(np.float32)
    for name in ("g1", "g2"):
        out[name] = (1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32)
    for name in ("be1", "be2"):
        out[name] = (0.1 * rng.standard_normal(d)).astype(np.float32)
    n1 = 2 * f if bcfg.mlp_kind == "swiglu" else f
    mats = {"w1": (0.02 * rng.standard_normal((d, n1), dtype=np.float32)).astype(np.float32),
            "w2": (0.02 * rng.standard_normal((f, d), dtype=np.float32)).astype(np.float32)}
    if bcfg.biases:
        dq, dkv = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
        for name, n in (("bq", dq), ("bk", dkv), ("bv", dkv), ("bo", d), ("b1", n1), ("b2", d)):
            mats[name] = (0.1 * rng.standard_normal(n)).astype(np.float32)
    if cfg.dtype == "bf16":
        mats = {k: round_to_bf16(v) for k, v in mats.items()}
    out.update(mats)
    return out


def generate_stack(bcfg: BlockConfig, n_layers: int) -> dict:
    """Tensors of n_layers blocks: {"x": [N, D] fp32 stream entering block 0, "cls": [n_dev, D] (if n_cls),
    "layers": list of per-block dicts as generate_block() gives them (without x / cls), block l drawn with seed
    layer.seed + 1000 * l}."""
    first = generate_block(bcfg)
    out = {"x": first.pop("x"), "layers": [first]}
    if "cls" in first:
        out["cls"] = first.pop("cls")
    for l in range(1, n_layers):
        p = generate_block(replace(bcfg, layer=replace(bcfg.layer, seed=bcfg.layer.seed + 1000 * l)))
        p.pop("x")
        p.pop("cls", None)
        out["layers"].append(p)
    return out


# ---- the variant that quantises K and V after projection (App. memory cost: C = 2 codebooks of dimension H_kv * dh) ----
KV_GROUPS = {"tiny_vit_f32": 4, "vit_base_bf16": 16, "gpt2_small_bf16": 32, "llama3_8b_bf16": 32}


def generate_kv(cfg: LayerConfig, n_groups_kv: int | None = None) -> dict:
    """generate(cfg) plus the two codebooks of the KV-space variant, codebook_k and codebook_v [G_kv, K, dkv / G_kv]
    ~ N(0, 1.3^2) (the scale of K = X W_k for unit-variance rows and N(0, 0.02^2) weights at D = 4096); the X-space
    codebook of generate() stays in the dict but is not used by that variant.  Llama: G_kv = 32, K = 1024, i.e.
    2 * 32 * 10 = 640 bits per token PER BLOCK (20 480 over the 32 blocks: the G = 32 row of the paper's Llama table; the
    640 that table prints for G = 1 is 32 blocks x 2 codebooks x 10 bits)."""
    out = generate(cfg)
    g = n_groups_kv if n_groups_kv is not None else KV_GROUPS.get(cfg.name, cfg.n_groups)
    dkv = cfg.n_kv_heads * cfg.head_dim
    assert dkv % g == 0
    rng = np.random.default_rng(cfg.seed + 4243)
    for name in ("codebook_k", "codebook_v"):
        cb = (1.3 * rng.standard_normal((g, cfg.codebook_size, dkv // g), dtype=np.float32)).astype(np.float32)
        out[name] = round_to_bf16(cb) if cfg.dtype == "bf16" else cb
    return out
