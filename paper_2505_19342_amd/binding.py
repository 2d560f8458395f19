"""ctypes binding of libastra_hip.so (include/astra.h).  Argument marshalling only: every step runs
in the HIP kernels.  Tensors are torch CUDA(ROCm) tensors used purely as device memory; the current
torch stream is handed to the library.  There is no CPU fallback: a missing library raises."""
from __future__ import annotations

import ctypes
import os

ASTRA_F32, ASTRA_BF16 = 0, 1
ASTRA_CODE_U8, ASTRA_CODE_U16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libastra_hip.so")
_lib = None

EXPORTS = ("astra_vq_prepare", "astra_vq_encode", "astra_vq_encode_workspace_bytes", "astra_vq_encode_ws", "astra_vq_decode", "astra_mixed_attention",
           "astra_mixed_attention_valid", "astra_layer_forward_valid",
           "astra_vq_project_codebook", "astra_layer_forward_preprojected",
           "astra_layer_workspace_bytes", "astra_layer_encode_fused", "astra_layer_forward", "astra_layer_forward_profiled",
           "astra_block_workspace_bytes", "astra_block_forward", "astra_stack_forward",
           "astra_layer_kv_workspace_bytes", "astra_layer_forward_kv",
           "astra_decode_attention_workspace_bytes", "astra_decode_attention",
           "astra_decode_attention_static_max_bytes", "astra_decode_attention_static",
           "astra_codebook_stats_workspace_bytes", "astra_codebook_stats", "astra_codebook_update", "astra_navq_forward",
           "astra_probe_mfma_bf16", "astra_status_string", "astra_version")
ASTRA_NORM_LAYER, ASTRA_NORM_RMS = 0, 1
ASTRA_MLP_GELU_TANH, ASTRA_MLP_GELU_ERF, ASTRA_MLP_SWIGLU = 0, 1, 2
NORM_KINDS = {"layernorm": ASTRA_NORM_LAYER, "rmsnorm": ASTRA_NORM_RMS}
MLP_KINDS = {"gelu_tanh": ASTRA_MLP_GELU_TANH, "gelu_erf": ASTRA_MLP_GELU_ERF, "swiglu": ASTRA_MLP_SWIGLU}


class AstraError(RuntimeError):
    pass


class VqDesc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("code_type", ctypes.c_int32), ("d_model", ctypes.c_int32),
                ("n_groups", ctypes.c_int32), ("codebook_size", ctypes.c_int32)]


class AttnDesc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("n_cls", ctypes.c_int32), ("n_local", ctypes.c_int32),
                ("n_nonlocal", ctypes.c_int32), ("causal", ctypes.c_int32), ("n_nonlocal_before", ctypes.c_int32),
                ("scale", ctypes.c_float)]


class LayerDesc(ctypes.Structure):
    _fields_ = [("vq", VqDesc), ("attn", AttnDesc)]


class LayerKvDesc(ctypes.Structure):
    _fields_ = [("vq", VqDesc), ("attn", AttnDesc), ("d_model", ctypes.c_int32)]


class DecodeDesc(ctypes.Structure):
    _fields_ = [("vq", VqDesc), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("n_local", ctypes.c_int32), ("n_nonlocal", ctypes.c_int32), ("scale", ctypes.c_float)]


class BlockDesc(ctypes.Structure):
    _fields_ = [("layer", LayerDesc), ("norm_kind", ctypes.c_int32), ("mlp_kind", ctypes.c_int32), ("d_ff", ctypes.c_int32),
                ("eps", ctypes.c_float), ("rope_base", ctypes.c_float)]


_BLOCK_WEIGHT_NAMES = ("codebook", "cnorm", "wq", "wk", "wv", "wo", "bq", "bk", "bv", "bo",
                       "norm1_gain", "norm1_bias", "norm2_gain", "norm2_bias", "w1", "b1", "w2", "b2")


class BlockWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in _BLOCK_WEIGHT_NAMES]


def load(build_if_missing: bool = True):
    """Load the built library (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise AstraError(f"{LIB_PATH} is not built; run paper_2505_19342_amd/build.py")
        from . import build as _build
        _build.build()
    # torch brings its own HIP runtime; it has to be in the process before this library resolves its dependency on one,
    # or two runtimes end up loaded and launches on torch's streams fail
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, f32p = ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p
    lib.astra_vq_prepare.argtypes = [ctypes.POINTER(VqDesc), vp, f32p, vp]
    lib.astra_vq_encode.argtypes = [ctypes.POINTER(VqDesc), vp, i64, vp, f32p, vp, vp]
    lib.astra_vq_decode.argtypes = [ctypes.POINTER(VqDesc), vp, i64, vp, vp, vp]
    lib.astra_mixed_attention.argtypes = [ctypes.POINTER(AttnDesc)] + [vp] * 8
    lib.astra_mixed_attention_valid.argtypes = [ctypes.POINTER(AttnDesc)] + [vp] * 9
    lib.astra_layer_forward_valid.argtypes = [ctypes.POINTER(LayerDesc)] + [vp] * 16 + [ctypes.c_size_t, vp]
    lib.astra_vq_encode_workspace_bytes.argtypes = [ctypes.POINTER(VqDesc), i64]
    lib.astra_vq_encode_workspace_bytes.restype = ctypes.c_size_t
    lib.astra_vq_encode_ws.argtypes = [ctypes.POINTER(VqDesc), vp, i64, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.astra_vq_encode_ws.restype = ctypes.c_int
    lib.astra_vq_project_codebook.argtypes = [ctypes.POINTER(VqDesc), vp, vp, ctypes.c_int32, vp, vp]
    lib.astra_vq_project_codebook.restype = ctypes.c_int
    lib.astra_layer_forward_preprojected.argtypes = [ctypes.POINTER(LayerDesc)] + [vp] * 18 + [ctypes.c_size_t, vp]
    lib.astra_layer_forward_preprojected.restype = ctypes.c_int
    lib.astra_layer_workspace_bytes.argtypes = [ctypes.POINTER(LayerDesc)]
    lib.astra_layer_workspace_bytes.restype = ctypes.c_size_t
    lib.astra_probe_mfma_bf16.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    lib.astra_probe_mfma_bf16.restype = ctypes.c_int
    lib.astra_layer_encode_fused.argtypes = [ctypes.POINTER(LayerDesc)]
    lib.astra_layer_encode_fused.restype = ctypes.c_int
    lib.astra_layer_forward.argtypes = [ctypes.POINTER(LayerDesc)] + [vp] * 15 + [ctypes.c_size_t, vp]
    lib.astra_layer_forward_profiled.argtypes = [ctypes.POINTER(LayerDesc)] + [vp] * 15 + [ctypes.c_size_t, vp,
                                                                                     ctypes.POINTER(ctypes.c_void_p)]
    lib.astra_block_workspace_bytes.argtypes = [ctypes.POINTER(BlockDesc)]
    lib.astra_block_workspace_bytes.restype = ctypes.c_size_t
    lib.astra_block_forward.argtypes = [ctypes.POINTER(BlockDesc), ctypes.POINTER(BlockWeights)] + [vp] * 7 + [ctypes.c_size_t, vp]
    lib.astra_block_forward.restype = ctypes.c_int
    lib.astra_layer_kv_workspace_bytes.argtypes = [ctypes.POINTER(LayerKvDesc)]
    lib.astra_layer_kv_workspace_bytes.restype = ctypes.c_size_t
    lib.astra_layer_forward_kv.argtypes = [ctypes.POINTER(LayerKvDesc)] + [vp] * 22 + [ctypes.c_size_t, vp]
    lib.astra_layer_forward_kv.restype = ctypes.c_int
    lib.astra_decode_attention_workspace_bytes.argtypes = [ctypes.POINTER(DecodeDesc)]
    lib.astra_decode_attention_workspace_bytes.restype = ctypes.c_size_t
    lib.astra_decode_attention.argtypes = [ctypes.POINTER(DecodeDesc)] + [vp] * 11 + [ctypes.c_size_t, vp]
    lib.astra_decode_attention.restype = ctypes.c_int
    lib.astra_decode_attention_static_max_bytes.argtypes = []
    lib.astra_decode_attention_static_max_bytes.restype = ctypes.c_size_t
    lib.astra_decode_attention_static.argtypes = [ctypes.POINTER(DecodeDesc)] + [vp] * 11
    lib.astra_decode_attention_static.restype = ctypes.c_int
    lib.astra_codebook_stats_workspace_bytes.argtypes = [ctypes.POINTER(VqDesc), i64]
    lib.astra_codebook_stats_workspace_bytes.restype = ctypes.c_size_t
    lib.astra_codebook_stats.argtypes = [ctypes.POINTER(VqDesc), vp, vp, i64, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.astra_codebook_stats.restype = ctypes.c_int
    lib.astra_codebook_update.argtypes = [ctypes.POINTER(VqDesc), vp, vp, ctypes.c_float, vp, vp, vp, vp, vp]
    lib.astra_codebook_update.restype = ctypes.c_int
    lib.astra_navq_forward.argtypes = [ctypes.POINTER(VqDesc), vp, i64, vp, vp, ctypes.c_float, vp, vp, vp, vp]
    lib.astra_navq_forward.restype = ctypes.c_int
    pp = ctypes.POINTER(ctypes.c_void_p)
    lib.astra_stack_forward.argtypes = [ctypes.POINTER(BlockDesc), ctypes.c_int32, ctypes.POINTER(BlockWeights), vp, pp, pp, vp, pp,
                                        vp, ctypes.c_size_t, vp]
    lib.astra_stack_forward.restype = ctypes.c_int
    lib.astra_status_string.argtypes = [ctypes.c_int]
    lib.astra_status_string.restype = ctypes.c_char_p
    lib.astra_version.restype = ctypes.c_int
    for name in EXPORTS[:4] + ("astra_layer_forward", "astra_layer_forward_profiled"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        raise AstraError(f"{what}: {load().astra_status_string(rc).decode()} ({rc})")


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise AstraError("device tensor required")
    if not t.is_contiguous():
        raise AstraError("contiguous tensor required")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def astra_version() -> int:
    return int(load().astra_version())


def astra_vq_prepare(desc: VqDesc, codebook, cnorm_out):
    _check(load().astra_vq_prepare(ctypes.byref(desc), _ptr(codebook), _ptr(cnorm_out), _stream()), "astra_vq_prepare")


def astra_vq_encode(desc: VqDesc, x, n_tokens: int, codebook, cnorm, codes_out):
    _check(load().astra_vq_encode(ctypes.byref(desc), _ptr(x), n_tokens, _ptr(codebook), _ptr(cnorm), _ptr(codes_out),
                                  _stream()), "astra_vq_encode")


def astra_vq_decode(desc: VqDesc, codes, n_tokens: int, codebook, x_hat_out):
    _check(load().astra_vq_decode(ctypes.byref(desc), _ptr(codes), n_tokens, _ptr(codebook), _ptr(x_hat_out), _stream()),
           "astra_vq_decode")


def astra_mixed_attention(desc: AttnDesc, q, k_local, v_local, k_hat, v_hat, out, lse_out=None):
    _check(load().astra_mixed_attention(ctypes.byref(desc), _ptr(q), _ptr(k_local), _ptr(v_local), _ptr(k_hat), _ptr(v_hat),
                                        _ptr(out), _ptr(lse_out), _stream()), "astra_mixed_attention")


def astra_mixed_attention_valid(desc: AttnDesc, q, k_local, v_local, k_hat, v_hat, valid_bits, out, lse_out=None):
    """valid_bits: int64 device tensor of ceil(T_n / 64) words (see pack_valid_bits) or None."""
    _check(load().astra_mixed_attention_valid(ctypes.byref(desc), _ptr(q), _ptr(k_local), _ptr(v_local), _ptr(k_hat), _ptr(v_hat),
                                              _ptr(valid_bits), _ptr(out), _ptr(lse_out), _stream()), "astra_mixed_attention_valid")


def astra_layer_forward_valid(desc: LayerDesc, x_local, codes_nonlocal, valid_bits, codebook, cnorm, wq, wk, wv, wo,
                              bq, bk, bv, bo, y_out, codes_local_out, workspace):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().astra_layer_forward_valid(ctypes.byref(desc), _ptr(x_local), _ptr(codes_nonlocal), _ptr(valid_bits),
                                            _ptr(codebook), _ptr(cnorm), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo),
                                            _ptr(bq), _ptr(bk), _ptr(bv), _ptr(bo), _ptr(y_out), _ptr(codes_local_out),
                                            _ptr(workspace), nbytes, _stream()), "astra_layer_forward_valid")


def astra_vq_encode_workspace_bytes(desc: VqDesc, n_tokens: int) -> int:
    return int(load().astra_vq_encode_workspace_bytes(ctypes.byref(desc), n_tokens))


def astra_vq_encode_ws(desc: VqDesc, x, n_tokens: int, codebook, cnorm, codes_out, workspace):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().astra_vq_encode_ws(ctypes.byref(desc), _ptr(x), n_tokens, _ptr(codebook), _ptr(cnorm), _ptr(codes_out),
                                     _ptr(workspace), nbytes, _stream()), "astra_vq_encode_ws")


def astra_vq_project_codebook(desc: VqDesc, codebook, w, n_out: int, p_out):
    _check(load().astra_vq_project_codebook(ctypes.byref(desc), _ptr(codebook), _ptr(w), n_out, _ptr(p_out), _stream()),
           "astra_vq_project_codebook")


def astra_layer_forward_preprojected(desc: LayerDesc, x_local, codes_nonlocal, valid_bits, codebook, cnorm, p_k, p_v, wq, wk, wv, wo,
                                     bq, bk, bv, bo, y_out, codes_local_out, workspace):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().astra_layer_forward_preprojected(ctypes.byref(desc), _ptr(x_local), _ptr(codes_nonlocal), _ptr(valid_bits),
                                                   _ptr(codebook), _ptr(cnorm), _ptr(p_k), _ptr(p_v), _ptr(wq), _ptr(wk), _ptr(wv),
                                                   _ptr(wo), _ptr(bq), _ptr(bk), _ptr(bv), _ptr(bo), _ptr(y_out),
                                                   _ptr(codes_local_out), _ptr(workspace), nbytes, _stream()),
           "astra_layer_forward_preprojected")


def pack_valid_bits(valid):
    """Host helper: a 0/1 array [T_n] -> numpy uint64 words, bit (t % 64) of word t / 64 = valid[t]."""
    import numpy as np
    v = np.asarray(valid) != 0
    n_words = (v.size + 63) // 64
    padded = np.zeros(n_words * 64, dtype=np.uint8)
    padded[:v.size] = v
    return np.packbits(padded, bitorder="little").view(np.uint64)


def astra_layer_workspace_bytes(desc: LayerDesc) -> int:
    return int(load().astra_layer_workspace_bytes(ctypes.byref(desc)))


def astra_block_workspace_bytes(desc: BlockDesc) -> int:
    return int(load().astra_block_workspace_bytes(ctypes.byref(desc)))


def block_weights(**tensors) -> BlockWeights:
    """Device tensors by the field names of astra_block_weights (missing or None = NULL).  The caller keeps the
    tensors alive: the structure holds bare addresses."""
    unknown = set(tensors) - set(_BLOCK_WEIGHT_NAMES)
    if unknown:
        raise AstraError(f"unknown block weight(s): {sorted(unknown)}")
    w = BlockWeights()
    for n in _BLOCK_WEIGHT_NAMES:
        p = _ptr(tensors.get(n))
        setattr(w, n, p.value if p is not None else None)
    return w


def astra_block_forward(desc: BlockDesc, weights: BlockWeights, x, codes_nonlocal, valid_bits, x_out, codes_local_out, h_out,
                        workspace):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().astra_block_forward(ctypes.byref(desc), ctypes.byref(weights), _ptr(x), _ptr(codes_nonlocal), _ptr(valid_bits),
                                      _ptr(x_out), _ptr(codes_local_out), _ptr(h_out), _ptr(workspace), nbytes, _stream()),
           "astra_block_forward")


def astra_layer_kv_workspace_bytes(desc: LayerKvDesc) -> int:
    return int(load().astra_layer_kv_workspace_bytes(ctypes.byref(desc)))


def astra_layer_forward_kv(desc: LayerKvDesc, x_local, codes_k_nonlocal, codes_v_nonlocal, valid_bits, codebook_k, cnorm_k,
                           codebook_v, cnorm_v, wq, wk, wv, wo, bq, bk, bv, bo, y_out, codes_k_local_out, codes_v_local_out,
                           k_out, v_out, workspace):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().astra_layer_forward_kv(
        ctypes.byref(desc), _ptr(x_local), _ptr(codes_k_nonlocal), _ptr(codes_v_nonlocal), _ptr(valid_bits), _ptr(codebook_k),
        _ptr(cnorm_k), _ptr(codebook_v), _ptr(cnorm_v), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo), _ptr(bq), _ptr(bk), _ptr(bv),
        _ptr(bo), _ptr(y_out), _ptr(codes_k_local_out), _ptr(codes_v_local_out), _ptr(k_out), _ptr(v_out), _ptr(workspace),
        nbytes, _stream()), "astra_layer_forward_kv")


def astra_decode_attention_workspace_bytes(desc: DecodeDesc) -> int:
    return int(load().astra_decode_attention_workspace_bytes(ctypes.byref(desc)))


def astra_decode_attention(desc: DecodeDesc, q, k_cache, v_cache, codes_k, codes_v, valid_bits, codebook_k, codebook_v, out,
                           lse_out, workspace):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().astra_decode_attention(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(codes_k), _ptr(codes_v),
                                         _ptr(valid_bits), _ptr(codebook_k), _ptr(codebook_v), _ptr(out), _ptr(lse_out),
                                         _ptr(workspace), nbytes, _stream()), "astra_decode_attention")


def astra_decode_attention_static_max_bytes() -> int:
    return int(load().astra_decode_attention_static_max_bytes())


def astra_decode_attention_static(desc: DecodeDesc, q, k_cache, v_cache, codes_k, codes_v, valid_bits, codebook_k, codebook_v, out,
                                  lse_out):
    _check(load().astra_decode_attention_static(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(codes_k),
                                                _ptr(codes_v), _ptr(valid_bits), _ptr(codebook_k), _ptr(codebook_v), _ptr(out),
                                                _ptr(lse_out), _stream()), "astra_decode_attention_static")


def astra_codebook_stats_workspace_bytes(desc: VqDesc, n_tokens: int) -> int:
    return int(load().astra_codebook_stats_workspace_bytes(ctypes.byref(desc), n_tokens))


def astra_codebook_stats(desc: VqDesc, x, codes, n_tokens: int, codebook, counts_out, sums_out, sqerr_out, workspace):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().astra_codebook_stats(ctypes.byref(desc), _ptr(x), _ptr(codes), n_tokens, _ptr(codebook), _ptr(counts_out),
                                       _ptr(sums_out), _ptr(sqerr_out), _ptr(workspace), nbytes, _stream()), "astra_codebook_stats")


def astra_codebook_update(desc: VqDesc, counts, sums, gamma: float, ema_n, ema_m, codebook_old, codebook_new_out):
    _check(load().astra_codebook_update(ctypes.byref(desc), _ptr(counts), _ptr(sums), gamma, _ptr(ema_n), _ptr(ema_m),
                                        _ptr(codebook_old), _ptr(codebook_new_out), _stream()), "astra_codebook_update")


def astra_navq_forward(desc: VqDesc, codes, n_tokens: int, codebook, mu, lam: float, z, noise_factor, x_tilde_out):
    _check(load().astra_navq_forward(ctypes.byref(desc), _ptr(codes), n_tokens, _ptr(codebook), _ptr(mu), lam, _ptr(z),
                                     _ptr(noise_factor), _ptr(x_tilde_out), _stream()), "astra_navq_forward")


def _ptr_array(tensors):
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        p = _ptr(t)
        arr[i] = p.value if p is not None else None
    return arr


def astra_stack_forward(desc: BlockDesc, weights, x, codes_nonlocal, valid_bits, x_out, codes_local_out, workspace):
    """weights: list of BlockWeights (one per block); codes_nonlocal, codes_local_out: lists of device tensors;
    valid_bits: None or a list of (tensor | None)."""
    n = len(weights)
    if len(codes_nonlocal) != n or len(codes_local_out) != n or (valid_bits is not None and len(valid_bits) != n):
        raise AstraError("one entry per block required")
    w_arr = (BlockWeights * n)(*weights)
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().astra_stack_forward(ctypes.byref(desc), n, w_arr, _ptr(x), _ptr_array(codes_nonlocal),
                                      None if valid_bits is None else _ptr_array(valid_bits), _ptr(x_out),
                                      _ptr_array(codes_local_out), _ptr(workspace), nbytes, _stream()), "astra_stack_forward")


def astra_probe_mfma_bf16(out, n_blocks: int, iters: int):
    """out: float32 device tensor with at least n_blocks * 512 elements."""
    _check(load().astra_probe_mfma_bf16(_ptr(out), n_blocks, iters, _stream()), "astra_probe_mfma_bf16")


def astra_layer_encode_fused(desc: LayerDesc) -> bool:
    rc = int(load().astra_layer_encode_fused(ctypes.byref(desc)))
    if rc < 0:
        _check(rc, "astra_layer_encode_fused")
    return rc == 1


def astra_layer_forward(desc: LayerDesc, x_local, codes_nonlocal, codebook, cnorm, wq, wk, wv, wo,
                        bq, bk, bv, bo, y_out, codes_local_out, workspace):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().astra_layer_forward(ctypes.byref(desc), _ptr(x_local), _ptr(codes_nonlocal), _ptr(codebook), _ptr(cnorm),
                                      _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo), _ptr(bq), _ptr(bk), _ptr(bv), _ptr(bo),
                                      _ptr(y_out), _ptr(codes_local_out), _ptr(workspace), nbytes, _stream()),
           "astra_layer_forward")


def astra_layer_forward_profiled(desc: LayerDesc, x_local, codes_nonlocal, codebook, cnorm, wq, wk, wv, wo,
                                 bq, bk, bv, bo, y_out, codes_local_out, workspace, stage_events):
    """stage_events: a ctypes array of 7 hipEvent_t handles (see HipEvents and include/astra.h)."""
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().astra_layer_forward_profiled(
        ctypes.byref(desc), _ptr(x_local), _ptr(codes_nonlocal), _ptr(codebook), _ptr(cnorm),
        _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo), _ptr(bq), _ptr(bk), _ptr(bv), _ptr(bo),
        _ptr(y_out), _ptr(codes_local_out), _ptr(workspace), nbytes, _stream(), stage_events),
        "astra_layer_forward_profiled")


class HipEvents:
    """n timing-enabled hipEvent_t created through the HIP runtime itself (no torch objects), for the
    profiled entry point.  elapsed_ms(i, j) is valid after the stream has been synchronised."""

    def __init__(self, n: int):
        self._hip = ctypes.CDLL("libamdhip64.so")
        self._hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self._hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self._hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.handles = (ctypes.c_void_p * n)()
        for i in range(n):
            ev = ctypes.c_void_p()
            if self._hip.hipEventCreate(ctypes.byref(ev)) != 0:
                raise AstraError("hipEventCreate failed")
            self.handles[i] = ev

    def elapsed_ms(self, i: int, j: int) -> float:
        ms = ctypes.c_float()
        if self._hip.hipEventElapsedTime(ctypes.byref(ms), self.handles[i], self.handles[j]) != 0:
            raise AstraError("hipEventElapsedTime failed")
        return float(ms.value)

    def __del__(self):
        try:
            for h in self.handles:
                if h:
                    self._hip.hipEventDestroy(h)
        except Exception:
            pass


# ---- descriptor helpers (pure bookkeeping) ------------------------------------------------------

def vq_desc(dtype: str, d_model: int, n_groups: int, codebook_size: int) -> VqDesc:
    return VqDesc(ASTRA_BF16 if dtype == "bf16" else ASTRA_F32,
                  ASTRA_CODE_U8 if codebook_size <= 256 else ASTRA_CODE_U16, d_model, n_groups, codebook_size)


def attn_desc(dtype: str, n_q_heads: int, n_kv_heads: int, head_dim: int, n_cls: int, n_local: int, n_nonlocal: int,
              causal: bool, n_before: int = 0, scale: float = 0.0) -> AttnDesc:
    return AttnDesc(ASTRA_BF16 if dtype == "bf16" else ASTRA_F32, n_q_heads, n_kv_heads, head_dim, n_cls, n_local,
                    n_nonlocal, int(bool(causal)), n_before if causal else 0, scale)


def block_desc(layer: LayerDesc, norm_kind: str, mlp_kind: str, d_ff: int, eps: float, rope_base: float = 0.0) -> BlockDesc:
    return BlockDesc(layer, NORM_KINDS[norm_kind], MLP_KINDS[mlp_kind], d_ff, eps, rope_base)
