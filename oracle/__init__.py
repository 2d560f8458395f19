"""CPU oracle for the Astra attention layer -- TEST INFRASTRUCTURE ONLY.

A thin ctypes layer over ``astra_oracle.c`` (plain C, fp64 arithmetic).  Only
tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the product path never does, and this package never imports the
product.  It holds no GPU code and shares nothing with the HIP library.

Notation follows the paper: ``X`` token embeddings, ``G`` groups, ``K``
codewords per group, ``Q = X W_q`` with ``W_q`` of shape ``[D, H_q*dh]``,
Eq. 1 for the mixed-precision attention.  Parity status: every function here
is pinned by tests/test_oracle_*.py (brute force, library routines, closed
forms, invariants); the outputs of the authors' trained models are "parity
unpinned" because the paper prints no worked numerical example.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "astra_oracle.c")
_LIB = os.path.join(_HERE, "libastra_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc (OpenMP over rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-fno-fast-math", "-ffp-contract=off", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # tests/test_oracle_mutations.py points this at deliberately broken builds of the C source to show that the pins
        # notice; nothing else sets it
        override = os.environ.get("ASTRA_ORACLE_LIB_OVERRIDE")
        if not override:
            build(force=False)
        lib = ctypes.CDLL(override or _LIB)
        lib.oracle_num_threads.restype = ctypes.c_int
        for name in ("oracle_vq_encode", "oracle_vq_decode", "oracle_linear",
                     "oracle_mixed_attention", "oracle_mixed_attention_valid",
                     "oracle_layer_forward", "oracle_layer_forward_valid",
                     "oracle_norm", "oracle_mlp", "oracle_block_forward", "oracle_layer_forward_kv",
                     "oracle_decode_attention", "oracle_codebook_stats", "oracle_codebook_update", "oracle_navq",
                     "oracle_rope", "oracle_layer_forward_rope", "oracle_block_forward_rope"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def vq_encode(x, codebook, return_gap: bool = False):
    """codes[t, g] = argmin_k ||X[t, g-th slice] - C[g, k]||^2, lowest index on ties.

    x [T, D] float, codebook [G, K, dg].  Returns int32 codes [T, G] (and the
    relative best/second-best gap [T, G] when asked).
    """
    x = _f32(x)
    codebook = _f32(codebook)
    G, K, dg = codebook.shape
    T, D = x.shape
    assert D == G * dg, "D must equal G * dg"
    codes = np.empty((T, G), dtype=np.int32)
    gap = np.empty((T, G), dtype=np.float64) if return_gap else None
    rc = _load().oracle_vq_encode(_p(x), ctypes.c_int64(T), D, G, K, _p(codebook), _p(codes), _p(gap))
    if rc:
        raise ValueError(f"oracle_vq_encode failed ({rc})")
    return (codes, gap) if return_gap else codes


def vq_decode(codes, codebook):
    """X_hat[t, g-th slice] = C[g, codes[t, g]] (exact copy)."""
    codebook = _f32(codebook)
    codes = _i32(codes)
    G, K, dg = codebook.shape
    T = codes.shape[0]
    assert codes.shape == (T, G)
    out = np.empty((T, G * dg), dtype=np.float32)
    rc = _load().oracle_vq_decode(_p(codes), ctypes.c_int64(T), G * dg, G, K, _p(codebook), _p(out))
    if rc:
        raise ValueError(f"oracle_vq_decode failed ({rc})")
    return out


def linear(x, w, bias=None):
    """x [T, D_in] @ w [D_in, D_out] (+ bias), fp64."""
    x = _f64(x)
    w = _f32(w)
    bias = _f32(bias)
    T, d_in = x.shape
    assert w.shape[0] == d_in
    out = np.empty((T, w.shape[1]), dtype=np.float64)
    rc = _load().oracle_linear(_p(x), ctypes.c_int64(T), d_in, w.shape[1], _p(w), _p(bias), _p(out))
    if rc:
        raise ValueError(f"oracle_linear failed ({rc})")
    return out


def project_codebook(codebook, w):
    """Pre-projected codebooks: P[g, k, :] = codebook[g, k, :] @ w[g*dg:(g+1)*dg, :], fp64 [G, K, D_out].  Written as the
    definition it comes from: the projection (linear) of the row that holds codeword k in slice g and zeros elsewhere,
    i.e. that codeword's share of the projection of any rebuilt row (Sec. 3.2: X-hat is rebuilt from the indices and
    projected with the same weights as the local rows)."""
    codebook = _f32(codebook)
    w = _f32(w)
    G, K, dg = codebook.shape
    assert w.shape[0] == G * dg
    out = np.empty((G, K, w.shape[1]), dtype=np.float64)
    for g in range(G):
        rows = np.zeros((K, G * dg), dtype=np.float32)
        rows[:, g * dg:(g + 1) * dg] = codebook[g]
        out[g] = linear(rows, w)
    return out


def gather_sum(codes, p, bias=None):
    """out[t, :] = bias + sum_g p[g, codes[t, g], :], fp64 (groups added in ascending order)."""
    codes = _i32(codes)
    p = _f64(p)
    G, K, n = p.shape
    T = codes.shape[0]
    assert codes.shape == (T, G) and (T == 0 or (codes.min() >= 0 and codes.max() < K))
    out = np.zeros((T, n), dtype=np.float64)
    if bias is not None:
        out += _f64(bias)[None, :]
    for g in range(G):
        out += p[g, codes[:, g], :]
    return out


def _u8(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a) != 0, dtype=np.uint8)


def mixed_attention(q, k_loc, v_loc, k_hat, v_hat, *, n_cls=0, causal=False, n_before=0,
                    scale=0.0, return_lse=False, return_probs=False, valid_hat=None):
    """Eq. 1 for one device.  q [T_q, H_q, dh]; k_loc/v_loc [T_q, H_kv, dh];
    k_hat/v_hat [T_n, H_kv, dh].  Returns out [T_q, H_q, dh] fp64
    (+ lse [H_q, T_q], + probs [H_q, T_q, T_q+T_n] when asked).
    valid_hat (optional, [T_n] of 0/1): non-local tokens whose codes never arrived (0) are dropped
    from the key/value set (Sec. 4.5, packet loss without retransmission)."""
    q, k_loc, v_loc, k_hat, v_hat = map(_f64, (q, k_loc, v_loc, k_hat, v_hat))
    Tq, Hq, dh = q.shape
    Hkv = k_loc.shape[1]
    Tn = k_hat.shape[0]
    assert k_loc.shape == (Tq, Hkv, dh) and v_loc.shape == (Tq, Hkv, dh)
    assert k_hat.shape == (Tn, Hkv, dh) and v_hat.shape == (Tn, Hkv, dh)
    out = np.empty((Tq, Hq, dh), dtype=np.float64)
    lse = np.empty((Hq, Tq), dtype=np.float64) if return_lse else None
    probs = np.empty((Hq, Tq, Tq + Tn), dtype=np.float64) if return_probs else None
    valid_hat = _u8(valid_hat)
    assert valid_hat is None or valid_hat.shape == (Tn,)
    rc = _load().oracle_mixed_attention_valid(
        _p(q), _p(k_loc), _p(v_loc), _p(k_hat), _p(v_hat), _p(valid_hat), Hq, Hkv, dh,
        int(n_cls), Tq - int(n_cls), Tn, int(bool(causal)), int(n_before),
        ctypes.c_double(scale), _p(out), _p(lse), _p(probs))
    if rc:
        raise ValueError(f"oracle_mixed_attention failed ({rc})")
    res = [out]
    if return_lse:
        res.append(lse)
    if return_probs:
        res.append(probs)
    return res[0] if len(res) == 1 else tuple(res)


def layer_forward(x_local, codes_nonlocal, codebook, wq, wk, wv, wo, *, n_q_heads, n_kv_heads,
                  n_cls=0, causal=False, n_before=0, scale=0.0,
                  bq=None, bk=None, bv=None, bo=None, return_gap=False, valid_nonlocal=None, rope_base=0.0):
    """One device's layer (Sec. 3.1).  Weights in the paper's orientation
    ``[D_in, D_out]``.  Returns (y [T_q, D] fp64, codes_local [T_l, G] int32
    [, gap [T_l, G]]).  valid_nonlocal (optional, [T_n] of 0/1): rows whose codes never
    arrived (0) are neither looked up nor attended to.  rope_base > 0 (optional, outside the paper):
    Q, K and K-hat are rotated by `rope` at their positions in the whole sequence."""
    x_local = _f32(x_local)
    codebook = _f32(codebook)
    codes_nonlocal = _i32(codes_nonlocal)
    wq, wk, wv, wo = map(_f32, (wq, wk, wv, wo))
    bq, bk, bv, bo = map(_f32, (bq, bk, bv, bo))
    G, K, dg = codebook.shape
    Tq, D = x_local.shape
    Tn = codes_nonlocal.shape[0]
    assert D == G * dg and codes_nonlocal.shape == (Tn, G)
    dh = wq.shape[1] // n_q_heads
    assert wq.shape == (D, n_q_heads * dh) and wk.shape == (D, n_kv_heads * dh)
    assert wv.shape == (D, n_kv_heads * dh) and wo.shape == (n_q_heads * dh, D)
    n_local = Tq - int(n_cls)
    y = np.empty((Tq, D), dtype=np.float64)
    codes_local = np.empty((n_local, G), dtype=np.int32)
    gap = np.empty((n_local, G), dtype=np.float64) if return_gap else None
    valid_nonlocal = _u8(valid_nonlocal)
    assert valid_nonlocal is None or valid_nonlocal.shape == (Tn,)
    rc = _load().oracle_layer_forward_rope(
        _p(x_local), _p(codes_nonlocal), _p(valid_nonlocal), _p(codebook), D, G, K,
        _p(wq), _p(wk), _p(wv), _p(wo), _p(bq), _p(bk), _p(bv), _p(bo),
        n_q_heads, n_kv_heads, dh, int(n_cls), n_local, Tn,
        int(bool(causal)), int(n_before), ctypes.c_double(scale), ctypes.c_double(rope_base),
        _p(y), _p(codes_local), _p(gap))
    if rc:
        raise ValueError(f"oracle_layer_forward failed ({rc})")
    return (y, codes_local, gap) if return_gap else (y, codes_local)


def rope(mat, pos, n_heads, base=10000.0):
    """Rotary position embedding (Su et al., RoFormer, Eq. 34, interleaved pairs; not part of the paper): mat [rows,
    n_heads * head_dim] rotated row by row at the positions pos [rows] (a negative position leaves the row as it is).
    Returns a new fp64 array."""
    out = _f64(mat).copy()
    rows, width = out.shape
    pos = np.ascontiguousarray(pos, dtype=np.int64)
    assert pos.shape == (rows,) and width % n_heads == 0
    rc = _load().oracle_rope(_p(out), ctypes.c_int64(rows), int(n_heads), width // n_heads, _p(pos), ctypes.c_double(base))
    if rc:
        raise ValueError(f"oracle_rope failed ({rc})")
    return out


NORM_KINDS = {"layernorm": 0, "rmsnorm": 1}
MLP_KINDS = {"gelu_tanh": 0, "gelu_erf": 1, "swiglu": 2}


def norm(x, kind, eps, gain=None, bias=None):
    """Row-wise LayerNorm / RMSNorm of x [T, D] in fp64 (the pre-norm of a Transformer block)."""
    x = _f64(x)
    gain, bias = _f32(gain), _f32(bias)
    T, D = x.shape
    out = np.empty((T, D), dtype=np.float64)
    rc = _load().oracle_norm(_p(x), ctypes.c_int64(T), D, NORM_KINDS[kind], ctypes.c_double(eps), _p(gain), _p(bias), _p(out))
    if rc:
        raise ValueError(f"oracle_norm failed ({rc})")
    return out


def mlp(h, kind, w1, w2, b1=None, b2=None):
    """Position-wise MLP (Sec. 3.1: run locally on each device).  h [T, D]; w1 [D, d_ff] (GELU kinds) or
    [D, 2 d_ff] = [gate | up] (swiglu); w2 [d_ff, D].  fp64."""
    h = _f64(h)
    w1, w2, b1, b2 = map(_f32, (w1, w2, b1, b2))
    T, D = h.shape
    d_ff = w2.shape[0]
    assert w1.shape == (D, 2 * d_ff if kind == "swiglu" else d_ff) and w2.shape == (d_ff, D)
    out = np.empty((T, D), dtype=np.float64)
    rc = _load().oracle_mlp(_p(h), ctypes.c_int64(T), D, d_ff, MLP_KINDS[kind], _p(w1), _p(b1), _p(w2), _p(b2), _p(out))
    if rc:
        raise ValueError(f"oracle_mlp failed ({rc})")
    return out


def block_forward(x, codes_nonlocal, codebook, wq, wk, wv, wo, *, norm_kind, eps, g1, g2, be1=None, be2=None,
                  mlp_kind, w1, w2, b1=None, b2=None, n_q_heads, n_kv_heads, n_cls=0, causal=False, n_before=0,
                  scale=0.0, bq=None, bk=None, bv=None, bo=None, valid_nonlocal=None, h_is_bf16=False, rope_base=0.0):
    """One Transformer block on one device (Sec. 3.1): out = r + mlp(norm2(r)), r = x + layer(norm1(x)).
    rope_base > 0: the layer rotates Q, K and K-hat (see layer_forward).
    x [T_q, D] is the fp64 residual stream.  Returns (x_out [T_q, D] fp64, codes_local [T_l, G] int32,
    gap [T_l, G], h [T_q, D] fp32 = the normalised tensor that was quantised and projected)."""
    x = _f64(x)
    codebook = _f32(codebook)
    codes_nonlocal = _i32(codes_nonlocal)
    wq, wk, wv, wo, w1, w2 = map(_f32, (wq, wk, wv, wo, w1, w2))
    bq, bk, bv, bo, b1, b2, g1, g2, be1, be2 = map(_f32, (bq, bk, bv, bo, b1, b2, g1, g2, be1, be2))
    G, K, dg = codebook.shape
    Tq, D = x.shape
    Tn = codes_nonlocal.shape[0]
    assert D == G * dg and codes_nonlocal.shape == (Tn, G)
    dh = wq.shape[1] // n_q_heads
    d_ff = w2.shape[0]
    assert wq.shape == (D, n_q_heads * dh) and wk.shape == (D, n_kv_heads * dh)
    assert wv.shape == (D, n_kv_heads * dh) and wo.shape == (n_q_heads * dh, D)
    assert w1.shape == (D, 2 * d_ff if mlp_kind == "swiglu" else d_ff) and w2.shape == (d_ff, D)
    n_local = Tq - int(n_cls)
    x_out = np.empty((Tq, D), dtype=np.float64)
    h = np.empty((Tq, D), dtype=np.float32)
    codes_local = np.empty((n_local, G), dtype=np.int32)
    gap = np.empty((n_local, G), dtype=np.float64)
    valid_nonlocal = _u8(valid_nonlocal)
    assert valid_nonlocal is None or valid_nonlocal.shape == (Tn,)
    rc = _load().oracle_block_forward_rope(
        _p(x), _p(codes_nonlocal), _p(valid_nonlocal), _p(codebook), D, G, K,
        NORM_KINDS[norm_kind], ctypes.c_double(eps), _p(g1), _p(be1), _p(g2), _p(be2),
        _p(wq), _p(wk), _p(wv), _p(wo), _p(bq), _p(bk), _p(bv), _p(bo),
        MLP_KINDS[mlp_kind], d_ff, _p(w1), _p(b1), _p(w2), _p(b2),
        n_q_heads, n_kv_heads, dh, int(n_cls), n_local, Tn, int(bool(causal)), int(n_before), ctypes.c_double(scale),
        int(bool(h_is_bf16)), ctypes.c_double(rope_base), _p(x_out), _p(codes_local), _p(gap), _p(h))
    if rc:
        raise ValueError(f"oracle_block_forward failed ({rc})")
    return x_out, codes_local, gap, h


def model_forward(x_all, layers, *, n_dev, n_q_heads, n_kv_heads, norm_kind, eps, mlp_kind, causal=False, cls=None,
                  h_is_bf16=False, lost=None, rope_base=0.0):
    """The whole multi-device procedure of Sec. 3.1 simulated on the CPU: the sequence x_all [N, D] (fp64 residual
    stream entering block 0) is cut into n_dev contiguous chunks; per block every device normalises and quantises its
    chunk, the codes are exchanged, and every device runs block_forward on its chunk with the others' codes
    (non-local rows in sequence order).  cls [n_dev, D] (optional): one class-token replica per device, first local
    row, never quantised; after the last block the replicas are averaged (Sec. 3.3).
    layers: list of dicts with codebook, wq, wk, wv, wo, g1, g2, w1, w2 and optionally be1, be2, bq, bk, bv, bo, b1, b2.
    lost (optional): lost[l][d] = 0/1 array over device d's non-local tokens at block l (1 = arrived).
    rope_base > 0 (optional, causal models only, where n_before places every chunk): rotary positions inside every layer.
    Returns dict: x [n_dev][T_q, D] final streams, codes [L][n_dev] (what each device sent), codes_nonlocal [L][n_dev]
    (what each device received), cls_pooled [D] or None."""
    x_all = _f64(x_all)
    N = x_all.shape[0]
    assert N % n_dev == 0
    assert not rope_base or causal
    tl = N // n_dev
    n_cls = 0 if cls is None else 1
    streams = []
    for d in range(n_dev):
        chunk = x_all[d * tl:(d + 1) * tl]
        streams.append(chunk if cls is None else np.concatenate([_f64(cls)[d:d + 1], chunk], axis=0))
    sent, received = [], []
    for l, p in enumerate(layers):
        opt = {k: p.get(k) for k in ("be1", "be2", "bq", "bk", "bv", "bo", "b1", "b2")}
        # phase 1: every device quantises the content rows of its normalised chunk
        codes = []
        for d in range(n_dev):
            h = norm(streams[d], norm_kind, eps, p["g1"], opt["be1"]).astype(np.float32)
            if h_is_bf16:
                u = h.view(np.uint32)
                h = ((u + (((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)).view(np.float32)
            codes.append(vq_encode(h[n_cls:], p["codebook"]))
        # phase 2: exchange, then every device runs its block
        nxt, rec = [], []
        for d in range(n_dev):
            nl = np.concatenate([codes[e] for e in range(n_dev) if e != d], axis=0)
            out, c_loc, _, _ = block_forward(
                streams[d], nl, p["codebook"], p["wq"], p["wk"], p["wv"], p["wo"], norm_kind=norm_kind, eps=eps,
                g1=p["g1"], g2=p["g2"], be1=opt["be1"], be2=opt["be2"], mlp_kind=mlp_kind, w1=p["w1"], w2=p["w2"],
                b1=opt["b1"], b2=opt["b2"], n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, n_cls=n_cls, causal=causal,
                n_before=d * tl if causal else 0, bq=opt["bq"], bk=opt["bk"], bv=opt["bv"], bo=opt["bo"],
                valid_nonlocal=None if lost is None else lost[l][d], h_is_bf16=h_is_bf16, rope_base=rope_base)
            assert np.array_equal(c_loc, codes[d])          # the block quantises the same tensor phase 1 did
            nxt.append(out)
            rec.append(nl)
        streams = nxt
        sent.append(codes)
        received.append(rec)
    pooled = None if cls is None else np.mean(np.stack([s[0] for s in streams]), axis=0)
    return {"x": streams, "codes": sent, "codes_nonlocal": received, "cls_pooled": pooled}


def layer_forward_kv(x_local, codes_k_nonlocal, codes_v_nonlocal, codebook_k, codebook_v, wq, wk, wv, wo, *, n_q_heads,
                     n_kv_heads, n_cls=0, causal=False, n_before=0, scale=0.0, bq=None, bk=None, bv=None, bo=None,
                     valid_nonlocal=None, kv_is_bf16=False):
    """The layer with K and V quantised after projection (App. memory cost: two codebooks per layer of dimension
    H_kv * dh).  codebook_k, codebook_v [G, K, dkv / G]; codes_*_nonlocal [T_n, G].  Returns dict: y [T_q, D] fp64,
    codes_k, codes_v [T_l, G] int32 (what this device sends), gap_k, gap_v, k, v [T_q, dkv] fp32 (K and V as stored)."""
    x_local = _f32(x_local)
    codebook_k, codebook_v = _f32(codebook_k), _f32(codebook_v)
    codes_k_nonlocal, codes_v_nonlocal = _i32(codes_k_nonlocal), _i32(codes_v_nonlocal)
    wq, wk, wv, wo = map(_f32, (wq, wk, wv, wo))
    bq, bk, bv, bo = map(_f32, (bq, bk, bv, bo))
    G, K, dg = codebook_k.shape
    Tq, D = x_local.shape
    Tn = codes_k_nonlocal.shape[0]
    dh = wq.shape[1] // n_q_heads
    dkv = n_kv_heads * dh
    assert codebook_v.shape == (G, K, dg) and G * dg == dkv
    assert codes_k_nonlocal.shape == (Tn, G) and codes_v_nonlocal.shape == (Tn, G)
    assert wq.shape == (D, n_q_heads * dh) and wk.shape == (D, dkv) and wv.shape == (D, dkv) and wo.shape == (n_q_heads * dh, D)
    n_local = Tq - int(n_cls)
    y = np.empty((Tq, D), dtype=np.float64)
    ck, cv = np.empty((n_local, G), dtype=np.int32), np.empty((n_local, G), dtype=np.int32)
    gk, gv = np.empty((n_local, G), dtype=np.float64), np.empty((n_local, G), dtype=np.float64)
    k, v = np.empty((Tq, dkv), dtype=np.float32), np.empty((Tq, dkv), dtype=np.float32)
    valid_nonlocal = _u8(valid_nonlocal)
    assert valid_nonlocal is None or valid_nonlocal.shape == (Tn,)
    rc = _load().oracle_layer_forward_kv(
        _p(x_local), _p(codes_k_nonlocal), _p(codes_v_nonlocal), _p(valid_nonlocal), _p(codebook_k), _p(codebook_v), D, G, K,
        _p(wq), _p(wk), _p(wv), _p(wo), _p(bq), _p(bk), _p(bv), _p(bo), n_q_heads, n_kv_heads, dh,
        int(n_cls), n_local, Tn, int(bool(causal)), int(n_before), ctypes.c_double(scale), int(bool(kv_is_bf16)),
        _p(y), _p(ck), _p(cv), _p(gk), _p(gv), _p(k), _p(v))
    if rc:
        raise ValueError(f"oracle_layer_forward_kv failed ({rc})")
    return {"y": y, "codes_k": ck, "codes_v": cv, "gap_k": gk, "gap_v": gv, "k": k, "v": v}


def decode_attention(q, k_loc, v_loc, codes_k, codes_v, codebook_k, codebook_v, *, scale=0.0, valid=None, return_lse=False):
    """One decoding step over a KV cache whose non-local part is VQ indices (App. memory cost).  q [H_q, dh];
    k_loc, v_loc [n_local, H_kv, dh]; codes_k, codes_v [n_nonlocal, G]; codebooks [G, K, dkv / G].
    Returns out [H_q, dh] fp64 (+ lse [H_q])."""
    q, k_loc, v_loc = map(_f64, (q, k_loc, v_loc))
    codes_k, codes_v = _i32(codes_k), _i32(codes_v)
    codebook_k, codebook_v = _f32(codebook_k), _f32(codebook_v)
    Hq, dh = q.shape
    n_local, Hkv = k_loc.shape[0], k_loc.shape[1]
    G, K, dg = codebook_k.shape
    Tn = codes_k.shape[0]
    assert k_loc.shape == (n_local, Hkv, dh) and v_loc.shape == (n_local, Hkv, dh)
    assert codes_k.shape == (Tn, G) and codes_v.shape == (Tn, G) and codebook_v.shape == (G, K, dg) and G * dg == Hkv * dh
    valid = _u8(valid)
    out = np.empty((Hq, dh), dtype=np.float64)
    lse = np.empty(Hq, dtype=np.float64)
    rc = _load().oracle_decode_attention(_p(q), _p(k_loc), _p(v_loc), _p(codes_k), _p(codes_v), _p(valid), _p(codebook_k),
                                         _p(codebook_v), G, K, Hq, Hkv, dh, n_local, Tn, ctypes.c_double(scale), _p(out), _p(lse))
    if rc:
        raise ValueError(f"oracle_decode_attention failed ({rc})")
    return (out, lse) if return_lse else out


def codebook_stats(x, codes, codebook):
    """Per-codeword statistics of an assignment (Sec. 3.2 training of the VQ module): counts [G, K] int64,
    sums [G, K, dg] fp64, sqerr [G] fp64 = sum_t ||x[t, slice g] - codebook[g, codes[t, g]]||^2 (Eq. 2's commitment
    term is beta * sqerr.sum())."""
    x, codes, codebook = _f32(x), _i32(codes), _f32(codebook)
    G, K, dg = codebook.shape
    T, D = x.shape
    assert D == G * dg and codes.shape == (T, G)
    counts = np.empty((G, K), dtype=np.int64)
    sums = np.empty((G, K, dg), dtype=np.float64)
    sqerr = np.empty(G, dtype=np.float64)
    rc = _load().oracle_codebook_stats(_p(x), _p(codes), _p(codebook), ctypes.c_int64(T), D, G, K, _p(counts), _p(sums), _p(sqerr))
    if rc:
        raise ValueError(f"oracle_codebook_stats failed ({rc})")
    return counts, sums, sqerr


def codebook_update(counts, sums, codebook_old, gamma=0.0, ema_n=None, ema_m=None):
    """EMA update of the codebook (gamma in (0, 1); ema_n [G, K], ema_m [G, K, dg] fp64 are updated in place), or with
    gamma = 0 one K-means centroid step.  A codeword whose (averaged) count is zero keeps its old value.
    Returns the new codebook [G, K, dg] fp64."""
    counts = np.ascontiguousarray(counts, dtype=np.int64)
    sums = _f64(sums)
    codebook_old = _f32(codebook_old)
    G, K, dg = codebook_old.shape
    assert counts.shape == (G, K) and sums.shape == (G, K, dg)
    for a in (ema_n, ema_m):
        assert a is None or (a.dtype == np.float64 and a.flags["C_CONTIGUOUS"])
    out = np.empty((G, K, dg), dtype=np.float64)
    rc = _load().oracle_codebook_update(_p(counts), _p(sums), ctypes.c_double(gamma), _p(ema_n), _p(ema_m), _p(codebook_old),
                                        G, K, dg, _p(out))
    if rc:
        raise ValueError(f"oracle_codebook_update failed ({rc})")
    return out


def navq(codes, codebook, mu, l_factor, z, lam):
    """NAVQ (Sec. 3.3): x_tilde = decode(codes) + lam * (mu + z @ l_factor.T), z standard normal draws passed in."""
    codes, codebook, mu, l_factor, z = _i32(codes), _f32(codebook), _f32(mu), _f32(l_factor), _f32(z)
    G, K, dg = codebook.shape
    T, D = z.shape
    assert D == G * dg and codes.shape == (T, G) and mu.shape == (D,) and l_factor.shape == (D, D)
    out = np.empty((T, D), dtype=np.float64)
    rc = _load().oracle_navq(_p(codes), _p(codebook), ctypes.c_int64(T), D, G, K, _p(mu), _p(l_factor), _p(z),
                             ctypes.c_double(lam), _p(out))
    if rc:
        raise ValueError(f"oracle_navq failed ({rc})")
    return out
