"""Pins for the oracle's optional rotary position embedding (not part of the paper, which never says how its
Llama-shaped model encodes positions; Su et al., "RoFormer", Sec. 3.2.2 / Eq. 34, interleaved pairs).  The rotation
is pinned to its closed form on a worked example, to the complex-number statement of the same definition written
independently below, and to the properties the definition exists for (relative positions, norms); where the layer
applies it, and at which positions, is pinned by library attention on independently rotated queries and keys and
by the lossless-codebook case, in which a device must reproduce its rows of the single-device model."""
import numpy as np
import pytest
import torch

import oracle


def rope_complex(mat, pos, n_heads, base):
    """The same definition through complex multiplication: (x[2i] + j x[2i+1]) * exp(j * m * base^(-2i/dh))."""
    rows, width = mat.shape
    dh = width // n_heads
    x = np.asarray(mat, dtype=np.float64).reshape(rows, n_heads, dh // 2, 2)
    z = x[..., 0] + 1j * x[..., 1]
    theta = np.asarray(base, dtype=np.float64) ** (-2.0 * np.arange(dh // 2) / dh)
    ang = np.asarray(pos, dtype=np.float64)[:, None, None] * theta[None, None, :]
    z = z * np.exp(1j * ang)
    return np.stack([z.real, z.imag], axis=-1).reshape(rows, width)


def test_worked_example_closed_form():
    # one head of four values at position 1, base 10000: the angles are 1 and 10000^(-1/2) = 0.01 radians
    out = oracle.rope(np.array([[1.0, 0.0, 0.0, 2.0]]), [1], 1, 10000.0)
    expect = [np.cos(1.0), np.sin(1.0), -2.0 * np.sin(0.01), 2.0 * np.cos(0.01)]
    np.testing.assert_allclose(out[0], expect, rtol=1e-15, atol=1e-16)
    # a quarter turn: position pi/2 with angle factor 1 (pair 0) maps (a, b) to (-b, a)
    out = oracle.rope(np.array([[3.0, 4.0]]), [1], 1, base=1.0)      # base 1: every pair turns by the position itself
    np.testing.assert_allclose(out[0], [3 * np.cos(1) - 4 * np.sin(1), 3 * np.sin(1) + 4 * np.cos(1)], rtol=1e-15)


@pytest.mark.parametrize("n_heads,dh,base", [(1, 2, 10000.0), (3, 8, 10000.0), (2, 64, 500000.0), (4, 6, 17.0)])
def test_equals_complex_multiplication(n_heads, dh, base):
    rng = np.random.default_rng(n_heads * 100 + dh)
    x = rng.standard_normal((9, n_heads * dh))
    pos = np.array([0, 1, 2, 3, 50, 1000, 8191, 100000, 7])
    np.testing.assert_allclose(oracle.rope(x, pos, n_heads, base), rope_complex(x, pos, n_heads, base), rtol=1e-11, atol=1e-12)


def test_properties_position_zero_norms_relative_positions_and_skipped_rows():
    rng = np.random.default_rng(5)
    n_heads, dh = 2, 16
    q, k = rng.standard_normal((1, n_heads * dh)), rng.standard_normal((1, n_heads * dh))
    assert np.array_equal(oracle.rope(q, [0], n_heads), q)                       # position 0 is the identity
    assert np.array_equal(oracle.rope(q, [-1], n_heads), q)                      # a row without a position is left alone
    r = oracle.rope(q, [37], n_heads)
    np.testing.assert_allclose((r.reshape(n_heads, dh) ** 2).sum(-1), (q.reshape(n_heads, dh) ** 2).sum(-1), rtol=1e-14)
    assert np.abs(r - q).max() > 0.1
    # per head, <R_m q, R_n k> depends on m - n only
    def dots(m, n):
        a, b = oracle.rope(q, [m], n_heads).reshape(n_heads, dh), oracle.rope(k, [n], n_heads).reshape(n_heads, dh)
        return (a * b).sum(-1)
    np.testing.assert_allclose(dots(12, 5), dots(107, 100), rtol=1e-11)
    np.testing.assert_allclose(dots(12, 5), dots(7, 0), rtol=1e-11)
    assert np.abs(dots(12, 5) - dots(12, 6)).max() > 1e-3
    # the lowest pair turns fastest (angle = position), the highest slowest: position 1 moves pair 0 by one radian
    e = np.zeros((1, dh)); e[0, 0] = 1.0
    np.testing.assert_allclose(oracle.rope(e, [1], 1)[0, :2], [np.cos(1.0), np.sin(1.0)], rtol=1e-15)
    e = np.zeros((1, dh)); e[0, dh - 2] = 1.0
    t_last = 10000.0 ** (-(dh - 2) / dh)
    np.testing.assert_allclose(oracle.rope(e, [1], 1)[0, dh - 2:], [np.cos(t_last), np.sin(t_last)], rtol=1e-15)


def sdpa(q, k, v, causal):
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).permute(1, 0, 2)[None] for a in (q, k, v))
    if tk.shape[1] != tq.shape[1]:
        rep = tq.shape[1] // tk.shape[1]
        tk, tv = tk.repeat_interleave(rep, dim=1), tv.repeat_interleave(rep, dim=1)
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)[0].permute(1, 0, 2).numpy()


def single_device_layer(x, wq, wk, wv, wo, hq, hkv, dh, causal, base):
    """The unquantised layer on one device through library routines, queries and keys rotated by the complex form."""
    n = x.shape[0]
    x64 = x.astype(np.float64)
    pos = np.arange(n)
    q = rope_complex(x64 @ wq.astype(np.float64), pos, hq, base).reshape(n, hq, dh)
    k = rope_complex(x64 @ wk.astype(np.float64), pos, hkv, base).reshape(n, hkv, dh)
    v = (x64 @ wv.astype(np.float64)).reshape(n, hkv, dh)               # values are not rotated
    return sdpa(q, k, v, causal).reshape(n, hq * dh) @ wo.astype(np.float64)


def make_layer(rng, n, d, hq, hkv, dh):
    x = rng.standard_normal((n, d)).astype(np.float32)
    w = lambda a, b: (rng.standard_normal((a, b)) / np.sqrt(a)).astype(np.float32)
    return x, w(d, hq * dh), w(d, hkv * dh), w(d, hkv * dh), w(hq * dh, d)


@pytest.mark.parametrize("causal", [False, True])
def test_all_local_layer_is_library_attention_on_rotated_queries_and_keys(causal):
    rng = np.random.default_rng(31)
    n, d, hq, hkv, dh = 24, 16, 4, 2, 8
    x, wq, wk, wv, wo = make_layer(rng, n, d, hq, hkv, dh)
    codebook = rng.standard_normal((2, 4, d // 2)).astype(np.float32)
    none = np.zeros((0, 2), np.int32)
    y, _ = oracle.layer_forward(x, none, codebook, wq, wk, wv, wo, n_q_heads=hq, n_kv_heads=hkv, causal=causal, rope_base=10000.0)
    np.testing.assert_allclose(y, single_device_layer(x, wq, wk, wv, wo, hq, hkv, dh, causal, 10000.0), rtol=1e-9, atol=1e-11)
    y0, _ = oracle.layer_forward(x, none, codebook, wq, wk, wv, wo, n_q_heads=hq, n_kv_heads=hkv, causal=causal)
    assert np.abs(y - y0).max() > 1e-3                                    # and it is not the unrotated layer


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("rank", [0, 1, 3])
def test_lossless_codebook_recovers_the_single_device_layer_at_every_rank(causal, rank):
    """Every non-local token is its own codeword (G = 1), so X-hat = X and the device must produce its rows of the
    single-device layer: this fixes the positions of local rows (n_before + i) and of non-local rows on either side
    of the local chunk."""
    rng = np.random.default_rng(40 + rank)
    n, n_dev, d, hq, hkv, dh = 32, 4, 12, 4, 2, 6
    x, wq, wk, wv, wo = make_layer(rng, n, d, hq, hkv, dh)
    tl = n // n_dev
    lo, hi = rank * tl, (rank + 1) * tl
    x_nonlocal = np.concatenate([x[:lo], x[hi:]])
    codebook = x_nonlocal[None]
    codes_nonlocal = oracle.vq_encode(x_nonlocal, codebook)
    y, _ = oracle.layer_forward(x[lo:hi], codes_nonlocal, codebook, wq, wk, wv, wo, n_q_heads=hq, n_kv_heads=hkv,
                                causal=causal, n_before=lo, rope_base=10000.0)
    ref = single_device_layer(x, wq, wk, wv, wo, hq, hkv, dh, causal, 10000.0)[lo:hi]
    np.testing.assert_allclose(y, ref, rtol=1e-9, atol=1e-11)


def test_class_row_is_not_rotated_and_block_passes_the_base_through():
    rng = np.random.default_rng(9)
    n, d, hq, hkv, dh = 10, 16, 2, 2, 8
    x, wq, wk, wv, wo = make_layer(rng, n, d, hq, hkv, dh)
    codebook = rng.standard_normal((2, 4, d // 2)).astype(np.float32)
    none = np.zeros((0, 2), np.int32)
    # with a class row first: content row i sits at position i, the class row keeps its unrotated query and key
    y, _ = oracle.layer_forward(x, none, codebook, wq, wk, wv, wo, n_q_heads=hq, n_kv_heads=hkv, n_cls=1, rope_base=100.0)
    x64 = x.astype(np.float64)
    pos = np.concatenate([[0], np.arange(n - 1)])           # position 0 is the identity: stands in for "not rotated"
    q = rope_complex(x64 @ wq.astype(np.float64), pos, hq, 100.0).reshape(n, hq, dh)
    k = rope_complex(x64 @ wk.astype(np.float64), pos, hkv, 100.0).reshape(n, hkv, dh)
    v = (x64 @ wv.astype(np.float64)).reshape(n, hkv, dh)
    np.testing.assert_allclose(y, sdpa(q, k, v, False).reshape(n, hq * dh) @ wo.astype(np.float64), rtol=1e-9, atol=1e-11)
    # the block: same wiring as without rotation, with the rotated layer inside
    g = np.ones(d, np.float32)
    w1 = (rng.standard_normal((d, 24)) / 4).astype(np.float32)
    w2 = (rng.standard_normal((24, d)) / 5).astype(np.float32)
    xs = rng.standard_normal((n, d))
    kw = dict(norm_kind="rmsnorm", eps=1e-6, g1=g, g2=g, mlp_kind="gelu_tanh", w1=w1, w2=w2, n_q_heads=hq, n_kv_heads=hkv, causal=True)
    out, _, _, h = oracle.block_forward(xs, none, codebook, wq, wk, wv, wo, rope_base=10000.0, **kw)
    yl, _ = oracle.layer_forward(h, none, codebook, wq, wk, wv, wo, n_q_heads=hq, n_kv_heads=hkv, causal=True, rope_base=10000.0)
    r = xs + yl
    ref = r + oracle.mlp(oracle.norm(r, "rmsnorm", 1e-6, g), "gelu_tanh", w1, w2)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    out0, _, _, _ = oracle.block_forward(xs, none, codebook, wq, wk, wv, wo, **kw)
    assert np.abs(out - out0).max() > 1e-4
