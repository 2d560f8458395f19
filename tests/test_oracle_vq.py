"""Pins for the CPU oracle's grouped VQ encode / decode (Sec. 2 "Vanilla VQ", "Grouped VQ";
Sec. 3.2 "Vector-Quantized Non-Local Tokens").  None of these re-call the oracle's own formula:
they use a second formulation (expanded distance + full sort), a library nearest-neighbour
routine, hand-computed cases and invariants."""
import numpy as np
import pytest
from scipy.cluster.vq import vq as scipy_vq
from scipy.spatial.distance import cdist

import oracle


def brute_force_codes(x, codebook):
    """Independent formulation: ||c||^2 - 2 x.c + ||x||^2 in long double, then a full stable
    sort of the K distances (first of equal keys = lowest index)."""
    G, K, dg = codebook.shape
    T = x.shape[0]
    xs = x.astype(np.longdouble).reshape(T, G, dg)
    cb = codebook.astype(np.longdouble)
    codes = np.empty((T, G), dtype=np.int32)
    gaps = np.empty((T, G), dtype=np.float64)
    for t in range(T):
        for g in range(G):
            d = np.array([np.dot(cb[g, k], cb[g, k]) - 2 * np.dot(xs[t, g], cb[g, k]) + np.dot(xs[t, g], xs[t, g])
                          for k in range(K)], dtype=np.longdouble)
            order = np.argsort(d, kind="stable")
            codes[t, g] = order[0]
            gaps[t, g] = float((d[order[1]] - d[order[0]]) / d[order[0]]) if K > 1 and d[order[0]] > 0 else np.inf
    return codes, gaps


@pytest.mark.parametrize("seed", range(6))
def test_encode_matches_brute_force_tiny(seed):
    rng = np.random.default_rng(seed)
    T, G, K, dg = rng.integers(1, 9), rng.integers(1, 4), rng.integers(2, 9), rng.integers(1, 5)
    x = rng.standard_normal((T, G * dg)).astype(np.float32)
    cb = rng.standard_normal((G, K, dg)).astype(np.float32)
    codes, gap = oracle.vq_encode(x, cb, return_gap=True)
    ref, ref_gap = brute_force_codes(x, cb)
    assert np.array_equal(codes, ref)
    np.testing.assert_allclose(gap, ref_gap, rtol=1e-9)


def test_encode_hand_worked_example():
    # D = 4, G = 2, dg = 2, K = 3.  Distances worked by hand:
    #   token 0 = (0,0 | 3,4): group 0 vs {(1,0),(0,0.5),(2,2)} -> {1, 0.25, 8}  -> code 1
    #                          group 1 vs {(3,3),(0,0),(3,5)}   -> {1, 25, 1}    -> tie, lowest index 0
    #   token 1 = (2,1 | -1,0): group 0 -> {2, 4.25, 1} -> code 2; group 1 -> {25, 1, 41} -> code 1
    cb = np.array([[[1, 0], [0, 0.5], [2, 2]], [[3, 3], [0, 0], [3, 5]]], dtype=np.float32)
    x = np.array([[0, 0, 3, 4], [2, 1, -1, 0]], dtype=np.float32)
    codes, gap = oracle.vq_encode(x, cb, return_gap=True)
    assert codes.tolist() == [[1, 0], [2, 1]]
    np.testing.assert_allclose(gap, [[(1 - 0.25) / 0.25, 0.0], [(2 - 1) / 1, (25 - 1) / 1]])


def test_encode_exact_ties_take_lowest_index():
    cb = np.zeros((1, 5, 3), dtype=np.float32)
    cb[0, 1] = cb[0, 3] = [1, 2, 3]          # duplicates: 1 must win over 3
    cb[0, 0] = [9, 9, 9]
    cb[0, 2] = cb[0, 4] = [-1, -2, -3]        # duplicates: 2 must win over 4
    x = np.array([[1, 2, 3], [-1, -2, -3.5], [0, 0, 0]], dtype=np.float32)
    codes = oracle.vq_encode(x, cb)
    assert codes[:, 0].tolist() == [1, 2, 1]  # the origin is equidistant from +-(1,2,3): lowest of {1,2,3,4}


def test_every_codeword_encodes_to_itself_and_decodes_back():
    rng = np.random.default_rng(10)
    G, K, dg = 3, 17, 5
    cb = rng.standard_normal((G, K, dg)).astype(np.float32)
    # token k is the concatenation of codeword k of every group
    x = np.concatenate([cb[g] for g in range(G)], axis=1)
    codes = oracle.vq_encode(x, cb)
    assert np.array_equal(codes, np.repeat(np.arange(K)[:, None], G, axis=1))
    assert np.array_equal(oracle.vq_decode(codes, cb), x)          # decode(encode(c)) == c, bit for bit


def test_single_group_is_vanilla_vq_library_routine():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((200, 24)).astype(np.float32)
    cb = rng.standard_normal((1, 64, 24)).astype(np.float32)
    codes = oracle.vq_encode(x, cb)[:, 0]
    lib_codes, _ = scipy_vq(x.astype(np.float64), cb[0].astype(np.float64))
    assert np.array_equal(codes, lib_codes)
    assert np.array_equal(codes, np.argmin(cdist(x.astype(np.float64), cb[0].astype(np.float64), "sqeuclidean"), axis=1))


def test_grouped_equals_per_group_library_routine():
    rng = np.random.default_rng(12)
    G, K, dg = 4, 32, 6
    x = rng.standard_normal((50, G * dg)).astype(np.float32)
    cb = rng.standard_normal((G, K, dg)).astype(np.float32)
    codes = oracle.vq_encode(x, cb)
    for g in range(G):                      # contiguous slice g against codebook g only
        lib_codes, _ = scipy_vq(x[:, g * dg:(g + 1) * dg].astype(np.float64), cb[g].astype(np.float64))
        assert np.array_equal(codes[:, g], lib_codes)


def test_groups_are_independent():
    rng = np.random.default_rng(13)
    G, K, dg = 4, 16, 3
    x = rng.standard_normal((20, G * dg)).astype(np.float32)
    cb = rng.standard_normal((G, K, dg)).astype(np.float32)
    base = oracle.vq_encode(x, cb)
    x2 = x.copy()
    x2[:, dg:] = rng.standard_normal((20, (G - 1) * dg)).astype(np.float32)
    assert np.array_equal(oracle.vq_encode(x2, cb)[:, 0], base[:, 0])
    cb2 = cb.copy()
    cb2[1:] = rng.standard_normal((G - 1, K, dg)).astype(np.float32)
    assert np.array_equal(oracle.vq_encode(x, cb2)[:, 0], base[:, 0])


def test_permuting_codewords_permutes_codes():
    rng = np.random.default_rng(14)
    G, K, dg = 2, 32, 4
    x = rng.standard_normal((40, G * dg)).astype(np.float32)
    cb = rng.standard_normal((G, K, dg)).astype(np.float32)
    perm = rng.permutation(K)
    codes = oracle.vq_encode(x, cb)
    codes_p = oracle.vq_encode(x, cb[:, perm])     # new index j holds old codeword perm[j]
    assert np.array_equal(perm[codes_p], codes)


def test_larger_nested_codebook_never_increases_distortion():
    # C subset of C' => min over C' <= min over C, the monotonicity behind the high-rate bound.
    rng = np.random.default_rng(15)
    x = rng.standard_normal((64, 8)).astype(np.float32)
    big = rng.standard_normal((1, 128, 8)).astype(np.float32)
    prev = None
    for K in (4, 16, 64, 128):
        cb = big[:, :K]
        err = ((x - oracle.vq_decode(oracle.vq_encode(x, cb), cb)).astype(np.float64) ** 2).sum(axis=1)
        if prev is not None:
            assert np.all(err <= prev)
        prev = err


def test_decode_is_a_pure_gather():
    rng = np.random.default_rng(16)
    G, K, dg, T = 5, 11, 7, 33
    cb = rng.standard_normal((G, K, dg)).astype(np.float32)
    codes = rng.integers(0, K, size=(T, G)).astype(np.int32)
    expect = np.stack([cb[g, codes[:, g]] for g in range(G)], axis=1).reshape(T, G * dg)
    assert np.array_equal(oracle.vq_decode(codes, cb), expect)
    with pytest.raises(ValueError):
        oracle.vq_decode(np.full((1, G), K, dtype=np.int32), cb)


def test_empty_inputs():
    cb = np.ones((2, 4, 3), dtype=np.float32)
    assert oracle.vq_encode(np.zeros((0, 6), dtype=np.float32), cb).shape == (0, 2)
    assert oracle.vq_decode(np.zeros((0, 2), dtype=np.int32), cb).shape == (0, 6)
