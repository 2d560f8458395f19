"""Pins for the oracle's training-side VQ operations (Sec. 3.2: K-means initialisation, EMA updates, the commitment
term of Eq. 2; Sec. 3.3: NAVQ).  Pinned to scikit-learn's Lloyd iteration and inertia, to numpy / torch library routines
(bincount, index_add, Cholesky sampling), to closed forms and to invariants."""
import numpy as np
import pytest
import torch

import oracle


def data(rng, T=200, G=3, K=7, dg=5):
    x = rng.standard_normal((T, G * dg)).astype(np.float32)
    cb = rng.standard_normal((G, K, dg)).astype(np.float32)
    return x, cb


def test_stats_equal_library_reductions():
    rng = np.random.default_rng(80)
    x, cb = data(rng)
    codes = oracle.vq_encode(x, cb)
    counts, sums, sqerr = oracle.codebook_stats(x, codes, cb)
    G, K, dg = cb.shape
    for g in range(G):
        np.testing.assert_array_equal(counts[g], np.bincount(codes[:, g], minlength=K))
        ref = torch.zeros(K, dg, dtype=torch.float64).index_add_(0, torch.from_numpy(codes[:, g].astype(np.int64)),
                                                                 torch.from_numpy(x[:, g * dg:(g + 1) * dg].astype(np.float64)))
        np.testing.assert_allclose(sums[g], ref.numpy(), rtol=1e-13, atol=1e-13)
    # the commitment term written out: || X - X-hat ||_2^2 over all elements
    xh = oracle.vq_decode(codes, cb)
    np.testing.assert_allclose(sqerr.sum(), np.sum((x.astype(np.float64) - xh) ** 2), rtol=1e-13)
    # invariants: every token is counted once per group; the sums add up to the column sums of x
    assert np.all(counts.sum(1) == x.shape[0])
    np.testing.assert_allclose(sums.sum(1).reshape(-1), x.astype(np.float64).sum(0), rtol=1e-12, atol=1e-12)


def test_kmeans_step_equals_scikit_learn_lloyd_iteration():
    """gamma = 0: encode + statistics + update is one Lloyd iteration; scikit-learn's KMeans started from the same
    centroids and stopped after one iteration gives the same centroids and (evaluated on the start centroids) the same
    inertia as the commitment sum.  One group (G = 1) is plain K-means; each group of a grouped VQ is its own instance."""
    from sklearn.cluster import KMeans
    rng = np.random.default_rng(81)
    x, cb = data(rng, T=300, G=2, K=6, dg=4)
    pick = rng.choice(300, 6, replace=False)                # start from data points: no cluster starts empty
    cb = np.ascontiguousarray(x[pick].reshape(6, 2, 4).transpose(1, 0, 2))
    codes = oracle.vq_encode(x, cb)
    counts, sums, sqerr = oracle.codebook_stats(x, codes, cb)
    new = oracle.codebook_update(counts, sums, cb)
    for g in range(2):
        xs = x[:, g * 4:(g + 1) * 4].astype(np.float64)
        km = KMeans(n_clusters=6, init=cb[g].astype(np.float64), n_init=1, max_iter=1, algorithm="lloyd", tol=0.0).fit(xs)
        assert np.all(counts[g] > 0)
        np.testing.assert_allclose(new[g], km.cluster_centers_, rtol=1e-10, atol=1e-10)
        d = ((xs[:, None, :] - cb[g].astype(np.float64)[None]) ** 2).sum(-1)
        np.testing.assert_allclose(sqerr[g], d.min(1).sum(), rtol=1e-12)
    # Lloyd's monotonicity: re-assigning to the new centroids cannot raise the objective
    codes2 = oracle.vq_encode(x, new.astype(np.float32))
    _, _, sq2 = oracle.codebook_stats(x, codes2, new.astype(np.float32))
    assert sq2.sum() <= sqerr.sum() + 1e-9


def test_update_special_cases():
    rng = np.random.default_rng(82)
    x, cb = data(rng, T=50, G=2, K=9, dg=3)
    codes = oracle.vq_encode(x, cb)
    codes[codes == 4] = 5                                   # make cluster 4 empty in both groups
    counts, sums, _ = oracle.codebook_stats(x, codes, cb)
    assert np.all(counts[:, 4] == 0)
    new = oracle.codebook_update(counts, sums, cb)
    np.testing.assert_array_equal(new[:, 4], cb[:, 4].astype(np.float64))        # an empty cluster keeps its codeword
    # EMA: closed form after one step from given running statistics, and gamma -> weights (1 - gamma)
    n0 = rng.random((2, 9)) * 10
    m0 = rng.standard_normal((2, 9, 3))
    n, m = n0.copy(), m0.copy()
    g = 0.9
    ema = oracle.codebook_update(counts, sums, cb, gamma=g, ema_n=n, ema_m=m)
    np.testing.assert_allclose(n, g * n0 + (1 - g) * counts, rtol=1e-15)
    np.testing.assert_allclose(m, g * m0 + (1 - g) * sums, rtol=1e-15, atol=1e-15)
    np.testing.assert_allclose(ema, m / n[..., None], rtol=1e-14)
    # running statistics that already equal the batch statistics are a fixed point, and then EMA = K-means centroids
    keep = counts > 0
    n, m = counts.astype(np.float64), sums.copy()
    ema = oracle.codebook_update(counts, sums, cb, gamma=0.5, ema_n=n, ema_m=m)
    np.testing.assert_allclose(ema[keep], new[keep], rtol=1e-14)
    with pytest.raises(ValueError):
        oracle.codebook_update(counts, sums, cb, gamma=1.0, ema_n=n, ema_m=m)


def test_navq_equals_cholesky_sampling_and_reproduces_the_residual_moments():
    """x_tilde - x_hat = lam * xi with xi = mu + L z: compared with torch's matmul on the same draws; over many draws the
    noise has the mean and covariance of the residuals it was fitted to (the statement NAVQ is built on)."""
    rng = np.random.default_rng(83)
    T, G, K, dg = 4000, 2, 8, 3
    D = G * dg
    x, cb = data(rng, T=T, G=G, K=K, dg=dg)
    codes = oracle.vq_encode(x, cb)
    eps = x.astype(np.float64) - oracle.vq_decode(codes, cb)
    mu = eps.mean(0)
    sigma = np.cov(eps.T, bias=True)
    L = np.linalg.cholesky(sigma)
    z = rng.standard_normal((T, D)).astype(np.float32)
    lam = 0.7
    out = oracle.navq(codes, cb, mu.astype(np.float32), L.astype(np.float32), z, lam)
    xi = torch.from_numpy(mu.astype(np.float32).astype(np.float64)) + torch.from_numpy(z.astype(np.float64)) @ torch.from_numpy(
        L.astype(np.float32).astype(np.float64)).T
    np.testing.assert_allclose(out, oracle.vq_decode(codes, cb) + lam * xi.numpy(), rtol=1e-12, atol=1e-12)
    noise = (out - oracle.vq_decode(codes, cb)) / lam
    np.testing.assert_allclose(noise.mean(0), mu, atol=5 * np.sqrt(np.diag(sigma) / T).max())
    np.testing.assert_allclose(np.cov(noise.T, bias=True), sigma, atol=0.08 * np.abs(sigma).max())
    # lam = 0 is the deterministic inference path
    np.testing.assert_array_equal(oracle.navq(codes, cb, mu.astype(np.float32), L.astype(np.float32), z, 0.0), oracle.vq_decode(codes, cb))
