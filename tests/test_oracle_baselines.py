"""Pins for the oracle's baseline aggregators (Sec. 4.1: the coordinate-wise and geometric
medians) -- CPU only."""
import numpy as np
import pytest
from scipy import optimize

import oracle


def rng(seed):
    return np.random.default_rng(seed)


def objective(G, v):
    return np.linalg.norm(G.astype(np.float64) - v[None, :], axis=1).sum()


@pytest.mark.parametrize("seed,n,d", [(1, 5, 6), (2, 8, 3), (3, 16, 10)])
def test_geometric_median_minimises_the_sum_of_distances(seed, n, d):
    G = rng(seed).standard_normal((n, d)).astype(np.float32)
    G[-2:] *= np.float32(15.0)
    v, iters, sn = oracle.geometric_median(G, [0, d], 1e-12, 1e-12, 5000)
    assert 1 < iters[0] < 5000
    res = optimize.minimize(lambda x: objective(G, x), G.astype(np.float64).mean(axis=0),
                            method="BFGS", options={"gtol": 1e-10})
    assert objective(G, v) <= res.fun * (1 + 1e-10)
    np.testing.assert_allclose(v, res.x, atol=2e-5)
    # first-order condition away from the inputs: the unit vectors to the inputs cancel
    r = G.astype(np.float64) - v[None, :]
    assert np.linalg.norm((r / np.linalg.norm(r, axis=1, keepdims=True)).sum(axis=0)) < 1e-8


def test_geometric_median_special_cases():
    # collinear inputs, odd n: the median along the line
    u = rng(4).standard_normal(7); u /= np.linalg.norm(u)
    cs = np.array([-3.0, 0.25, 0.5, 2.0, 40.0])
    G = (cs[:, None] * u[None, :]).astype(np.float32)
    v, iters, sn = oracle.geometric_median(G, [0, 7], 1e-13, 1e-13, 100000)
    np.testing.assert_allclose(v, G[2].astype(np.float64), atol=1e-6)
    # an equilateral triangle: its centre; more than half the inputs at one point: that point
    tri = np.array([[1.0, 0.0], [-0.5, np.sqrt(3) / 2], [-0.5, -np.sqrt(3) / 2]], dtype=np.float32)
    v, _, _ = oracle.geometric_median(tri, [0, 2], 1e-12, 1e-14, 1000)
    np.testing.assert_allclose(v, [0.0, 0.0], atol=1e-7)
    pts = np.array([[2.0, 1.0]] * 3 + [[-5.0, 7.0], [9.0, 9.0]], dtype=np.float32)
    v, _, _ = oracle.geometric_median(pts, [0, 2], 1e-9, 1e-13, 100000)
    np.testing.assert_allclose(v, [2.0, 1.0], atol=1e-6)
    # n = 1 and identical inputs: one update that does not move
    v, iters, sn = oracle.geometric_median(pts[:1], [0, 2], 1e-9, 1e-9, 10)
    assert iters[0] == 1 and sn[0] == 0.0 and np.array_equal(v, [2.0, 1.0])


def test_geometric_median_descends_and_is_equivariant():
    G = rng(5).standard_normal((9, 12)).astype(np.float32)
    G[7:] += np.float32(30.0)
    off = [0, 5, 12]
    prev = None
    for M in range(0, 8):
        v, iters, _ = oracle.geometric_median(G, off, 1e-12, 0.0, M)
        f = sum(objective(G[:, off[j]:off[j + 1]], v[off[j]:off[j + 1]]) for j in range(2))
        assert prev is None or f <= prev + 1e-12         # Weiszfeld never increases the objective
        prev = f
    v, iters, sn = oracle.geometric_median(G, off, 1e-12, 1e-10, 2000)
    # partitions are independent problems
    for j in range(2):
        vj, itj, _ = oracle.geometric_median(np.ascontiguousarray(G[:, off[j]:off[j + 1]]),
                                             [0, off[j + 1] - off[j]], 1e-12, 1e-10, 2000)
        np.testing.assert_allclose(v[off[j]:off[j + 1]], vj, atol=1e-12)
        assert itj[0] == iters[j]
    # permutation of the inputs; translation by an exactly representable vector; scaling by 2
    perm = rng(6).permutation(9)
    vp, _, _ = oracle.geometric_median(G[perm], off, 1e-12, 1e-10, 2000)
    np.testing.assert_allclose(vp, v, atol=1e-9)
    v2, _, _ = oracle.geometric_median(G * np.float32(2.0), off, 2e-12, 2e-10, 2000)
    np.testing.assert_allclose(v2, 2.0 * v, atol=1e-9)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 7, 16, 33, 64])
def test_coordinate_median_is_numpy_median(n):
    G = rng(n).standard_normal((n, 257)).astype(np.float32)
    G[:, 5] = G[0, 5]                                   # ties
    if n > 2:
        G[1, :] = 1e30
        G[2, :] = -1e30
    np.testing.assert_array_equal(oracle.coordinate_median(G), np.median(G.astype(np.float64), axis=0))
    wide = np.zeros((n, 300), dtype=np.float32)
    wide[:, :257] = G
    np.testing.assert_array_equal(oracle.coordinate_median(wide[:, :257]),
                                  np.median(G.astype(np.float64), axis=0))
