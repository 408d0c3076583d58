"""Pins for the oracle's pre-clipping (BTARD-Clipped-SGD, App. E.3, Alg. 9: every peer
clips each partition of its gradient to radius lambda before BTARD) -- CPU only.

The scaled code paths of the oracle are checked against things they do not compute
themselves: numpy norms, the plain oracle on materialised rows where the products are
exact (power-of-two factors), the hand-worked case, and invariances.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle


def same(a, b, tol=1e-12):
    """Equal up to the order of the fp64 sums (the oracle's loops are OpenMP reductions)."""
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return a.shape == b.shape and np.abs(a - b).max(initial=0.0) <= tol * max(1.0, np.abs(b).max(initial=0.0))


def rng(seed):
    return np.random.default_rng(seed)


def case(seed, n=6, d=90, P=3, big=(1, 4)):
    G = rng(seed).standard_normal((n, d)).astype(np.float32)
    for i in big:
        G[i] *= np.float32(7.0)
    return G, [int(x) for x in oracle.split(d, P)]


def test_scales_are_min_one_lambda_over_norm():
    G, off = case(1)
    lam = 6.0
    alpha, norms = oracle.preclip_scales(G, off, lam)
    for j in range(len(off) - 1):
        ref = np.linalg.norm(G[:, off[j]:off[j + 1]].astype(np.float64), axis=1)
        np.testing.assert_allclose(norms[:, j], ref, rtol=1e-14)
        np.testing.assert_allclose(alpha[:, j], np.minimum(1.0, lam / ref), rtol=1e-14)
        clipped = alpha[:, j] * ref
        np.testing.assert_allclose(clipped, np.minimum(ref, lam), rtol=1e-14)
    assert (alpha <= 1.0).all() and (alpha[[1, 4]] < 1.0).all() and (alpha[[0, 2]] == 1.0).any()


def test_zero_rows_and_huge_lambda_are_left_alone():
    G, off = case(2)
    G[3] = 0.0
    alpha, norms = oracle.preclip_scales(G, off, 1e30)
    assert (alpha == 1.0).all()
    alpha, norms = oracle.preclip_scales(G, off, 0.5)
    assert (alpha[3] == 1.0).all() and (norms[3] == 0.0).all()
    # with all factors 1 the scaled entry points ARE the plain ones
    ones = np.ones_like(alpha)
    a = oracle.centered_clip(G, off, 1.0, 1e-6, 40, scale=ones)
    b = oracle.centered_clip(G, off, 1.0, 1e-6, 40)
    assert same(a[0], b[0]) and np.array_equal(a[1], b[1]) and same(a[2], b[2])
    va = oracle.verify(G, off, a[0], 1.0, 99, scale=ones, want_delta=True)
    vb = oracle.verify(G, off, a[0], 1.0, 99, want_delta=True)
    for k in ("norms", "weights", "proj", "colsum", "delta"):
        assert same(va[k], vb[k]), k


@pytest.mark.parametrize("seed", [3, 4])
def test_power_of_two_factors_equal_the_plain_oracle_on_materialised_rows(seed):
    """scale[i, j] * G[i, x] is exact in fp32 for power-of-two factors, so running on the
    factors must give what the plain oracle gives on the scaled copy (up to the order of
    the fp64 sums): a factor applied to the wrong row or the wrong partition fails this."""
    G, off = case(seed, n=5, d=64, P=4)
    P = len(off) - 1
    scale = 2.0 ** -rng(seed + 100).integers(0, 4, size=(5, P)).astype(np.float64)
    assert len(np.unique(scale)) > 2
    Gs = G.copy()
    for j in range(P):
        Gs[:, off[j]:off[j + 1]] *= scale[:, j:j + 1].astype(np.float32)
    a = oracle.centered_clip(G, off, 0.7, 1e-6, 60, scale=scale, want_trace=True)
    b = oracle.centered_clip(Gs, off, 0.7, 1e-6, 60, want_trace=True)
    assert same(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert same(a[2], b[2]) and same(a[3], b[3])
    v0 = rng(seed).standard_normal(64)
    a = oracle.centered_clip(G, off, 0.7, 0.0, 9, v0=v0, scale=scale)
    b = oracle.centered_clip(Gs, off, 0.7, 0.0, 9, v0=v0)
    assert same(a[0], b[0])
    va = oracle.verify(G, off, a[0], 0.7, 0xABCDEF, scale=scale, want_delta=True)
    vb = oracle.verify(Gs, off, a[0], 0.7, 0xABCDEF, want_delta=True)
    for k in ("norms", "weights", "proj", "colsum", "delta"):
        assert same(va[k], vb[k]), k


def test_hand_worked_case_reached_by_pre_clipping(golden_dir):
    """tests/golden/hand_n3_d8.txt with the third peer sending 20 u instead of 10 u and
    lambda = 10: its factor is exactly 1/2, the clipped rows are the hand case's rows, so
    iterations, v and the last step norm are the hand-derived ones."""
    rows, kv = [], {}
    for line in open(os.path.join(golden_dir, "hand_n3_d8.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *rest = line.split()
        if k == "g":
            rows.append([float(x) for x in rest])
        else:
            kv[k] = rest[0]
    G = np.array(rows, dtype=np.float32)
    G[2] *= np.float32(2.0)
    off = [0, 8]
    alpha, norms = oracle.preclip_scales(G, off, 10.0)
    assert alpha[:, 0].tolist() == [1.0, 1.0, 0.5] and norms[2, 0] == 20.0
    v, iters, sn, _ = oracle.centered_clip(G, off, float(kv["tau"]), float(kv["eps"]),
                                           int(kv["max_iters"]), scale=alpha)
    assert iters[0] == int(kv["iters"])
    t = float(Fraction(int(kv["t_final_num"]), int(kv["t_final_den"])))
    np.testing.assert_allclose(v, t * np.array([.5, .5, .5, .5, 0, 0, 0, 0]), rtol=0, atol=1e-15)
    np.testing.assert_allclose(sn[0], 1.0 / int(kv["last_step_norm_inv"]), rtol=1e-9)


def test_one_peer_returns_its_clipped_gradient():
    g = rng(5).standard_normal((1, 50)).astype(np.float32) * np.float32(4.0)
    off = [0, 20, 50]
    alpha, norms = oracle.preclip_scales(g, off, 3.0)
    v, iters, sn, _ = oracle.centered_clip(g, off, 1.0, 1e-6, 10, scale=alpha)
    assert iters.tolist() == [1, 1]
    for j in range(2):
        seg = g[0, off[j]:off[j + 1]].astype(np.float64)
        np.testing.assert_allclose(v[off[j]:off[j + 1]], seg * min(1.0, 3.0 / np.linalg.norm(seg)),
                                   rtol=1e-15)
        assert abs(np.linalg.norm(v[off[j]:off[j + 1]]) - min(3.0, norms[0, j])) < 1e-12


def test_growing_an_already_clipped_row_changes_nothing():
    """A row beyond the radius is projected onto the sphere: its length does not matter."""
    G, off = case(6)
    lam = 5.0
    alpha, _ = oracle.preclip_scales(G, off, lam)
    G2 = G.copy()
    G2[1] *= np.float32(4.0)                      # row 1 is clipped in every partition
    assert (alpha[1] < 1.0).all()
    alpha2, _ = oracle.preclip_scales(G2, off, lam)
    np.testing.assert_allclose(alpha2[1], alpha[1] / 4.0, rtol=1e-14)
    a = oracle.centered_clip(G, off, 1.0, 1e-6, 80, scale=alpha)
    b = oracle.centered_clip(G2, off, 1.0, 1e-6, 80, scale=alpha2)
    assert np.array_equal(a[1], b[1])
    np.testing.assert_allclose(a[0], b[0], rtol=0, atol=1e-13)
    # and the aggregate of the clipped rows stays within lambda of every clipped row's sphere
    for j in range(len(off) - 1):
        assert np.linalg.norm(a[0][off[j]:off[j + 1]]) <= lam + 1e-12


def test_verification_identity_holds_for_the_clipped_rows():
    """colsum_j = n <z[j], next CenteredClip step> (linearity of eq. (2)) on alpha * g."""
    G, off = case(7, n=7, d=120, P=3, big=(0, 5))
    n = G.shape[0]
    alpha, _ = oracle.preclip_scales(G, off, 4.0)
    tau, seed = 0.8, 424242
    v, iters, _, _ = oracle.centered_clip(G, off, tau, 0.0, 6, scale=alpha)
    out = oracle.verify(G, off, v, tau, seed, scale=alpha, want_delta=True)
    v_next, _, _, _ = oracle.centered_clip(G, off, tau, 0.0, 1, v0=v, scale=alpha)
    z = oracle.z_hat(seed, 0, off[-1]) / oracle.z_norm(seed, off[-1])
    for j in range(len(off) - 1):
        lo, hi = off[j], off[j + 1]
        assert abs(out["colsum"][j] - n * np.dot(z[lo:hi], (v_next - v)[lo:hi])) < 1e-12
        for i in range(n):
            r = alpha[i, j] * G[i, lo:hi].astype(np.float64) - v[lo:hi]
            assert abs(out["norms"][i, j] - np.linalg.norm(r)) < 1e-12
            np.testing.assert_allclose(out["delta"][i, lo:hi], out["weights"][i, j] * r, atol=1e-14)
