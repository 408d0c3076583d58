"""Pins for the fp64 oracle's Split and CenteredClip (CPU only).

Each test checks the oracle against something the paper or the mathematics
fixes independently of the oracle's own loops: closed forms, special cases,
a hand-worked example, an independent optimiser, invariants.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import optimize

import oracle


def rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------
# Split (App. D.1): first d mod n parts have ceil(d/n), the rest floor(d/n)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("d,parts", [(10, 3), (8, 8), (7, 8), (0, 4), (1, 1),
                                     (11173962, 16), (17683968, 64), (2 ** 28, 8),
                                     (1315758080, 16), (1000003, 7)])
def test_split_closed_form(d, parts):
    off = oracle.split(d, parts)
    sizes = np.diff(off)
    assert off[0] == 0 and off[-1] == d and len(off) == parts + 1
    r = d % parts
    assert (sizes[:r] == -(-d // parts)).all()
    assert (sizes[r:] == d // parts).all()


def test_split_resnet18_sizes():
    sizes = np.diff(oracle.split(11173962, 16))
    assert list(sizes) == [698373] * 10 + [698372] * 6


# --------------------------------------------------------------------------
# Hand-worked case (tests/golden/hand_n3_d8.txt)
# --------------------------------------------------------------------------
def _read_hand(golden_dir):
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
    return np.array(rows, dtype=np.float32), kv


def test_hand_worked_n3_d8(golden_dir):
    G, kv = _read_hand(golden_dir)
    assert G.shape == (int(kv["n"]), int(kv["d"]))
    v, iters, sn, trace = oracle.centered_clip(
        G, [0, G.shape[1]], float(kv["tau"]), float(kv["eps"]), int(kv["max_iters"]),
        want_trace=True)
    assert iters[0] == int(kv["iters"])
    t = Fraction(int(kv["t_final_num"]), int(kv["t_final_den"]))
    u = np.array([0.5] * 4 + [0.0] * 4)
    np.testing.assert_allclose(v, float(t) * u, rtol=0, atol=1e-14)
    assert sn[0] == pytest.approx(1.0 / int(kv["last_step_norm_inv"]), rel=1e-9)
    # trajectory of step norms: eight steps of 1/3, then (1/9) 3^-(m-1)
    expect = [1 / 3] * 8 + [(1 / 9) * 3.0 ** -(m - 1) for m in range(1, 13)]
    np.testing.assert_allclose(trace[0, :20], expect, rtol=1e-9)
    # verification quantities at the returned v
    out = oracle.verify(G, [0, 8], v, 1.0, seed=7, want_delta=True)
    tf = float(t)
    np.testing.assert_allclose(out["norms"][:, 0], [tf, tf, 10 - tf], rtol=1e-13)
    np.testing.assert_allclose(out["weights"][:, 0], [1, 1, 1 / (10 - tf)], rtol=1e-13)
    np.testing.assert_allclose(out["delta"].sum(axis=0), (1 - 2 * tf) * u, atol=1e-14)


# --------------------------------------------------------------------------
# Special cases with textbook answers
# --------------------------------------------------------------------------
def test_tau_infinite_is_the_mean():
    G = rng(1).normal(size=(7, 53)).astype(np.float32)
    off = oracle.split(53, 4)
    mean = G.astype(np.float64).mean(axis=0)
    for tau in (math.inf, 1e9):
        v, iters, sn, _ = oracle.centered_clip(G, off, tau, 1e-6, 50)
        np.testing.assert_allclose(v, mean, rtol=0, atol=1e-15)
        assert (iters == 1).all() and (sn < 1e-15).all()
    # from another starting point: one step lands on the mean, the second is zero
    v0 = rng(2).normal(size=53)
    v, iters, sn, trace = oracle.centered_clip(G, off, math.inf, 1e-6, 50, v0=v0,
                                               want_trace=True)
    np.testing.assert_allclose(v, mean, rtol=0, atol=1e-14)
    assert (iters == 2).all()
    for j in range(4):
        lo, hi = off[j], off[j + 1]
        assert trace[j, 0] == pytest.approx(np.linalg.norm(mean[lo:hi] - v0[lo:hi]), rel=1e-12)


def test_identical_peers_and_single_peer():
    g = rng(3).normal(size=40).astype(np.float32)
    G = np.tile(g, (5, 1))
    v, iters, sn, _ = oracle.centered_clip(G, [0, 13, 40], 0.01, 1e-6, 50)
    np.testing.assert_array_equal(v, g.astype(np.float64))
    assert (iters == 1).all() and (sn == 0).all()
    v, iters, _, _ = oracle.centered_clip(g[None, :], [0, 40], 0.5, 1e-6, 50)
    np.testing.assert_array_equal(v, g.astype(np.float64))
    assert iters[0] == 1


def test_zero_iterations_returns_v0():
    G = rng(4).normal(size=(4, 10)).astype(np.float32)
    v, iters, sn, _ = oracle.centered_clip(G, [0, 10], 1.0, 1e-6, 0)
    np.testing.assert_allclose(v, G.astype(np.float64).mean(axis=0), atol=1e-16)
    assert iters[0] == 0 and sn[0] == 0
    v0 = np.arange(10.0)
    v, _, _, _ = oracle.centered_clip(G, [0, 10], 1.0, 1e-6, 0, v0=v0)
    np.testing.assert_array_equal(v, v0)


def test_collinear_inputs_reduce_to_scalar_clamp_recursion():
    # g_i = c_i u, v0 = t0 u (|u| = 1): the iteration is t <- t + mean(clamp(c_i - t, +-tau))
    r = rng(5)
    u = np.zeros(16); u[3] = 0.6; u[11] = -0.8          # exact in fp32 after scaling below
    c = np.array([-4.0, -1.5, 0.25, 0.5, 2.0, 8.0, 64.0])
    G = (c[:, None] * u[None, :]).astype(np.float32)
    c = (G.astype(np.float64) @ u)                      # coefficients actually stored
    tau, eps, M = 0.75, 1e-9, 200
    t = c.mean()
    steps = 0
    while steps < M:
        s = np.clip(c - t, -tau, tau).mean()
        t += s
        steps += 1
        if abs(s) < eps:
            break
    v, iters, _, _ = oracle.centered_clip(G, [0, 16], tau, eps, M)
    assert iters[0] == steps
    np.testing.assert_allclose(v, t * u, atol=1e-12)
    del r


# --------------------------------------------------------------------------
# Fixed point == minimiser of the summed Huber potential (eq. (1) is its
# stationarity condition); found here with an independent optimiser
# --------------------------------------------------------------------------
def huber_potential(x, G, tau):
    r = np.linalg.norm(G - x[None, :], axis=1)
    return np.where(r <= tau, 0.5 * r * r, tau * r - 0.5 * tau * tau).sum()


@pytest.mark.parametrize("seed,tau", [(0, 0.5), (1, 1.0), (2, 3.0)])
def test_fixed_point_is_huber_minimiser(seed, tau):
    r = rng(seed)
    G = r.normal(size=(6, 3))
    G[4] = [15.0, -9.0, 4.0]          # two far outliers
    G[5] = [-20.0, 1.0, 30.0]
    G = G.astype(np.float32)
    Gd = G.astype(np.float64)
    v, iters, sn, _ = oracle.centered_clip(G, [0, 3], tau, 1e-13, 100000)
    assert 0 < iters[0] < 100000
    res = optimize.minimize(huber_potential, Gd.mean(axis=0), args=(Gd, tau),
                            method="Nelder-Mead",
                            options=dict(xatol=1e-10, fatol=1e-16, maxiter=20000))
    np.testing.assert_allclose(v, res.x, atol=2e-6)
    assert huber_potential(v, Gd, tau) <= res.fun + 1e-12
    # eq. (1): sum_i Delta_i = 0 at the fixed point
    out = oracle.verify(G, [0, 3], v, tau, seed=11, want_delta=True)
    assert np.linalg.norm(out["delta"].sum(axis=0)) < 1e-11


def test_potential_decreases_and_steps_are_bounded():
    # the update is a gradient step of length 1 on (1/n) * potential, which is 1-smooth
    r = rng(8)
    n, d, tau = 9, 24, 0.8
    G = r.normal(size=(n, d)).astype(np.float32)
    G[6:] *= -30.0
    Gd = G.astype(np.float64)
    prev = None
    vk = None
    for k in range(0, 12):
        v, iters, sn, trace = oracle.centered_clip(G, [0, d], tau, 0.0, k, want_trace=True)
        assert iters[0] == k
        pot = huber_potential(v, Gd, tau)
        if prev is not None:
            assert pot <= prev + 1e-12
            # restart consistency: one more step from the previous output
            v_again, _, _, _ = oracle.centered_clip(G, [0, d], tau, 0.0, 1, v0=vk)
            np.testing.assert_allclose(v, v_again, atol=1e-13)
            assert (trace[0, :k] <= tau * (1 + 1e-12)).all()
            assert np.linalg.norm(v - vk) == pytest.approx(trace[0, k - 1], rel=1e-9)
        prev, vk = pot, v


def test_byzantine_rows_move_one_step_by_at_most_tau_b_over_n():
    # each clipped residual has norm <= tau, so b rows change a step by <= 2 tau b / n
    r = rng(9)
    n, d, tau, b = 10, 30, 0.3, 3
    G = r.normal(size=(n, d)).astype(np.float32)
    v0 = r.normal(size=d)
    G2 = G.copy()
    G2[:b] = (1e4 * r.normal(size=(b, d))).astype(np.float32)
    v1, _, _, _ = oracle.centered_clip(G, [0, d], tau, 0.0, 1, v0=v0)
    v2, _, _, _ = oracle.centered_clip(G2, [0, d], tau, 0.0, 1, v0=v0)
    assert np.linalg.norm(v1 - v2) <= 2 * tau * b / n * (1 + 1e-12)
    assert np.linalg.norm(v2 - v0) <= tau * (1 + 1e-12)


# --------------------------------------------------------------------------
# Symmetries of eq. (CenteredClip)
# --------------------------------------------------------------------------
def test_equivariance_translation_rotation_permutation():
    r = rng(10)
    n, d, tau, M = 6, 12, 0.7, 9
    G = r.normal(size=(n, d)).astype(np.float32)
    G[5] *= 25
    v0 = r.normal(size=d)
    v, _, _, tr = oracle.centered_clip(G, [0, d], tau, 0.0, M, v0=v0, want_trace=True)
    # permutation of the peers
    perm = r.permutation(n)
    vp, _, _, _ = oracle.centered_clip(G[perm], [0, d], tau, 0.0, M, v0=v0)
    np.testing.assert_allclose(vp, v, atol=1e-13)
    # signed coordinate permutation: an orthogonal map that is exact in fp32
    cp = r.permutation(d)
    sg = r.choice([-1.0, 1.0], size=d)
    Gq = (G[:, cp] * sg[None, :]).astype(np.float32)
    vq, _, _, trq = oracle.centered_clip(Gq, [0, d], tau, 0.0, M, v0=v0[cp] * sg,
                                         want_trace=True)
    np.testing.assert_allclose(vq, v[cp] * sg, atol=1e-13)
    np.testing.assert_allclose(trq, tr, rtol=1e-11)
    # translation by a vector that is exact in fp32 arithmetic here
    G8 = np.round(G * 256) / 256
    G8 = G8.astype(np.float32)
    t = np.round(r.normal(size=d) * 4) / 4
    va, _, _, _ = oracle.centered_clip(G8, [0, d], tau, 0.0, M, v0=v0)
    vb, _, _, _ = oracle.centered_clip((G8 + t[None, :]).astype(np.float32), [0, d], tau,
                                       0.0, M, v0=v0 + t)
    np.testing.assert_allclose(vb, va + t, atol=1e-12)
    # scaling: (G, v0, tau) -> (2G, 2v0, 2tau) scales v by 2
    vs, _, _, _ = oracle.centered_clip(2 * G, [0, d], 2 * tau, 0.0, M, v0=2 * v0)
    np.testing.assert_allclose(vs, 2 * v, atol=1e-13)


def test_partitions_are_independent_and_ld_is_honoured():
    r = rng(11)
    n, d, ld = 5, 37, 45
    buf = r.normal(size=(n, ld)).astype(np.float32)
    G = buf[:, :d]                      # row stride ld > d
    off = [0, 9, 9, 30, 37]             # includes an empty partition
    v, iters, sn, _ = oracle.centered_clip(G, off, 0.4, 1e-6, 25)
    assert iters[1] in (0, 1)           # empty partition: nothing to iterate on
    for j in range(4):
        lo, hi = off[j], off[j + 1]
        if hi == lo:
            continue
        sub = np.ascontiguousarray(G[:, lo:hi])
        vj, itj, snj, _ = oracle.centered_clip(sub, [0, hi - lo], 0.4, 1e-6, 25)
        # equal up to the order of fp64 additions (the OpenMP chunks shift with lo)
        np.testing.assert_allclose(v[lo:hi], vj, rtol=0, atol=1e-14)
        assert iters[j] == itj[0] and sn[j] == pytest.approx(snj[0], rel=1e-9)


def test_one_step_matches_definition_in_numpy():
    # not a pin on its own (same formula), but guards the weights/denominator
    r = rng(12)
    n, d, tau = 8, 20, 1.1
    G = r.normal(size=(n, d)).astype(np.float32)
    Gd = G.astype(np.float64)
    v0 = r.normal(size=d)
    res = Gd - v0
    nr = np.linalg.norm(res, axis=1)
    w = np.minimum(1.0, tau / nr)
    expect = v0 + (w[:, None] * res).sum(axis=0) / n
    v, _, _, _ = oracle.centered_clip(G, [0, d], tau, 0.0, 1, v0=v0)
    np.testing.assert_allclose(v, expect, atol=1e-14)


def test_nonfinite_norm_is_flagged():
    G = np.ones((3, 6), dtype=np.float32)
    G[1, 2] = np.inf
    _, iters, _, _ = oracle.centered_clip(G, [0, 3, 6], 1.0, 1e-6, 5,
                                          v0=np.zeros(6))
    assert iters[0] == -1 and iters[1] > 0


def test_bad_arguments_raise():
    G = np.ones((2, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.centered_clip(G, [0, 5], 1.0, 1e-6, 5)
    with pytest.raises(ValueError):
        oracle.centered_clip(G, [0, 4], -1.0, 1e-6, 5)
