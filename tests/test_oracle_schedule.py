"""Pins for the oracle's tau_l schedule (App. D.2, eq. (5)), CenteredClip with per-iteration
radii, and Verification 3 of Alg. 6 -- CPU only."""
import math

import numpy as np
import pytest

import oracle


def rng(seed):
    return np.random.default_rng(seed)


@pytest.mark.parametrize("delta,sigma,B0", [(0.1, 1.0, 10.0), (0.05, 0.3, 0.0), (0.15, 2.0, 1.0)])
def test_schedule_closed_form(delta, sigma, B0):
    """B_l^2 is a linear recurrence: B_l^2 = (B_0^2 - B*) q^l + B*, q = 6.45 delta,
    B* = 5 sigma^2 / (1 - q); tau_l follows from it by the formula of eq. (5)."""
    L = 40
    tau, b2 = oracle.tau_schedule(delta, sigma, B0, L)
    q = 6.45 * delta
    bstar = 5.0 * sigma ** 2 / (1.0 - q)
    ls = np.arange(L)
    ref_b2 = (B0 ** 2 - bstar) * q ** ls + bstar
    np.testing.assert_allclose(b2, ref_b2, rtol=1e-12)
    ref_tau = 4.0 * np.sqrt((1 - delta) * (ref_b2 / 3 + sigma ** 2) / (math.sqrt(3) * delta))
    np.testing.assert_allclose(tau, ref_tau, rtol=1e-12)
    # contraction (q < 1): the radii converge monotonically to the stationary one
    assert (np.diff(np.abs(tau - tau[-1])) <= 1e-12).all()


def test_schedule_is_constant_at_the_stationary_point():
    delta, sigma = 0.1, 0.7
    bstar = 5.0 * sigma ** 2 / (1.0 - 6.45 * delta)
    tau, b2 = oracle.tau_schedule(delta, sigma, math.sqrt(bstar), 25)
    np.testing.assert_allclose(b2, bstar, rtol=1e-12)
    np.testing.assert_allclose(tau, tau[0], rtol=1e-12)
    with pytest.raises(ValueError):
        oracle.tau_schedule(0.0, 1.0, 1.0, 3)
    with pytest.raises(ValueError):
        oracle.tau_schedule(0.1, -1.0, 1.0, 3)


def test_constant_radii_equal_the_constant_tau_run():
    G = rng(1).standard_normal((7, 60)).astype(np.float32)
    G[5:] *= np.float32(9.0)
    off = [0, 25, 60]
    a = oracle.centered_clip(G, off, 0.8, 1e-6, 30, tau_l=[0.8] * 30, want_trace=True)
    b = oracle.centered_clip(G, off, 0.8, 1e-6, 30, want_trace=True)
    assert np.array_equal(a[1], b[1])
    np.testing.assert_allclose(a[0], b[0], rtol=0, atol=1e-13)
    np.testing.assert_allclose(a[3], b[3], rtol=1e-12)


def test_collinear_inputs_follow_the_scalar_recursion_with_varying_clamp():
    """g_i = c_i u, v0 on the line: t <- t + (1/n) sum_i clamp(c_i - t, -tau_l, tau_l)."""
    d = 12
    u = rng(2).standard_normal(d)
    u /= np.linalg.norm(u)
    cs = np.array([0.0, 0.5, -0.25, 8.0, -6.0])
    G = (cs[:, None] * u[None, :]).astype(np.float32)
    uf = G[3].astype(np.float64) / 8.0                       # the direction as fp32 holds it
    cs_f = np.array([np.dot(G[i].astype(np.float64), uf) / np.dot(uf, uf) for i in range(5)])
    taus = [3.0, 0.1, 2.0, 0.05, 1.0, 0.7, 0.3, 5.0]
    v, iters, sn, trace = oracle.centered_clip(G, [0, d], 1.0, 0.0, len(taus), tau_l=taus,
                                               want_trace=True)
    nu = np.linalg.norm(uf)
    t = cs_f.mean()
    for l, tau in enumerate(taus):
        step = np.mean(np.clip((cs_f - t) * nu, -tau, tau)) / nu
        t += step
        assert abs(trace[0][l] - abs(step) * nu) < 1e-9
    np.testing.assert_allclose(v, t * uf, atol=1e-7)
    assert iters[0] == len(taus)


def test_huge_first_radius_is_the_mean_step():
    G = rng(3).standard_normal((6, 40)).astype(np.float32)
    v, iters, sn, _ = oracle.centered_clip(G, [0, 40], 1e-3, 1e-9, 5, tau_l=[1e30] * 5)
    assert iters[0] == 1 and sn[0] < 1e-12                   # all weights 1: the step from the mean is 0
    np.testing.assert_allclose(v, G.astype(np.float64).mean(axis=0), atol=1e-14)
    with pytest.raises(ValueError):
        oracle.centered_clip(G, [0, 40], 1.0, 1e-6, 3, tau_l=[1.0, 0.0, 1.0])


def test_verification3_counts_and_strict_majority():
    norms = np.array([[1.0, 5.0, 2.0, 9.0],
                      [3.0, 0.0, 2.0, 9.0],
                      [4.0, 6.0, 2.0, 9.0],
                      [0.5, 7.0, 2.5, 9.0]])
    check, votes, trigger = oracle.verification3(norms, 2.0)
    assert np.array_equal(check, (norms > 2.0).astype(np.uint8))
    assert votes.tolist() == [2, 3, 1, 4]
    # n = 4: CheckAveraging needs MORE than n/2 = 2 votes
    assert trigger.tolist() == [0, 1, 0, 1]
    check, votes, trigger = oracle.verification3(norms[:3], 2.0)     # n = 3: 2 votes suffice
    assert votes.tolist() == [2, 2, 0, 3] and trigger.tolist() == [1, 1, 0, 1]
    r = rng(4).random((9, 6)) * 3
    check, votes, trigger = oracle.verification3(r, 1.5)
    assert np.array_equal(votes, (r > 1.5).sum(axis=0)) and np.array_equal(trigger, votes * 2 > 9)
