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


def test_verifications_1_and_2_on_an_honest_run_and_on_planted_lies():
    """The comparisons of Alg. 6 (Verification 1: broadcast norm vs recomputed; Verification 2:
    broadcast projection vs recomputed, and the column sums) on the oracle's own verification
    quantities at a CenteredClip fixed point: an honest broadcast raises no flag (the column
    sums vanish there, eq. (2)); a lie about one norm, one projection, or a wrong aggregate
    raises exactly the flags the algorithm describes."""
    rng = np.random.default_rng(12)
    n, d, P = 7, 240, 4
    G = rng.standard_normal((n, d)).astype(np.float32)
    G[5:] *= np.float32(9.0)
    off = [int(x) for x in oracle.split(d, P)]
    tau, seed = 1.5, 99
    v, iters, _, _ = oracle.centered_clip(G, off, tau, 1e-13, 20000)
    assert (iters < 20000).all()
    out = oracle.verify(G, off, v, tau, seed)
    norms, proj = out["norms"], out["proj"]
    rtol, atol = 1e-9, 1e-9
    bn, bp, bs = oracle.verification12(norms, proj, norms, proj, rtol, atol)
    assert not bn.any() and not bp.any() and not bs.any()
    # tolerance: a relative change below rtol passes, above it fails (checked by hand here)
    cn = norms.copy(); cn[2, 1] *= 1 + 5e-10; cn[3, 0] *= 1 + 5e-9
    # ... and a projection moved to between the two thresholds: beyond atol + rtol |s_42|
    # (it does not match) but within atol + rtol sum_i |s_i2| (the column still sums to zero)
    col = np.abs(proj[:, 2]).sum()
    assert col > 2 * abs(proj[4, 2])
    cp = proj.copy(); cp[4, 2] += atol + rtol * abs(proj[4, 2]) + 0.5 * rtol * (col - abs(proj[4, 2]))
    bn, bp, bs = oracle.verification12(cn, cp, norms, proj, rtol, atol)
    assert bn.sum() == 1 and bn[3, 0] == 1
    assert bp.sum() == 1 and bp[4, 2] == 1
    assert not bs.any()
    # a peer that misreports its projection by a visible amount breaks the sum of its column
    cp = proj.copy(); cp[1, 3] += 0.5
    bn, bp, bs = oracle.verification12(norms, cp, norms, proj, rtol, atol)
    assert bp.sum() == 1 and bp[1, 3] == 1 and bs.tolist() == [0, 0, 0, 1]
    # a wrong aggregate for partition 2: honest peers' recomputed projections no longer sum to 0
    v_bad = v.copy(); v_bad[off[2]:off[3]] += 0.05
    out_bad = oracle.verify(G, off, v_bad, tau, seed)
    bn, bp, bs = oracle.verification12(out_bad["norms"], out_bad["proj"], out_bad["norms"],
                                       out_bad["proj"], rtol, atol)
    assert not bn.any() and not bp.any() and bs.tolist() == [0, 0, 1, 0]
    # NaN never matches; zero tolerances demand equality
    cn = norms.copy(); cn[0, 0] = np.nan
    bn, _, _ = oracle.verification12(cn, proj, norms, proj, rtol, atol)
    assert bn[0, 0] == 1 and bn.sum() == 1
    bn, bp, bs = oracle.verification12(norms, proj, norms, proj, 0.0, 0.0)
    assert not bn.any() and not bp.any()
    ones = np.array([[1.0], [-1.0], [0.25], [-0.25]])
    assert oracle.verification12(ones, ones, ones, ones, 0.0, 0.0)[2].tolist() == [0]
    ones[3, 0] = -0.5
    assert oracle.verification12(ones, ones, ones, ones, 0.0, 0.0)[2].tolist() == [1]
    assert oracle.verification12(ones, ones, ones, ones, 0.2, 0.0)[2].tolist() == [0]   # 0.25 <= 0.2 * 2.75
