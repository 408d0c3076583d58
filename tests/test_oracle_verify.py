"""Pins for the oracle's random direction z and verification quantities (CPU only)."""
import math
import os

import numpy as np
import pytest
from scipy import stats

import oracle


def rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------
# z-spec: Philox4x32-10 -> uniforms on the 2^-23 grid -> Box-Muller -> unit vector
# --------------------------------------------------------------------------
def test_philox_known_answers(golden_dir):
    rows = 0
    for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        assert oracle.philox4x32_10(w[0:4], w[4:6]) == w[6:10]
        rows += 1
    assert rows == 3


def test_uniforms_lie_on_the_open_23_bit_grid_and_follow_the_counter_layout():
    seed = 0x0123456789ABCDEF
    ab = oracle.z_uniforms(seed, 0, 4096)
    k = ab * 2 ** 23 - 0.5
    assert (k == np.round(k)).all() and (ab > 0).all() and (ab < 1).all()
    assert (ab.astype(np.float32).astype(np.float64) == ab).all()      # exact in fp32 too
    # coordinate x uses word x mod 4 of Philox(counter = floor(x/4), key = seed halves)
    for x in (0, 1, 2, 3, 4, 4093, 4095):
        words = oracle.philox4x32_10([x // 4, 0, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        assert ab[x] == ((words[x % 4] >> 9) + 0.5) / 2 ** 23
    # high half of the counter is used beyond 2^34 coordinates
    x = 4 * (2 ** 32 + 5) + 2
    words = oracle.philox4x32_10([5, 1, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
    assert oracle.z_uniforms(seed, x, 1)[0] == ((words[2] >> 9) + 0.5) / 2 ** 23
    # windows agree with each other
    np.testing.assert_array_equal(oracle.z_uniforms(seed, 1001, 50), ab[1001:1051])


def test_box_muller_can_be_inverted_back_to_the_uniforms():
    seed = 99
    zh = oracle.z_hat(seed, 0, 4000)
    ab = oracle.z_uniforms(seed, 0, 4000)
    a = ab[0::2]           # radius uniform of each pair (words 0 and 2)
    b = ab[1::2]           # angle uniform (words 1 and 3)
    c, s = zh[0::2], zh[1::2]
    np.testing.assert_allclose(np.exp(-0.5 * (c * c + s * s)), a, rtol=1e-12)
    ang = np.mod(np.arctan2(s, c) / (2 * math.pi), 1.0)
    np.testing.assert_allclose(ang, b, atol=1e-12)
    # windows: any start, any length
    np.testing.assert_array_equal(oracle.z_hat(seed, 777, 123), zh[777:900])


def test_z_is_a_unit_vector_and_gaussian_before_normalisation():
    seed, d = 20210611, 1_000_003
    zh = oracle.z_hat(seed, 0, d)
    Z = oracle.z_norm(seed, d)
    assert Z == pytest.approx(np.linalg.norm(zh), rel=1e-13)
    assert np.linalg.norm(zh / Z) == pytest.approx(1.0, abs=1e-13)
    assert abs(zh.mean()) < 4 / math.sqrt(d)
    assert abs(zh.var() - 1) < 4 * math.sqrt(2 / d)
    assert stats.kstest(zh, "norm").pvalue > 1e-3
    # neighbouring coordinates (sin/cos of one pair, the two pairs of a block) uncorrelated
    for lag in (1, 2, 3, 4):
        assert abs(np.corrcoef(zh[:-lag], zh[lag:])[0, 1]) < 5 / math.sqrt(d)
    # different seeds give different directions
    z2 = oracle.z_hat(seed + 1, 0, 4096)
    assert abs(np.corrcoef(zh[:4096], z2)[0, 1]) < 0.1


# --------------------------------------------------------------------------
# norms, weights, Delta, s (Alg. 6 lines 8-12; eq. (2))
# --------------------------------------------------------------------------
def _case(seed, n=7, d=61, P=4):
    r = rng(seed)
    G = r.normal(size=(n, d)).astype(np.float32)
    G[n - 2:] *= 12
    v = r.normal(size=d) * 0.3
    off = oracle.split(d, P)
    return G, v, off


def test_verify_against_numpy_linear_algebra():
    G, v, off = _case(1)
    n, d = G.shape
    tau, seed = 4.0, 424242
    seen = set()
    out = oracle.verify(G, off, v, tau, seed, want_delta=True)
    z = oracle.z_hat(seed, 0, d) / oracle.z_norm(seed, d)
    R = G.astype(np.float64) - v[None, :]
    for j in range(len(off) - 1):
        lo, hi = off[j], off[j + 1]
        nr = np.linalg.norm(R[:, lo:hi], axis=1)
        np.testing.assert_allclose(out["norms"][:, j], nr, rtol=1e-13)
        clipped = nr > tau
        seen.update(clipped.tolist())
        np.testing.assert_allclose(out["weights"][:, j], np.where(clipped, tau / nr, 1.0),
                                   rtol=1e-13)
        D = out["delta"][:, lo:hi]
        # Delta keeps the direction of the residual, with norm min(norm, tau)
        np.testing.assert_allclose(np.linalg.norm(D, axis=1), np.minimum(nr, tau), rtol=1e-12)
        cosang = (D * R[:, lo:hi]).sum(axis=1) / (np.linalg.norm(D, axis=1) * nr)
        np.testing.assert_allclose(cosang, 1.0, rtol=1e-12)
        # s_i^j = <z[j], Delta_i^j>, from the materialised Delta and z
        np.testing.assert_allclose(out["proj"][:, j], D @ z[lo:hi], rtol=1e-10, atol=1e-14)
        assert out["colsum"][j] == pytest.approx(out["proj"][:, j].sum(), rel=1e-12)
    assert seen == {True, False}          # both branches of the min were exercised


def test_column_sum_equals_n_times_projection_of_the_next_step():
    # linearity of eq. (2) in Delta and eq. (CenteredClip): sum_i s_i^j = n <z[j], step(v)[j]>
    G, v, off = _case(2, n=9, d=83, P=5)
    n, d = G.shape
    tau, seed = 1.3, 5
    out = oracle.verify(G, off, v, tau, seed)
    v1, _, _, _ = oracle.centered_clip(G, off, tau, 0.0, 1, v0=v)
    z = oracle.z_hat(seed, 0, d) / oracle.z_norm(seed, d)
    for j in range(5):
        lo, hi = off[j], off[j + 1]
        assert out["colsum"][j] == pytest.approx(n * z[lo:hi] @ (v1 - v)[lo:hi], rel=1e-10)


def test_column_sum_vanishes_at_the_fixed_point():
    G, _, off = _case(3, n=8, d=40, P=2)
    tau = 1.0
    v, iters, _, _ = oracle.centered_clip(G, off, tau, 1e-13, 100000)
    assert (iters < 100000).all()
    out = oracle.verify(G, off, v, tau, seed=17)
    assert np.abs(out["colsum"]).max() < 1e-11
    assert np.abs(out["proj"]).max() > 1e-3            # the terms themselves are not small
    # a tampered aggregate is caught by the same test (Verification 2)
    bad = v.copy(); bad[3] += 1e-3
    assert np.abs(oracle.verify(G, off, bad, tau, seed=17)["colsum"]).max() > 1e-6


def test_tau_infinite_projection_is_plain_inner_product():
    G, v, off = _case(4)
    n, d = G.shape
    seed = 31337
    out = oracle.verify(G, off, v, math.inf, seed)
    z = oracle.z_hat(seed, 0, d) / oracle.z_norm(seed, d)
    R = G.astype(np.float64) - v[None, :]
    mean = G.astype(np.float64).mean(axis=0)
    for j in range(len(off) - 1):
        lo, hi = off[j], off[j + 1]
        np.testing.assert_allclose(out["proj"][:, j], R[:, lo:hi] @ z[lo:hi], rtol=1e-10,
                                   atol=1e-14)
        assert out["colsum"][j] == pytest.approx(n * (mean - v)[lo:hi] @ z[lo:hi], rel=1e-9,
                                                 abs=1e-13)
    assert (out["weights"] == 1).all()


def test_partition_can_be_verified_on_its_own_with_x_base():
    G, v, off = _case(5, n=6, d=90, P=4)
    tau, seed = 0.9, 8
    full = oracle.verify(G, off, v, tau, seed, want_delta=True)
    Z = oracle.z_norm(seed, 90)
    for j in range(4):
        lo, hi = int(off[j]), int(off[j + 1])
        sub = np.ascontiguousarray(G[:, lo:hi])
        part = oracle.verify(sub, [0, hi - lo], v[lo:hi], tau, seed, x_base=lo, znorm=Z)
        np.testing.assert_allclose(part["proj"][:, 0], full["proj"][:, j], rtol=1e-12)
        np.testing.assert_allclose(part["norms"][:, 0], full["norms"][:, j], rtol=1e-13)
        assert part["colsum"][0] == pytest.approx(full["colsum"][j], rel=1e-10, abs=1e-15)
