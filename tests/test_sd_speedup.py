"""Pins for the speed-up model oracle (oracle/sd_speedup.py) and agreement of the package's
vectorised version with it.  CPU only."""
import math
from fractions import Fraction
from itertools import product

import numpy as np
import pytest

from oracle import sd_speedup as orc
from paper_2505_19645_amd import sdmodel


@pytest.mark.parametrize("gamma", [1, 2, 3, 5])
@pytest.mark.parametrize("alpha", [Fraction(0), Fraction(1, 3), Fraction(4, 5), Fraction(1)])
def test_sigma_against_enumeration_of_round_outcomes(alpha, gamma):
    # A round: draft tokens are accepted one after the other, each with probability alpha, up to the
    # first rejection; the verification forward always adds one more token (Sec. 3.1).  Enumerate every
    # accept/reject pattern exactly.
    expected = Fraction(0)
    for pattern in product([True, False], repeat=gamma):
        prob = Fraction(1)
        for ok in pattern:
            prob *= alpha if ok else (1 - alpha)
        accepted = 0
        for ok in pattern:
            if not ok:
                break
            accepted += 1
        expected += prob * (accepted + 1)
    assert orc.sigma(float(alpha), gamma) == pytest.approx(float(expected / (gamma + 1)), rel=1e-14)


def test_sigma_limits():
    assert orc.sigma(0.0, 4) == pytest.approx(1 / 5)
    assert orc.sigma(1.0, 4) == 1.0
    assert orc.sigma(1.0 - 1e-9, 4) == pytest.approx(1.0, abs=1e-8)
    # longer drafts waste more of their budget at a fixed acceptance rate
    assert orc.sigma(0.7, 2) > orc.sigma(0.7, 4)


@pytest.mark.parametrize("s,knee", [(1.05, 60.0), (1.5, 7.0), (2.0, 3.5)])
def test_G_is_exponential_then_its_tangent(s, knee):
    assert orc.G(0.0, knee, s) == 1.0
    assert orc.G(knee / 2, knee, s) == pytest.approx(s ** (knee / 2))
    h = 1e-6
    # value and first derivative continuous at the knee
    assert orc.G(knee + h, knee, s) == pytest.approx(orc.G(knee - h, knee, s), rel=1e-5)
    dl = (orc.G(knee, knee, s) - orc.G(knee - h, knee, s)) / h
    dr = (orc.G(knee + h, knee, s) - orc.G(knee, knee, s)) / h
    assert dl == pytest.approx(dr, rel=1e-4)
    assert dr == pytest.approx(math.log(s) * s ** knee, rel=1e-4)
    # straight line after the knee
    a, b, c = (orc.G(knee + x, knee, s) for x in (1.0, 2.0, 3.0))
    assert a + c == pytest.approx(2 * b, rel=1e-12)
    # convex before it
    a, b, c = (orc.G(x, knee, s) for x in (0.2 * knee, 0.4 * knee, 0.6 * knee))
    assert a + c > 2 * b


def test_speedup_worked_example_in_exact_arithmetic():
    # E=4, K=1, B=2, gamma=2, listing's reading (verification over B*gamma = 4 tokens), k1 = k3 = 0
    E, K, B, gamma = 4, 1, 2, 2
    n2 = 4 * (1 - Fraction(3, 4) ** 2)
    n4 = 4 * (1 - Fraction(3, 4) ** 4)
    assert orc.n_active(E, K, 2) == float(n2) and orc.n_active(E, K, 4) == float(n4)
    bias, k2, draft_bias, reject_bias, sig = Fraction(1), Fraction(2), Fraction(1, 2), Fraction(1, 4), Fraction(4, 5)
    ar = bias + k2 * n2
    verify = bias + k2 * n4
    want = sig * (gamma + 1) * ar / (gamma * draft_bias + verify + reject_bias)
    params = (1.0, 0.0, 2.0, 0.0, 0.5, 0.0, 0.25, 0.0, 0.5, 1.1)
    assert orc.compute_speedup(params, B, gamma, K, E, 0.8, RP=100.0) == pytest.approx(float(want), rel=1e-14)
    # with the bonus token the verification forward sees B*(gamma+1) = 6 tokens
    n6 = 4 * (1 - Fraction(3, 4) ** 6)
    want_b = sig * (gamma + 1) * ar / (gamma * draft_bias + bias + k2 * n6 + reject_bias)
    assert orc.compute_speedup(params, B, gamma, K, E, 0.8, RP=100.0, bonus=True) == pytest.approx(float(want_b), rel=1e-14)


def _random_params(rng):
    return (rng.uniform(1, 50), rng.uniform(0, 2), rng.uniform(0.5, 10), rng.uniform(0, 2), rng.uniform(0.1, 5),
            rng.uniform(0, 0.5), rng.uniform(0, 1), rng.uniform(0, 0.01), rng.uniform(0.2, 1.0), rng.uniform(1.001, 1.2))


def test_speedup_invariants():
    rng = np.random.default_rng(0)
    for _ in range(50):
        p = _random_params(rng)
        E = int(rng.integers(2, 65)); K = int(rng.integers(1, E + 1))
        B = int(rng.integers(1, 200)); gamma = int(rng.integers(1, 6)); sig = rng.uniform(0.2, 1.0)
        RP = rng.uniform(50, 400)
        sp = orc.compute_speedup(p, B, gamma, K, E, sig, RP)
        # Eq. (speedup) in its normalised form
        bias, k1, k2, k3, db, dk, rb, rk, lam, s = p
        tt1 = orc.target_time(bias, k1, k2, k3, lam, s, RP, E, K, B)
        ttg = orc.target_time(bias, k1, k2, k3, lam, s, RP, E, K, B * gamma)
        td = db + dk * orc.G(B, lam * RP, s)
        tr = rb + rk * B
        assert sp == pytest.approx(sig * (gamma + 1) / (gamma * td / tt1 + ttg / tt1 + tr / tt1), rel=1e-12)
        # a speed-up is a ratio of times: the unit of time cancels
        c = 7.5
        scaled = tuple(v * c for v in p[:8]) + p[8:]
        assert orc.compute_speedup(scaled, B, gamma, K, E, sig, RP) == pytest.approx(sp, rel=1e-12)
        # never above what perfect target efficiency and a free draft model would give
        assert sp <= sig * (gamma + 1) * tt1 / ttg + 1e-12
        # a slower draft model can only hurt
        slower = p[:4] + (p[4] * 2,) + p[5:]
        assert orc.compute_speedup(slower, B, gamma, K, E, sig, RP) < sp
        # target efficiency is the forward-time ratio
        assert orc.target_efficiency(p, B, gamma, K, E, RP) == pytest.approx(tt1 / ttg, rel=1e-12)


def test_dense_limit_has_constant_expert_term():
    # K = E: every expert is active from the first token on, T_exp = t
    for t in (1, 5, 40):
        assert orc.n_active(8, 8, t) == 8.0
        assert orc.t_exp(8, 8, t) == pytest.approx(t)


def test_package_agrees_with_oracle():
    rng = np.random.default_rng(1)
    for bonus in (False, True):
        for _ in range(20):
            p = _random_params(rng)
            E = int(rng.integers(2, 257)); K = int(rng.integers(1, min(E, 32) + 1))
            RP = rng.uniform(50, 400)
            B = rng.integers(1, 300, size=12); gamma = rng.integers(1, 6, size=12); sig = rng.uniform(0.2, 1.0, size=12)
            got = sdmodel.compute_speedup(np.array(p), B, gamma, K, E, sig, RP, bonus=bonus)
            eff = sdmodel.target_efficiency(np.array(p), B, gamma, K, E, RP, bonus=bonus)
            for i in range(12):
                want = orc.compute_speedup(p, int(B[i]), int(gamma[i]), K, E, float(sig[i]), RP, bonus=bonus)
                assert got[i] == pytest.approx(want, rel=1e-12)
                assert eff[i] == pytest.approx(orc.target_efficiency(p, int(B[i]), int(gamma[i]), K, E, RP, bonus=bonus),
                                               rel=1e-12)
    for a, g in ((0.0, 3), (0.8, 4), (1.0, 2)):
        assert float(sdmodel.sigma_from_alpha(a, g)) == pytest.approx(orc.sigma(a, g), rel=1e-14)


def test_fit_reproduces_speedups_generated_by_the_oracle():
    # measurements made by the oracle with known parameters; the fit must reproduce them (the parameters
    # themselves are not identifiable: a speed-up is invariant to the unit of time)
    E, K, RP = 64, 8, 300.0
    truth = (12.0, 0.4, 3.0, 0.6, 1.5, 0.05, 0.2, 0.001, 0.45, 1.02)
    Bs = [1, 2, 4, 8, 12, 16, 24, 32, 48, 64, 80, 100]
    rows = [(B, g) for g in (2, 4) for B in Bs]
    sig = [orc.sigma(0.8, g) for _, g in rows]
    sp = [orc.compute_speedup(truth, B, g, K, E, s, RP, bonus=True) for (B, g), s in zip(rows, sig)]
    fit = sdmodel.fit_speedup([r[0] for r in rows], [r[1] for r in rows], K, E, sig, sp, RP,
                              bias_min=6.0, k2_min=2.0, draft_bias_min=1.0, t_rej_max=1.0)
    assert fit["max_rel_err"] < 2e-2 and fit["mean_rel_err"] < 5e-3
    for name, lo, hi in (("lambda", 0.2, 1.0), ("s", 1.0, 2.0), ("bias", 6.0, 30.0), ("k2", 2.0, 10.0)):
        assert lo - 1e-9 <= fit["params"][name] <= hi + 1e-9


def test_layer_speedups_from_curve():
    t = {1: 40.0, 2: 55.0, 4: 70.0, 8: 100.0, 16: 150.0}
    rows = sdmodel.layer_speedups_from_curve(t, gammas=(1, 3), alpha=0.8, draft_ratio=0.1, reject_ratio=0.0)
    keyed = {(r["B"], r["gamma"]): r for r in rows}
    assert set(keyed) == {(1, 1), (2, 1), (4, 1), (8, 1), (1, 3), (2, 3), (4, 3)}
    r = keyed[(2, 3)]
    sg = orc.sigma(0.8, 3)
    assert r["speedup"] == pytest.approx(sg * 4 * 55.0 / (3 * 5.5 + 100.0))
    assert r["target_efficiency"] == pytest.approx(55.0 / 100.0)
