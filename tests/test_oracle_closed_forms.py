"""Pins for the oracle's closed forms (Sec. 3.2: Eq. N(t), Eq. T_thres, Eq. Texp;
Appendix B: monotonicity of Texp in rho).  None of these tests retypes the
formula: each checks it against enumeration, sampling, or a property the paper
states."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "enumerated_expectation.txt")


def _gold():
    rows = []
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            E, K, t, num, den = (int(v) for v in line.split())
            rows.append((E, K, t, Fraction(num, den)))
    return rows


def test_expected_active_matches_exact_enumeration(oracle):
    # exact expectation over every K-subset choice of every token (Sec. 3.2 model)
    for E, K, t, fr in _gold():
        got = oracle.expected_active_experts(E, K, t)
        assert abs(got - float(fr)) < 1e-12, (E, K, t, got, float(fr))


def test_expected_active_special_values(oracle):
    for E, K in [(8, 2), (60, 4), (64, 8), (256, 8), (7, 7), (5, 0)]:
        assert oracle.expected_active_experts(E, K, 0) == 0.0
        assert oracle.expected_active_experts(E, K, 1) == pytest.approx(K, abs=1e-12)  # one token: K
        big = oracle.expected_active_experts(E, K, 10**6)
        assert big == pytest.approx(E if K > 0 else 0.0, abs=1e-9)                    # saturates at E
        prev = -1.0
        for t in range(0, 200):
            v = oracle.expected_active_experts(E, K, t)
            assert v >= prev - 1e-15 and v <= E + 1e-12                               # monotone, bounded
            prev = v
    assert math.isnan(oracle.expected_active_experts(0, 0, 1))
    assert math.isnan(oracle.expected_active_experts(4, 5, 1))
    assert math.isnan(oracle.expected_active_experts(4, 2, -1))


@pytest.mark.parametrize("E,K,T", [(8, 2, 4), (60, 4, 16), (64, 8, 16), (256, 8, 64)])
def test_expected_active_vs_uniform_monte_carlo(oracle, E, K, T):
    """Uniform sampler (random K-subset per token) -> the oracle's permutation
    counts the activated experts; the mean must sit on the closed form."""
    rng = np.random.default_rng(1234 + E + T)
    R = 4000
    tot = 0.0
    sq = 0.0
    for _ in range(R):
        ids = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32)
        n = oracle.permute(E, K, ids)["n_active"]
        tot += n
        sq += n * n
    mean = tot / R
    sd = math.sqrt(max(sq / R - mean * mean, 1e-12))
    want = oracle.expected_active_experts(E, K, T)
    assert abs(mean - want) < 4.5 * sd / math.sqrt(R) + 1e-9, (mean, want, sd)


def test_token_threshold_defining_property(oracle):
    # T_thres is the first t with N(t) >= tau*E (Eq. T_thres)
    for E, K in [(8, 2), (60, 4), (64, 8), (256, 8), (16, 1), (62, 6)]:
        for tau in (0.5, 0.9, 0.95, 0.99):
            t = oracle.token_threshold(E, K, tau)
            assert t >= 1
            assert oracle.expected_active_experts(E, K, t) >= tau * E - 1e-12
            if t > 1:
                assert oracle.expected_active_experts(E, K, t - 1) < tau * E
            # the printed closed form: ceil(log_{1-rho}(1-tau))
            assert t == max(1, math.ceil(math.log(1 - tau) / math.log(1 - K / E) - 1e-12))
    assert oracle.token_threshold(8, 8, 0.95) == 1      # dense: one token activates all
    assert oracle.token_threshold(8, 0, 0.95) == -1
    assert oracle.token_threshold(8, 2, 1.0) == -1
    # the four benchmark shapes at tau = 0.95
    assert [oracle.token_threshold(E, K, 0.95) for E, K in [(8, 2), (60, 4), (64, 8), (256, 8)]] \
        == [11, 44, 23, 95]


def test_tokens_per_expert_properties(oracle):
    # Eq. Texp: Texp * N = t*K; one token -> 1; dense (rho = 1) -> t
    for E, K in [(8, 2), (60, 4), (64, 8), (256, 8)]:
        assert oracle.expected_tokens_per_expert(E, K, 1) == pytest.approx(1.0, abs=1e-12)
        for t in (2, 7, 64, 1000):
            te = oracle.expected_tokens_per_expert(E, K, t)
            assert te * oracle.expected_active_experts(E, K, t) == pytest.approx(t * K, rel=1e-12)
    for t in (1, 5, 300):
        assert oracle.expected_tokens_per_expert(16, 16, t) == pytest.approx(t, rel=1e-12)
    assert oracle.expected_tokens_per_expert(8, 2, 0) == 0.0


def test_tokens_per_expert_increases_with_rho(oracle):
    """Appendix B: for T > 1, Texp(T; rho) grows with rho, equivalently
    F(rho; T) = (1-rho)^(T-1) (rho T + 1 - rho) < 1 and F falls as rho grows."""
    E = 64
    for T in (2, 3, 8, 33, 257):
        prev = 0.0
        for K in range(1, E + 1):
            te = oracle.expected_tokens_per_expert(E, K, T)
            assert te > prev
            prev = te
        prev_f = 1.0
        for K in range(1, E):
            rho = K / E
            F = (1 - rho) ** (T - 1) * (rho * T + 1 - rho)
            assert F < 1.0 and (F < prev_f or prev_f < 1e-300)   # strict until it underflows
            prev_f = F
    # T = 1: flat in rho
    assert all(oracle.expected_tokens_per_expert(E, K, 1) == pytest.approx(1.0) for K in range(1, E + 1))
