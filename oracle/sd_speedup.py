"""Oracle (test infrastructure, not product code) for the paper's speculative-decoding
speed-up model: plain scalar Python in double precision, one function per formula, in the
paper's notation.  Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
import anything under oracle/.

What it follows:
  sigma(alpha, gamma)         Sec. 3.1, Eq. (sigma from alpha)
  G(t; lambda*RP, s)          Sec. 3.3, Eq. G(t)
  N(t), T_exp(t)              Sec. 3.2, Eq. N(t) and Eq. T_exp
  target forward time         Sec. 3.3 / Alg. 1, the ar_time and verify_time lines
  draft and rejection time    Alg. 1, the draft_time and reject_time lines
  speed-up                    Sec. 3.1, Eq. (speedup)

Readings taken where the paper disagrees with itself:
  * Alg. 1 prints the speed-up denominator as draft + ar + verify + reject; Eq. (speedup)
    has gamma * T_D + T_T(B, gamma) + T_reject.  The equation is derived in the text, the
    listing is not: the equation is followed.
  * Alg. 1 prices the verification forward at B*gamma tokens, the text counts a bonus token
    (gamma + 1 positions per request).  `bonus` selects the reading; the listing's (False) is
    the default here so that the listing can be reproduced, the layer benchmark uses True.
"""
from __future__ import annotations

import math


def sigma(alpha: float, gamma: int) -> float:
    """Expected generated tokens per round over the most a round can yield, gamma + 1."""
    if alpha == 1.0:
        return 1.0
    return ((1.0 - alpha ** (gamma + 1)) / (1.0 - alpha)) / (gamma + 1)


def G(t: float, knee: float, s: float) -> float:
    """s**t up to the knee (= lambda * RP), the tangent line at the knee after it."""
    if t <= knee:
        return s ** t
    return s ** knee * (1.0 + math.log(s) * (t - knee))


def n_active(E: int, K: int, t: float) -> float:
    return E * (1.0 - ((E - K) / E) ** t)


def t_exp(E: int, K: int, t: float) -> float:
    n = n_active(E, K, t)
    return t * K / n if n > 0.0 else 0.0


def target_time(bias, k1, k2, k3, lam, s, RP, E, K, t):
    """bias + k1*G(t) + k2*N(t) + k3*G(T_exp(t))."""
    knee = lam * RP
    return bias + k1 * G(t, knee, s) + k2 * n_active(E, K, t) + k3 * G(t_exp(E, K, t), knee, s)


def compute_speedup(params, B, gamma, K, E, sig, RP, bonus=False):
    """params = (bias, k1, k2, k3, draft_bias, draft_k, reject_bias, reject_k, lambda, s)."""
    bias, k1, k2, k3, draft_bias, draft_k, reject_bias, reject_k, lam, s = params
    ar_time = target_time(bias, k1, k2, k3, lam, s, RP, E, K, B)
    t_verify = B * (gamma + 1) if bonus else B * gamma
    verify_time = target_time(bias, k1, k2, k3, lam, s, RP, E, K, t_verify)
    draft_time = draft_bias + draft_k * G(B, lam * RP, s)
    reject_time = reject_bias + reject_k * B
    return sig * (gamma + 1) * ar_time / (gamma * draft_time + verify_time + reject_time)


def target_efficiency(params, B, gamma, K, E, RP, bonus=False):
    """T_T(B, 1) / T_T(B, gamma) (Sec. 3.1)."""
    bias, k1, k2, k3, _, _, _, _, lam, s = params
    t_verify = B * (gamma + 1) if bonus else B * gamma
    return (target_time(bias, k1, k2, k3, lam, s, RP, E, K, B) /
            target_time(bias, k1, k2, k3, lam, s, RP, E, K, t_verify))
