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


PARAM_NAMES = ("bias", "k1", "k2", "k3", "draft_bias", "draft_k", "reject_bias", "reject_k", "lam", "s")


def _named(params):
    """The ten fitted parameters by name (accepts a mapping or a sequence in PARAM_NAMES order)."""
    return dict(params) if hasattr(params, "keys") else dict(zip(PARAM_NAMES, params))


def target_time(bias, k1, k2, k3, lam, s, RP, E, K, t):
    """T_T over t tokens, Sec. 3.3: a fixed part, a dense part that follows the roofline in t, the
    loading of the N(t) activated experts, and the expert computation that follows the roofline in
    the per-expert load T_exp(t)."""
    knee = lam * RP
    return bias + k1 * G(t, knee, s) + k2 * n_active(E, K, t) + k3 * G(t_exp(E, K, t), knee, s)


def T_target(p, RP, E, K, t):
    return target_time(p["bias"], p["k1"], p["k2"], p["k3"], p["lam"], p["s"], RP, E, K, t)


def T_draft(p, RP, B):
    """One forward of the (dense) draft model over B tokens: fixed part + roofline in B."""
    return p["draft_bias"] + p["draft_k"] * G(B, p["lam"] * RP, p["s"])


def T_reject(p, B):
    """Rejection sampling: linear in the batch size."""
    return p["reject_bias"] + p["reject_k"] * B


def verified_tokens(B, gamma, bonus):
    return B * (gamma + 1) if bonus else B * gamma


def T_SD_round(p, B, gamma, K, E, RP, bonus):
    """Eq. (T_SD): one round = gamma draft forwards, one verification forward, one rejection step."""
    return gamma * T_draft(p, RP, B) + T_target(p, RP, E, K, verified_tokens(B, gamma, bonus)) + T_reject(p, B)


def compute_speedup(params, B, gamma, K, E, sig, RP, bonus=False):
    """Eq. (speedup): a round yields sigma * (gamma + 1) tokens per request in T_SD_round, against one
    token per autoregressive forward T_T(B)."""
    p = _named(params)
    tokens_per_round = sig * (gamma + 1)
    return tokens_per_round * T_target(p, RP, E, K, B) / T_SD_round(p, B, gamma, K, E, RP, bonus)


def target_efficiency(params, B, gamma, K, E, RP, bonus=False):
    """T_T(B, 1) / T_T(B, gamma) (Sec. 3.1)."""
    p = _named(params)
    return T_target(p, RP, E, K, B) / T_target(p, RP, E, K, verified_tokens(B, gamma, bonus))
