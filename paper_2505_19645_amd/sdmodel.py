"""The paper's forward-time model, used to overlay the measured layer-time curve.

Sec. 3.3 prices one target forward as  bias + k1*G(t) + k2*N + k3*G(T_exp)  (Alg. 1,
the ar_time / verify_time lines), with the roofline surrogate G of Eq. G(t): s^t up to
the knee lambda*RP and its tangent line after it.  For a single MoE layer the dense term
k1*G(t) belongs to attention and is left out; what remains is fitted to the measured
layer times by bounded least squares (trust-region reflective, as in Appendix C.2):

    t_layer(T) ~= c0 + c2 * n_active(T) + c3 * G(T_exp(T); lambda*RP, s)

c2 is the time to load one expert; Appendix C.2's floor for it is
k2_min = expert bytes / peak memory bandwidth.
"""
from __future__ import annotations

import math

import numpy as np


def roofline_G(t, knee, s):
    """Eq. G(t; lambda*RP, s): s**t for t <= knee, then the tangent at the knee
    (value and first derivative are continuous there)."""
    t = np.asarray(t, dtype=np.float64)
    below = np.power(s, np.minimum(t, knee))
    return np.where(t <= knee, below, (s ** knee) * (1.0 + math.log(s) * (t - knee)))


def layer_time(params, n_active, t_exp, ridge_point):
    c0, c2, c3, lam, s = params
    return c0 + c2 * np.asarray(n_active, np.float64) + c3 * roofline_G(t_exp, lam * ridge_point, s)


def fit_layer_curve(T, n_active, us, E, K, k2_min_us, ridge_point):
    """Fit (c0, c2, c3, lambda, s) to measured layer times.  Bounds follow Appendix C.2:
    c2 in [k2_min, 5*k2_min], lambda in [0.2, 1], s in [1, 2], c0, c3 >= 0."""
    from scipy.optimize import least_squares
    T = np.asarray(T, np.float64)
    n_active = np.asarray(n_active, np.float64)
    us = np.asarray(us, np.float64)
    t_exp = T * K / np.maximum(n_active, 1.0)
    lo = [0.0, k2_min_us, 0.0, 0.2, 1.0]
    hi = [np.inf, 5.0 * k2_min_us, np.inf, 1.0, 2.0]
    x0 = [max(us.min() * 0.2, 1e-3), 1.5 * k2_min_us, 1.0, 0.5, 1.05]

    def resid(p):
        return layer_time(p, n_active, t_exp, ridge_point) - us

    r = least_squares(resid, x0, bounds=(lo, hi), method="trf")
    pred = layer_time(r.x, n_active, t_exp, ridge_point)
    rel = np.abs(pred - us) / us
    return {"c0_us": float(r.x[0]), "c2_us_per_expert": float(r.x[1]), "c3_us": float(r.x[2]),
            "lambda": float(r.x[3]), "s": float(r.x[4]), "k2_min_us": float(k2_min_us),
            "c2_over_k2_min": float(r.x[1] / k2_min_us),
            "mean_rel_err": float(rel.mean()), "max_rel_err": float(rel.max()),
            "pred_us": [round(float(v), 2) for v in pred]}


# ---------------------------------------------------------------------------------------
# Speed-up model (Sec. 3.1 Eq. (speedup), Sec. 3.3 / Alg. 1), vectorised over measurements.
#
# Two places where the paper disagrees with itself, and what is done here:
#  * Alg. 1 prints the denominator as draft + ar + verify + reject; Eq. (speedup), which the
#    text derives, has gamma*T_D + T_T(B, gamma) + T_reject.  The equation is used.
#  * Alg. 1 prices verification at B*gamma tokens, the text adds a bonus token.  `bonus=True`
#    (B*(gamma+1) tokens) is the default because that is what the layer benchmark runs.

PARAM_NAMES = ("bias", "k1", "k2", "k3", "draft_bias", "draft_k", "reject_bias", "reject_k", "lambda", "s")


def sigma_from_alpha(alpha, gamma):
    """sigma = (1 - alpha^(gamma+1)) / ((1 - alpha) (gamma + 1)); 1 at alpha = 1."""
    alpha = np.asarray(alpha, np.float64)
    gamma = np.asarray(gamma, np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        v = (1.0 - np.power(alpha, gamma + 1.0)) / ((1.0 - alpha) * (gamma + 1.0))
    return np.where(alpha == 1.0, 1.0, v)


def expected_active(E, K, t):
    return E * (1.0 - np.power((E - K) / E, np.asarray(t, np.float64)))


def target_forward_time(p, E, K, t, ridge_point):
    """bias + k1*G(t) + k2*N(t) + k3*G(T_exp(t)) with p = the ten parameters."""
    t = np.asarray(t, np.float64)
    n = expected_active(E, K, t)
    t_exp = np.where(n > 0.0, t * K / np.maximum(n, 1e-300), 0.0)
    knee = p[8] * ridge_point
    return p[0] + p[1] * roofline_G(t, knee, p[9]) + p[2] * n + p[3] * roofline_G(t_exp, knee, p[9])


def compute_speedup(p, B, gamma, K, E, sigma, ridge_point, bonus=True):
    B = np.asarray(B, np.float64)
    gamma = np.asarray(gamma, np.float64)
    ar = target_forward_time(p, E, K, B, ridge_point)
    verify = target_forward_time(p, E, K, B * (gamma + 1.0 if bonus else gamma), ridge_point)
    draft = p[4] + p[5] * roofline_G(B, p[8] * ridge_point, p[9])
    reject = p[6] + p[7] * B
    return np.asarray(sigma, np.float64) * (gamma + 1.0) * ar / (gamma * draft + verify + reject)


def target_efficiency(p, B, gamma, K, E, ridge_point, bonus=True):
    B = np.asarray(B, np.float64)
    gamma = np.asarray(gamma, np.float64)
    return (target_forward_time(p, E, K, B, ridge_point) /
            target_forward_time(p, E, K, B * (gamma + 1.0 if bonus else gamma), ridge_point))


def fit_speedup(B, gamma, K, E, sigma, speedup, ridge_point, bias_min, k2_min, draft_bias_min=0.0,
                t_rej_max=np.inf, bonus=True, x0=None):
    """Alg. 1's last line: bounded least squares (trust-region reflective) of the ten
    parameters against measured speed-ups.  Bounds of Appendix C.2: bias in [bias_min,
    5 bias_min], k2 in [k2_min, 5 k2_min], draft_bias in [draft_bias_min, 5 draft_bias_min]
    (free above 0 when no draft model size is given), reject terms in [0, t_rej_max],
    lambda in [0.2, 1], s in [1, 2], k1, k3, draft_k >= 0."""
    from scipy.optimize import least_squares
    B = np.asarray(B, np.float64)
    gamma = np.asarray(gamma, np.float64)
    sigma = np.asarray(sigma, np.float64)
    speedup = np.asarray(speedup, np.float64)
    tiny = 1e-12
    lo = [bias_min, 0.0, k2_min, 0.0, draft_bias_min, 0.0, 0.0, 0.0, 0.2, 1.0 + 1e-9]
    hi = [max(5.0 * bias_min, tiny), np.inf, max(5.0 * k2_min, tiny),
          np.inf, 5.0 * draft_bias_min if draft_bias_min > 0.0 else np.inf, np.inf,
          t_rej_max, t_rej_max, 1.0, 2.0]
    if x0 is None:
        x0 = [1.5 * bias_min + tiny, 0.01 * (k2_min + tiny), 1.5 * k2_min + tiny, 0.01 * (k2_min + tiny),
              (1.5 * draft_bias_min) if draft_bias_min > 0.0 else 0.1 * (bias_min + k2_min + tiny), 0.0,
              0.0, 0.0, 0.5, 1.01]
    x0 = [min(max(v, l + 1e-12 * (1.0 + abs(l))), h if np.isfinite(h) else v + 1.0) for v, l, h in zip(x0, lo, hi)]

    def resid(p):
        return compute_speedup(p, B, gamma, K, E, sigma, ridge_point, bonus) - speedup

    r = least_squares(resid, x0, bounds=(lo, hi), method="trf", x_scale="jac")
    pred = compute_speedup(r.x, B, gamma, K, E, sigma, ridge_point, bonus)
    rel = np.abs(pred - speedup) / np.maximum(np.abs(speedup), 1e-300)
    return {"params": {n: float(v) for n, v in zip(PARAM_NAMES, r.x)}, "x": r.x,
            "pred": pred, "mean_rel_err": float(rel.mean()), "max_rel_err": float(rel.max()),
            "cost": float(r.cost)}


def layer_speedups_from_curve(times_us_by_T, gammas=(1, 2, 3, 4), alpha=0.8, draft_ratio=0.1, reject_ratio=0.01):
    """Turn measured layer times t(T) into layer-level speed-up 'measurements' with Eq.
    (speedup): the target forward is the measured layer, T_D = draft_ratio * t(B) (the paper
    notes T_D/T_T is usually below 1/10), T_reject = reject_ratio * t(B), sigma from a stated
    acceptance rate.  Only (B, gamma) with both t(B) and t(B*(gamma+1)) measured are used.
    -> list of dicts B, gamma, sigma, speedup, target_efficiency."""
    out = []
    for g in gammas:
        sg = float(sigma_from_alpha(alpha, g))
        for B in sorted(times_us_by_T):
            Tv = B * (g + 1)
            if Tv not in times_us_by_T:
                continue
            t1, tv = times_us_by_T[B], times_us_by_T[Tv]
            sp = sg * (g + 1) * t1 / (g * draft_ratio * t1 + tv + reject_ratio * t1)
            out.append({"B": B, "gamma": g, "sigma": sg, "speedup": sp, "target_efficiency": t1 / tv})
    return out
