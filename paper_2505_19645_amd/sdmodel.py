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
