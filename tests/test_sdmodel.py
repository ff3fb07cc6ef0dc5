"""The roofline surrogate G of the paper's Sec. 3.3 and the layer-curve fit built on it."""
import math

import numpy as np

from paper_2505_19645_amd import sdmodel


def test_G_is_exponential_then_tangent_and_C1_at_the_knee():
    knee, s = 40.0, 1.03
    # below the knee: s**t
    for t in (0.0, 1.0, 17.5, 40.0):
        assert sdmodel.roofline_G(t, knee, s) == np.float64(s) ** t
    # at the knee value and slope are continuous (Eq. G: first-order continuity)
    eps = 1e-6
    left = (sdmodel.roofline_G(knee, knee, s) - sdmodel.roofline_G(knee - eps, knee, s)) / eps
    right = (sdmodel.roofline_G(knee + eps, knee, s) - sdmodel.roofline_G(knee, knee, s)) / eps
    assert abs(left - right) < 1e-4 * left
    assert abs(left - math.log(s) * s ** knee) < 1e-4 * left
    # beyond: a straight line
    a, b, c = (float(sdmodel.roofline_G(t, knee, s)) for t in (50.0, 60.0, 70.0))
    assert abs((b - a) - (c - b)) < 1e-9
    assert (np.diff(sdmodel.roofline_G(np.linspace(0, 200, 400), knee, s)) > 0).all()


def test_fit_recovers_a_planted_curve():
    E, K = 60, 4
    T = np.array([1, 2, 4, 8, 16, 32, 64, 128, 256, 640], float)
    n = E * (1 - (1 - K / E) ** T)
    truth = (12.0, 3.1, 5.0, 0.5, 1.02)
    us = sdmodel.layer_time(truth, n, T * K / n, ridge_point=312.0)
    fit = sdmodel.fit_layer_curve(T, n, us, E, K, k2_min_us=2.2, ridge_point=312.0)
    assert fit["max_rel_err"] < 1e-3
    assert abs(fit["c2_us_per_expert"] - 3.1) < 0.05
