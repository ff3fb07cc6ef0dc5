"""Pins for the oracle's routing, permutation and layer arithmetic.

The paper prints no worked example of a layer output, so the layer is pinned by
what mathematics fixes: brute-force subset routing, invariants of the weights,
a library sort for the permutation, and special cases in which the whole layer
collapses to plain matrix products evaluated by numpy in fp64.
"""
import dataclasses
import itertools
from fractions import Fraction

import numpy as np
import pytest

from paper_2505_19645_amd import synth
from paper_2505_19645_amd.synth import LayerShape, bf16_bits_to_f32, f32_to_bf16_bits


def f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


def small_layer(shape, skew=0.0):
    return synth.make_layer(shape, skew_std=skew, threads=1)


# ---------------------------------------------------------------- routing ----

def brute_force_topk(keys, K):
    """Among all K-subsets pick the one with the largest exact key sum; on equal
    sums the lexicographically smallest index tuple."""
    E = len(keys)
    best, best_sum = None, None
    for sub in itertools.combinations(range(E), K):
        s = sum(Fraction(float(keys[e])) for e in sub)
        if best is None or s > best_sum:
            best, best_sum = sub, s
    return set(best)


@pytest.mark.parametrize("E,K,score", [(8, 2, 0), (8, 3, 1), (6, 6, 0), (5, 1, 0), (7, 4, 1)])
def test_route_matches_brute_force(oracle, E, K, score):
    shape = LayerShape("t", d=64, E=E, top_k=K, inter=16, score_func=score, seed=11)
    x = synth.make_tokens(shape, 16)
    r = synth.make_router(shape)
    ids, w, logits = oracle.route(shape, x, r["w_router"])
    # logits against a library matmul in fp64
    ref = f64(x) @ f64(r["w_router"]).T
    np.testing.assert_allclose(logits, ref, rtol=0, atol=1e-12)
    keys = logits.astype(np.float32)
    for t in range(16):
        assert set(ids[t].tolist()) == brute_force_topk(keys[t], K)
        # listed by descending key, equal keys by ascending index
        order = sorted(ids[t].tolist(), key=lambda e: (-float(keys[t, e]), e))
        assert ids[t].tolist() == order


def test_route_forced_ties(oracle):
    shape = LayerShape("t", d=32, E=8, top_k=3, inter=16, seed=5)
    r = synth.make_router(shape)
    # all-zero tokens: every logit equal -> lowest indices win, equal weights
    x0 = synth.make_tokens(shape, 4, zero=True)
    ids, w, _ = oracle.route(shape, x0, r["w_router"])
    assert (ids == np.arange(3)[None, :]).all()
    np.testing.assert_allclose(w, 1.0 / 3.0, rtol=0, atol=1e-15)
    # duplicated router rows: experts 2 and 5 always tie; 2 must precede 5
    wr = r["w_router"].copy()
    wr[5] = wr[2]
    x = synth.make_tokens(shape, 64)
    ids, w, logits = oracle.route(shape, x, wr)
    assert (logits[:, 2] == logits[:, 5]).all()
    seen_both = 0
    for t in range(64):
        row = ids[t].tolist()
        if 5 in row:
            assert 2 in row and row.index(2) + 1 == row.index(5)
            seen_both += 1
    assert seen_both > 0
    # a bias that dominates the logits dictates the winners
    bias = np.zeros(8, np.float32)
    bias[[6, 1]] = [50.0, 40.0]
    ids, _, _ = oracle.route(shape, x, r["w_router"], bias)
    assert (ids[:, 0] == 6).all() and (ids[:, 1] == 1).all()


def rounding_boundary_router():
    """A router whose logits are sums of a few products of powers of two, so they are exact in fp64 in any
    summation order, and which land on fp32 rounding boundaries.  Token x = s * (1, 2^-12, 2^-20, 0, ...):
      expert 2:  w = (1, 0, 0)            logit s * 1                       key s * 1
      expert 5:  w = (1, 2^-12, 0)        s * (1 + 2^-24): the midpoint of 1 and 1 + 2^-23, ties to even -> s * 1
      expert 7:  w = (1, 2^-12, 2^-20)    s * (1 + 2^-24 + 2^-40): just above the midpoint -> s * (1 + 2^-23)
      expert 1:  w = (1, 3 * 2^-12, 0)    s * (1 + 3 * 2^-24): midpoint of 1 + 2^-23 and 1 + 2^-22 -> even: s * (1 + 2^-22)
      others:    w = (0.5, 0, 0)          s * 0.5
    So the order is 1, 7, then experts 2 and 5 with equal keys (lower index first), whatever s > 0 (a power of two).
    -> (shape, weights, x, the ids every token must get)"""
    shape = LayerShape("rounding-boundaries", d=64, E=8, top_k=4, inter=64, seed=77)
    w = synth.make_layer(shape)
    wr = np.zeros((shape.E, shape.d), np.float32)
    wr[:, 0] = 0.5
    wr[2, :3] = (1.0, 0.0, 0.0)
    wr[5, :3] = (1.0, 2.0 ** -12, 0.0)
    wr[7, :3] = (1.0, 2.0 ** -12, 2.0 ** -20)
    wr[1, :3] = (1.0, 3.0 * 2.0 ** -12, 0.0)
    w["w_router"] = f32_to_bf16_bits(wr)
    assert np.array_equal(bf16_bits_to_f32(w["w_router"]), wr)   # every entry is a bf16 value
    x = np.zeros((3, shape.d), np.float32)
    for t, s_ in enumerate((1.0, 4.0, 0.25)):
        x[t, :3] = (s_, s_ * 2.0 ** -12, s_ * 2.0 ** -20)
    xb = f32_to_bf16_bits(x)
    assert np.array_equal(bf16_bits_to_f32(xb), x)
    return shape, w, xb, np.array([1, 7, 2, 5], np.int32)


def test_route_keys_on_fp32_rounding_boundaries(oracle):
    # one rounding of the exact logit to fp32, nearest-even on the midpoint, then ties to the lower index
    shape, w, x, want = rounding_boundary_router()
    ids, wts, logits = oracle.route(shape, x, w["w_router"])
    assert (ids == want[None, :]).all()
    assert logits[0, 5] == 1.0 + 2.0 ** -24 and logits[0, 7] == 1.0 + 2.0 ** -24 + 2.0 ** -40
    assert np.float32(logits[0, 5]) == np.float32(1.0) and np.float32(logits[0, 7]) == np.float32(1.0 + 2.0 ** -23)
    # the weights come from the fp64 logits, so the two experts with equal keys still get different weights
    assert wts[0, 2] < wts[0, 3]


@pytest.mark.parametrize("score", [0, 1])
@pytest.mark.parametrize("renorm", [0, 1])
def test_route_weight_invariants(oracle, score, renorm):
    shape = LayerShape("t", d=128, E=16, top_k=4, inter=16, score_func=score, renormalize=renorm,
                       routed_scale=1.0, seed=3)
    x = synth.make_tokens(shape, 32)
    r = synth.make_router(shape)
    ids, w, logits = oracle.route(shape, x, r["w_router"])
    assert (w > 0).all()
    assert (np.diff(w, axis=1) <= 1e-7 * w[:, :-1]).all()          # follows the key order
    sel = np.take_along_axis(logits, ids, axis=1)
    if renorm:
        np.testing.assert_allclose(w.sum(1), 1.0, rtol=0, atol=1e-12)
        if score == 0:
            # softmax then renormalise == softmax restricted to the winners
            z = np.exp(sel - sel.max(1, keepdims=True))
            np.testing.assert_allclose(w, z / z.sum(1, keepdims=True), rtol=1e-12)
        else:
            s = 1 / (1 + np.exp(-sel))
            np.testing.assert_allclose(w, s / s.sum(1, keepdims=True), rtol=1e-12)
    else:
        if score == 0:
            assert (w.sum(1) < 1.0).all()                          # part of the mass is left out
            full = np.exp(logits - logits.max(1, keepdims=True))
            full /= full.sum(1, keepdims=True)
            np.testing.assert_allclose(w, np.take_along_axis(full, ids, 1), rtol=1e-12)
        else:
            np.testing.assert_allclose(w, 1 / (1 + np.exp(-sel)), rtol=1e-12)
    # routed_scale multiplies the weights
    shape2 = dataclasses.replace(shape, routed_scale=2.5)
    _, w2, _ = oracle.route(shape2, x, r["w_router"])
    np.testing.assert_allclose(w2, 2.5 * w, rtol=1e-15)


def test_router_is_near_uniform_on_gaussian_inputs(oracle):
    """Synthetic stand-in for the paper's Fig. 1(a,b): activated experts counted
    by the oracle's own router on Gaussian tokens track Eq. N(t)."""
    shape = LayerShape("t", d=256, E=60, top_k=4, inter=16, seed=77)
    r = synth.make_router(shape)
    for T in (4, 16, 44):
        got = []
        for trial in range(60):
            x = synth.make_tokens(shape, T, point=1000 * T + trial)
            ids, _, _ = oracle.route(shape, x, r["w_router"])
            got.append(oracle.permute(shape.E, shape.top_k, ids)["n_active"])
        want = oracle.expected_active_experts(shape.E, shape.top_k, T)
        assert abs(np.mean(got) - want) < 0.03 * shape.E, (T, np.mean(got), want)


# ------------------------------------------------------------ permutation ----

@pytest.mark.parametrize("E,K,T", [(8, 2, 16), (60, 4, 37), (256, 8, 200), (4, 4, 5), (16, 1, 1),
                                   (8, 2, 0)])
def test_permute_matches_stable_argsort(oracle, E, K, T):
    rng = np.random.default_rng(E * 1000 + T)
    if T:
        ids = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32)
    else:
        ids = np.zeros((0, K), np.int32)
    r = oracle.permute(E, K, ids)
    flat = ids.ravel()
    n = T * K
    assert r["counts"].sum() == n
    np.testing.assert_array_equal(r["counts"], np.bincount(flat, minlength=E))
    np.testing.assert_array_equal(r["offsets"], np.concatenate([[0], np.cumsum(r["counts"])]))
    assert r["offsets"][E] == n
    np.testing.assert_array_equal(r["perm"], np.argsort(flat, kind="stable"))
    np.testing.assert_array_equal(r["inv"][r["perm"]], np.arange(n))
    assert r["n_active"] == len(set(flat.tolist()))
    srt = flat[r["perm"]]
    assert (np.diff(srt) >= 0).all()
    same = np.diff(srt) == 0
    assert (np.diff(r["perm"])[same] > 0).all()                   # stable within an expert


def test_permute_rejects_bad_ids(oracle):
    with pytest.raises(ValueError):
        oracle.permute(4, 2, np.array([[0, 4]], np.int32))


# --------------------------------------------------------- layer arithmetic ----

def dense_mlp(x, wg, wu, wd):
    g = x @ wg.T
    u = x @ wu.T
    return ((g / (1 + np.exp(-g))) * u) @ wd.T


def test_single_expert_is_a_dense_mlp(oracle):
    # E = 1, K = 1: the layer is three plain matrix products (numpy, fp64)
    shape = LayerShape("t", d=96, E=1, top_k=1, inter=80, seed=21)
    w = small_layer(shape)
    x = synth.make_tokens(shape, 9)
    r = oracle.moe_forward(shape, w, x)
    ref = dense_mlp(f64(x), f64(w["w_gate"][0]), f64(w["w_up"][0]), f64(w["w_down"][0]))
    np.testing.assert_allclose(r["out"], ref, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(r["w"], 1.0)


def test_shared_expert_only_and_gate(oracle):
    # zeroed routed down-projection leaves g_t * shared MLP
    shape = LayerShape("t", d=64, E=4, top_k=2, inter=32, shared_inter=48, shared_gate=1, seed=22)
    w = small_layer(shape)
    w["w_down"][:] = 0
    x = synth.make_tokens(shape, 7)
    r = oracle.moe_forward(shape, w, x)
    g = 1 / (1 + np.exp(-(f64(x) @ f64(w["w_shared_gate"]))))
    ref = g[:, None] * dense_mlp(f64(x), f64(w["ws_gate"]), f64(w["ws_up"]), f64(w["ws_down"]))
    np.testing.assert_allclose(r["out"], ref, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(r["gate"], g, rtol=1e-12)
    shape_ng = dataclasses.replace(shape, shared_gate=0)
    r2 = oracle.moe_forward(shape_ng, w, x)
    np.testing.assert_allclose(r2["out"], ref / g[:, None], rtol=1e-11, atol=1e-12)


def test_all_experts_selected_is_softmax_mixture(oracle):
    # K = E with renormalisation: softmax-weighted sum of every expert's MLP
    shape = LayerShape("t", d=64, E=5, top_k=5, inter=32, seed=23)
    w = small_layer(shape)
    x = synth.make_tokens(shape, 6)
    r = oracle.moe_forward(shape, w, x)
    X = f64(x)
    logits = X @ f64(w["w_router"]).T
    p = np.exp(logits - logits.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    ref = sum(p[:, e:e + 1] * dense_mlp(X, f64(w["w_gate"][e]), f64(w["w_up"][e]), f64(w["w_down"][e]))
              for e in range(5))
    np.testing.assert_allclose(r["out"], ref, rtol=1e-10, atol=1e-12)
    assert r["n_active"] == 5 and (r["counts"] == 6).all()


def test_general_case_against_per_token_matmuls(oracle):
    # top-2 of 6 with a shared expert: rebuild each token's output from numpy
    # matrix products of the experts the oracle says it chose
    shape = LayerShape("t", d=64, E=6, top_k=2, inter=48, shared_inter=32, shared_gate=1, seed=29)
    w = small_layer(shape)
    x = synth.make_tokens(shape, 10)
    r = oracle.moe_forward(shape, w, x)
    X = f64(x)
    g = 1 / (1 + np.exp(-(X @ f64(w["w_shared_gate"]))))
    sh = dense_mlp(X, f64(w["ws_gate"]), f64(w["ws_up"]), f64(w["ws_down"]))
    for t in range(10):
        acc = g[t] * sh[t]
        for s in range(2):
            e = r["ids"][t, s]
            acc = acc + r["w"][t, s] * dense_mlp(X[t:t + 1], f64(w["w_gate"][e]), f64(w["w_up"][e]),
                                                 f64(w["w_down"][e]))[0]
        np.testing.assert_allclose(r["out"][t], acc, rtol=1e-10, atol=1e-12)
    # token subset gives the same rows
    sub = oracle.moe_forward(shape, w, x, tokens=[7, 2, 9])
    np.testing.assert_array_equal(sub["out"], r["out"][[7, 2, 9]])
    np.testing.assert_array_equal(sub["out_bf16"], r["out_bf16"][[7, 2, 9]])


def test_identical_experts_collapse(oracle):
    # every expert holds the same weights and the top-k weights sum to one
    shape = LayerShape("t", d=64, E=6, top_k=3, inter=32, seed=24)
    w = small_layer(shape)
    for k in ("w_gate", "w_up", "w_down"):
        w[k][:] = w[k][0]
    x = synth.make_tokens(shape, 8)
    r = oracle.moe_forward(shape, w, x)
    ref = dense_mlp(f64(x), f64(w["w_gate"][0]), f64(w["w_up"][0]), f64(w["w_down"][0]))
    np.testing.assert_allclose(r["out"], ref, rtol=1e-10, atol=1e-12)


def test_zero_tokens_and_linearity_in_down(oracle):
    shape = LayerShape("t", d=64, E=8, top_k=2, inter=32, seed=25)
    w = small_layer(shape)
    x0 = synth.make_tokens(shape, 5, zero=True)
    r0 = oracle.moe_forward(shape, w, x0)
    assert (r0["out"] == 0).all() and (r0["out_bf16"] == 0).all()
    assert (r0["ids"] == np.array([0, 1])).all()
    x = synth.make_tokens(shape, 5)
    r = oracle.moe_forward(shape, w, x)
    w2 = dict(w)
    w2["w_down"] = f32_to_bf16_bits(2.0 * bf16_bits_to_f32(w["w_down"]))   # exact in bf16
    r2 = oracle.moe_forward(shape, w2, x)
    np.testing.assert_allclose(r2["out"], 2.0 * r["out"], rtol=1e-14)


def test_relabelling_experts_leaves_output_unchanged(oracle):
    shape = LayerShape("t", d=64, E=8, top_k=3, inter=32, seed=26)
    w = small_layer(shape, skew=1.0)
    x = synth.make_tokens(shape, 12)
    r = oracle.moe_forward(shape, w, x)
    pi = np.random.default_rng(0).permutation(8)                   # new label i holds old expert pi[i]
    w2 = dict(w)
    for k in ("w_router", "w_gate", "w_up", "w_down", "router_bias"):
        w2[k] = np.ascontiguousarray(w[k][pi])
    r2 = oracle.moe_forward(shape, w2, x)
    # distinct logits -> same experts under new names, same summation order per token
    np.testing.assert_array_equal(pi[r2["ids"]], r["ids"])
    np.testing.assert_allclose(r2["out"], r["out"], rtol=1e-13, atol=1e-15)


def test_fp32_twin_agrees(oracle):
    # the same loops carried in fp32 stay within fp32 round-off of the fp64 ones
    shape = LayerShape("t", d=256, E=2, top_k=1, inter=128, seed=27)
    w = small_layer(shape)
    x = synth.make_tokens(shape, 1)
    y64 = oracle.ffn_row(x[0], w["w_gate"][0], w["w_up"][0], w["w_down"][0])
    y32 = oracle.ffn_row(x[0], w["w_gate"][0], w["w_up"][0], w["w_down"][0], f32=True)
    rel = np.linalg.norm(y32 - y64) / np.linalg.norm(y64)
    assert rel < 1e-5
    ref = dense_mlp(f64(x), f64(w["w_gate"][0]), f64(w["w_up"][0]), f64(w["w_down"][0]))[0]
    np.testing.assert_allclose(y64, ref, rtol=1e-11, atol=1e-13)


def test_bf16_rounding_is_single_step_nearest_even(oracle):
    import torch
    rng = np.random.default_rng(9)
    v32 = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3,
                          np.array([1.0, -1.0, 0.0, 1.00390625, 1.01171875, 255.5, 3.0e-3], np.float32)])
    want = torch.from_numpy(v32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(oracle.round_bf16(v32.astype(np.float64)), want)
    # exact ties go to the even neighbour; a hair above a tie rounds up even
    # though a detour through fp32 would first land on the tie and round down
    tie = 1.0 + 2.0 ** -8                       # halfway between bf16 1.0 and 1.0078125
    assert oracle.round_bf16(np.array([tie]))[0] == 0x3F80
    assert oracle.round_bf16(np.array([tie + 2.0 ** -40]))[0] == 0x3F81
    assert oracle.round_bf16(np.array([1.0078125 + 2.0 ** -8]))[0] == 0x3F82
    # and the generator's own fp32 -> bf16 rounding agrees with the library's
    np.testing.assert_array_equal(f32_to_bf16_bits(v32), want)


def test_tiny_benchmark_config_runs(oracle):
    shape = synth.PRESETS["tiny"]
    w = synth.make_layer(shape)
    x = synth.make_tokens(shape, 16)
    r = oracle.moe_forward(shape, w, x)
    assert r["out"].shape == (16, 256) and np.isfinite(r["out"]).all()
    np.testing.assert_allclose(r["w"].sum(1), 1.0, atol=1e-12)
    assert r["counts"].sum() == 32
    rel = np.linalg.norm(f64(r["out_bf16"]) - r["out"]) / np.linalg.norm(r["out"])
    assert rel < 2.5e-3                          # one bf16 rounding
