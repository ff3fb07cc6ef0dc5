"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Integer outputs must be bit-exact; the layer output must
meet relative L2 <= 5e-3 and max-abs <= 2e-2 * RMS(out)."""
import dataclasses
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2505_19645_amd import synth
from paper_2505_19645_amd.synth import PRESETS, LayerShape


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import os
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_harness
    if os.path.exists(gpu_harness.PARITY_LOG):   # one log per test run
        os.remove(gpu_harness.PARITY_LOG)
    return gpu_harness


_FULL = {}


def full_size_weights(name, gpu=None):
    """Weights of a benchmark preset at full size, on the host and (with gpu) on the device; one preset is
    kept at a time (config 4 is 22.6 GB)."""
    if name not in _FULL:
        _FULL.clear()
        import gc
        gc.collect()
        if gpu is not None:
            gpu.torch.cuda.empty_cache()
        _FULL[name] = {"w": synth.make_layer(PRESETS[name], threads=16)}
    if gpu is not None and "layer" not in _FULL[name]:
        _FULL[name]["layer"] = gpu.GpuLayer(PRESETS[name], _FULL[name]["w"])
    return _FULL[name]["w"] if gpu is None else (_FULL[name]["w"], _FULL[name]["layer"])


ROW_CLASSES = ((1, 16), (17, 64), (65, 128), (129, 1 << 30))   # rows per expert: the kernels' tile classes


def class_of(m):
    return next(i for i, (lo, hi) in enumerate(ROW_CLASSES) if lo <= m <= hi)


def tokens_from_permutation(oracle, shape, w, x, budget=32):
    """Tokens to compare at a size where the oracle cannot evaluate them all, chosen from the oracle's own
    routing so that every kind of row position is hit: for each class of expert size (1..16, 17..64, 65..128,
    more rows) the first and last row of its smallest and of its largest expert; the rows on both sides of a
    64-row block border, of a 256-row border (where the tiled kernels' waves pass from their first token tile
    to their second) and of a 512-row block border; a token whose K experts lie in different classes; the first
    and the last token; then tokens drawn at random (seeded) up to the budget."""
    T, K = x.shape[0], shape.top_k
    ids, _, _ = oracle.route(shape, x, w["w_router"], w.get("router_bias"))
    pr = oracle.permute(shape.E, K, ids)
    counts, offsets, perm = pr["counts"], pr["offsets"], pr["perm"]
    rows = []
    for ci in range(len(ROW_CLASSES)):
        es = [e for e in range(shape.E) if counts[e] > 0 and class_of(counts[e]) == ci]
        if not es:
            continue
        for e in {min(es, key=lambda e: counts[e]), max(es, key=lambda e: counts[e])}:
            rows += [offsets[e], offsets[e + 1] - 1]
    big = [e for e in range(shape.E) if counts[e] > 64]
    if big:
        e = max(big, key=lambda e: counts[e])
        rows += [offsets[e] + 63, offsets[e] + 64]
        if counts[e] > 256:
            rows += [offsets[e] + 255, offsets[e] + 256, offsets[e] + 256 * ((counts[e] - 1) // 256) - 1]
        if counts[e] > 512:
            rows += [offsets[e] + 511, offsets[e] + 512]
    toks = [0, T - 1] + [int(perm[r]) // K for r in rows]
    for t in range(T):
        if len({class_of(counts[e]) for e in ids[t]}) > 1:
            toks.append(t)
            break
    out = []
    for t in toks:
        if t not in out:
            out.append(t)
    # the rest of the budget: tokens drawn at random (seeded by the size), so that rows in the middle of tiles are hit too
    for t in np.random.default_rng(T * 7919 + shape.E).permutation(T).tolist():
        if len(out) >= budget:
            break
        if t not in out:
            out.append(t)
    return np.array(sorted(out[:budget]), dtype=np.int32)


def run_case(gpu, oracle, shape, T, skew=0.0, zero_x=False, tokens=None, point=0, weights=None, layer=None, x=None):
    say(f"[case] {shape.name} d={shape.d} E={shape.E} K={shape.top_k} I={shape.inter} "
        f"S={shape.shared_inter} score={shape.score_func} T={T} skew={skew} zero={zero_x}")
    w = weights if weights is not None else synth.make_layer(shape, skew_std=skew)
    x = x if x is not None else synth.make_tokens(shape, T, point=point, zero=zero_x)
    layer = layer if layer is not None else gpu.GpuLayer(shape, w)
    got = layer.forward(x)
    ref = oracle.moe_forward(shape, w, x, tokens=tokens)
    gpu.check_routing(ref, got, shape.name)
    stats = gpu.check_outputs(ref, got, tokens=tokens, label=f"{shape.name} T={T}" + (f" skew={skew}" if skew else ""))
    say(f"       ok: {stats} n_active={got['n_active']}")
    return got, ref


def test_tiny_config(gpu, oracle):
    # benchmark config 0: d=256, E=8, top-2, I=512, T=16 (B=4, gamma=3), seed 0
    run_case(gpu, oracle, PRESETS["tiny"], 16)


@pytest.mark.parametrize("T", [1, 2, 5, 16, 17, 33, 64, 100])
def test_small_shapes_ragged_T(gpu, oracle, T):
    shape = LayerShape("ragged", d=384, E=12, top_k=3, inter=200, shared_inter=136, shared_gate=1, seed=7)
    run_case(gpu, oracle, shape, T)


@pytest.mark.parametrize("shape", [
    LayerShape("sig-nogate", d=512, E=40, top_k=6, inter=264, shared_inter=72, score_func=1, seed=8),
    LayerShape("norenorm", d=256, E=16, top_k=4, inter=128, renormalize=0, routed_scale=2.5, seed=9),
    LayerShape("sig-norenorm", d=256, E=16, top_k=4, inter=128, score_func=1, renormalize=0, seed=10),
    LayerShape("dense-like", d=256, E=4, top_k=4, inter=256, seed=11),
    LayerShape("one-expert", d=128, E=1, top_k=1, inter=64, seed=12),
    LayerShape("wide-E", d=128, E=300, top_k=8, inter=64, seed=13),
    LayerShape("k32", d=128, E=64, top_k=32, inter=64, seed=14),
    LayerShape("tails", d=264, E=6, top_k=2, inter=72, shared_inter=24, shared_gate=1, seed=15),
])
def test_variants(gpu, oracle, shape):
    run_case(gpu, oracle, shape, 23)


@pytest.mark.parametrize("shape,T", [
    (LayerShape("rows-gt-64", d=256, E=4, top_k=2, inter=192, shared_inter=96, shared_gate=1, seed=31), 300),
    (LayerShape("rows-gt-256", d=128, E=2, top_k=1, inter=136, seed=32), 700),
    (LayerShape("tiled-tails", d=264, E=3, top_k=2, inter=72, shared_inter=40, seed=33), 130),
    (LayerShape("mixed-classes", d=256, E=16, top_k=2, inter=128, shared_inter=64, shared_gate=1, seed=34), 200),
])
def test_many_rows_per_expert(gpu, oracle, shape, T):
    # experts above 64 rows go through the MFMA-tiled kernel; the skewed case mixes all three classes
    skew = 2.0 if shape.name == "mixed-classes" else 0.0
    got, ref = run_case(gpu, oracle, shape, T, skew=skew)
    assert got["counts"].max() > 64


@pytest.mark.parametrize("shape,T", [
    # about 90 rows per expert and enough tiles that the 128-row streaming class takes its wide form (four
    # weight slots per block) in the gate/up kernel (64 experts x 9 tiles, the last one ragged in rows and in k)
    (LayerShape("wide4-gate-up", d=328, E=64, top_k=8, inter=1096, shared_inter=200, shared_gate=1, seed=38), 700),
    # the same for the down projection (64 experts x 9 tiles of 512 output rows, the last with 8)
    (LayerShape("wide4-down", d=4104, E=64, top_k=8, inter=520, seed=39), 720),
])
def test_wide_tiles_with_four_weight_slots(gpu, oracle, shape, T):
    got, ref = run_case(gpu, oracle, shape, T)
    assert ((got["counts"] > 64) & (got["counts"] <= 128)).sum() >= 56


@pytest.mark.parametrize("shape,T", [
    # about 280 rows per expert: a full 256-row block and a last block of a few dozen rows, which the tiled
    # kernels take as a 64-token tile drawn from a counter; ragged contraction lengths and row tiles
    (LayerShape("narrow-tail", d=328, E=4, top_k=2, inter=520, seed=46), 560),
    (LayerShape("narrow-tail-shared", d=264, E=2, top_k=1, inter=200, shared_inter=136, shared_gate=1, seed=47), 580),
    (LayerShape("narrow-tail-fp8", d=336, E=4, top_k=2, inter=528, weight_format=1, seed=48), 560),
    # 16 experts with 512 +- 20 rows: narrow tiles beside a schedule of many whole tiles
    (LayerShape("narrow-tail-many", d=192, E=16, top_k=2, inter=1160, seed=49), 4096),
])
def test_last_blocks_with_few_rows(gpu, oracle, shape, T):
    tokens = None
    if T > 1000:
        w = synth.make_layer(shape, threads=16)
        x = synth.make_tokens(shape, T, point=0)
        tokens = tokens_from_permutation(oracle, shape, w, x, budget=40)
        got, ref = run_case(gpu, oracle, shape, T, tokens=tokens, weights=w, x=x)
    else:
        got, ref = run_case(gpu, oracle, shape, T)
    c = got["counts"]
    assert ((c > 256) & ((c - 1) % 256 < 64)).sum() >= 1


@pytest.mark.parametrize("shape,T", [
    # many row tiles and few stages: the persistent schedule cuts gate/up tiles (routed and shared region)
    (LayerShape("cut-gate-up", d=192, E=1, top_k=1, inter=12800, shared_inter=6400, seed=35), 520),
    # many token blocks x row tiles of the down projection: cuts there
    (LayerShape("cut-down", d=2048, E=1, top_k=1, inter=192, seed=36), 8500),
    # 600 rows per expert: the tiled shared expert is not split into k-parts, so its down projection is two
    # runs of 512 stages beside routed runs of one stage; the runs are cut into the shares of all the teams,
    # and the second kernel adds that many pieces
    (LayerShape("cut-shared-down", d=512, E=1, top_k=1, inter=64, shared_inter=32768, seed=37), 600),
])
def test_tiles_cut_by_the_schedule(gpu, oracle, shape, T):
    # On a 256-CU device the tiled kernels run 64 teams; with more runs of 4 tiles than teams and an
    # uneven split, shares end inside tiles and the second kernel adds the pieces.
    rng = np.random.default_rng(5)
    tokens = np.sort(rng.choice(T, size=48, replace=False)).astype(np.int32)
    run_case(gpu, oracle, shape, T, tokens=tokens)


@pytest.mark.parametrize("shape,T", [
    # group-limited selection (the routing rule of config 4's model family): one and several experts per lane,
    # sigmoid and softmax scores, the fused top-K + permutation kernel (T <= 32) and the separate ones
    (LayerShape("grp-16", d=256, E=16, top_k=4, inter=128, score_func=1, n_group=4, topk_group=2, seed=41), 23),
    (LayerShape("grp-256", d=256, E=256, top_k=8, inter=64, score_func=1, n_group=8, topk_group=4, seed=42), 29),
    (LayerShape("grp-256", d=256, E=256, top_k=8, inter=64, score_func=1, n_group=8, topk_group=4, seed=42), 150),
    (LayerShape("grp-softmax", d=128, E=24, top_k=5, inter=64, n_group=4, topk_group=2, renormalize=0, seed=43), 70),
    (LayerShape("grp-320", d=128, E=320, top_k=6, inter=64, score_func=1, n_group=64, topk_group=3, seed=44), 40),
    (LayerShape("grp-single", d=128, E=8, top_k=2, inter=64, score_func=1, n_group=8, topk_group=2, seed=45), 9),
])
def test_group_limited_selection(gpu, oracle, shape, T):
    got, ref = run_case(gpu, oracle, shape, T, skew=0.8)
    gs = shape.E // shape.n_group
    assert all(len(set((got["ids"][t] // gs).tolist())) <= shape.topk_group for t in range(T))


@pytest.mark.parametrize("T", [1, 5, 16, 17, 40, 64, 130, 300])
def test_fp8_weights_small_shapes(gpu, oracle, T):
    # expert weights as E4M3 codes with a scale per output row (64-row small tiles in the streaming kernels up to 16
    # rows per expert, the 64-row wide class up to 64; beyond that, and the shared expert beyond 64 tokens, the
    # MFMA-tiled kernels, which widen the codes on their way into LDS); ragged sizes (multiples of 16), gated shared expert
    shape = LayerShape("fp8-ragged", d=400, E=12, top_k=3, inter=208, shared_inter=144, shared_gate=1,
                       weight_format=1, seed=51)
    run_case(gpu, oracle, shape, T)


@pytest.mark.parametrize("shape,T,skew", [
    (LayerShape("fp8-sigmoid", d=512, E=40, top_k=6, inter=272, shared_inter=80, score_func=1, weight_format=1, seed=52), 23, 0.0),
    (LayerShape("fp8-no-shared", d=1040, E=24, top_k=2, inter=1040, weight_format=1, seed=53), 33, 0.0),
    (LayerShape("fp8-one-block", d=512, E=16, top_k=4, inter=512, weight_format=1, seed=54), 12, 0.0),   # one-slot tiles
    (LayerShape("fp8-skewed", d=256, E=16, top_k=2, inter=128, shared_inter=64, shared_gate=1, weight_format=1, seed=55), 200, 2.0),
    (LayerShape("fp8-many-rows", d=128, E=2, top_k=1, inter=144, weight_format=1, seed=56), 700, 0.0),
])
def test_fp8_weights_variants(gpu, oracle, shape, T, skew):
    run_case(gpu, oracle, shape, T, skew=skew)


def test_fp8_weights_benchmark_shapes_full_size(gpu, oracle):
    # benchmark configs 1 and 2 with their expert weights quantised to E4M3 (row scales), full size: T = 16 with
    # every token compared; T = 64 (the shared expert in the 64-row wide class) and T = 200 (experts with more than
    # 64 rows and the shared expert in the MFMA-tiled kernels) on tokens chosen from the permutation
    for name, pt in (("qwen1.5-moe-a2.7b", 180), ("qwen2-57b-a14b", 280)):
        shape = dataclasses.replace(PRESETS[name], name=name + "-fp8", weight_format=1)
        w = synth.make_layer(shape, threads=16)
        layer = gpu.GpuLayer(shape, w)
        run_case(gpu, oracle, shape, 16, point=pt, weights=w, layer=layer)
        for i, T in enumerate((64, 200)):
            x = synth.make_tokens(shape, T, point=pt + 1 + i)
            run_case(gpu, oracle, shape, T, tokens=tokens_from_permutation(oracle, shape, w, x), point=pt + 1 + i,
                     weights=w, layer=layer)
        del layer, w


def test_fp8_weights_mixtral_shape_full_size_tiled(gpu, oracle):
    # benchmark config 3 with E4M3 expert weights at T = 1024 and 2048: 256 and 512 rows per expert, the
    # MFMA-tiled kernels with the codes widened on the way into LDS, evenly split blocks, cut runs
    name = "mixtral-8x7b"
    shape = dataclasses.replace(PRESETS[name], name=name + "-fp8", weight_format=1)
    w = synth.make_layer(shape, threads=16)
    layer = gpu.GpuLayer(shape, w)
    for i, T in enumerate((1024, 2048)):
        x = synth.make_tokens(shape, T, point=380 + i)
        run_case(gpu, oracle, shape, T, tokens=tokens_from_permutation(oracle, shape, w, x), point=380 + i,
                 weights=w, layer=layer, x=x)
    del layer, w


def _random_shape(i):
    """A small layer with every size drawn at random (seeded): odd row counts, ragged contraction lengths,
    all expert classes, with and without shared expert, groups, bias."""
    rng = np.random.default_rng(1000 + i)
    E = int(rng.integers(1, 41))
    K = int(rng.integers(1, min(E, 8) + 1))
    kw = dict(d=8 * int(rng.integers(8, 66)), E=E, top_k=K, inter=8 * int(rng.integers(2, 40)),
              score_func=int(rng.integers(0, 2)), renormalize=int(rng.integers(0, 2)), seed=500 + i)
    if rng.random() < 0.6:
        kw.update(shared_inter=8 * int(rng.integers(2, 50)), shared_gate=int(rng.integers(0, 2)))
    divs = [g for g in range(2, E + 1) if E % g == 0 and g <= 64]
    if divs and rng.random() < 0.3:
        G = int(rng.choice(divs))
        need = -(-K // (E // G))
        kw.update(n_group=G, topk_group=int(rng.integers(need, G + 1)))
    T = int(rng.choice([1, 3, 9, 16, 17, 40, 64, 65, 129, 200, 333, 600]))
    return LayerShape(f"rnd{i}", **kw), T, float(rng.choice([0.0, 0.0, 1.0, 2.5]))


@pytest.mark.parametrize("i", range(24))
def test_random_small_shapes(gpu, oracle, i):
    shape, T, skew = _random_shape(i)
    run_case(gpu, oracle, shape, T, skew=skew)


def test_skewed_routing_and_bias(gpu, oracle):
    shape = LayerShape("skew", d=256, E=64, top_k=8, inter=128, shared_inter=256, shared_gate=1, seed=16)
    got, ref = run_case(gpu, oracle, shape, 48, skew=1.5)
    assert got["n_active"] < 64


def test_zero_tokens_tie_break(gpu, oracle):
    shape = LayerShape("zeros", d=256, E=8, top_k=3, inter=128, seed=17)
    got, _ = run_case(gpu, oracle, shape, 9, zero_x=True)
    assert (got["ids"] == np.arange(3)[None, :]).all()
    assert (got["out_bf16"] == 0).all()


def test_duplicate_router_rows_tie_break(gpu, oracle):
    shape = LayerShape("dups", d=256, E=8, top_k=3, inter=64, seed=18)
    w = synth.make_layer(shape)
    w["w_router"][5] = w["w_router"][2]
    w["w_router"][7] = w["w_router"][2]
    run_case(gpu, oracle, shape, 40, weights=w)


def test_keys_on_fp32_rounding_boundaries(gpu, oracle):
    # logits that are exact in fp64 whatever the summation order and sit on, just above and well above an
    # fp32 rounding boundary (tests/test_oracle_layer.py pins the oracle's answer by hand)
    from tests.test_oracle_layer import rounding_boundary_router
    shape, w, x, want = rounding_boundary_router()
    got, ref = run_case(gpu, oracle, shape, x.shape[0], weights=w, x=x)
    assert (got["ids"] == want[None, :]).all()


def test_empty_batch(gpu, oracle):
    shape = PRESETS["tiny"]
    w = synth.make_layer(shape)
    layer = gpu.GpuLayer(shape, w)
    got = layer.forward(synth.make_tokens(shape, 0))
    assert got["n_active"] == 0 and (got["counts"] == 0).all() and (got["offsets"] == 0).all()


def test_standalone_route_and_permute(gpu, oracle):
    import torch
    import paper_2505_19645_amd as moesd
    shape = LayerShape("rp", d=512, E=60, top_k=4, inter=64, seed=19)
    r = synth.make_router(shape, skew_std=0.5)
    for T in (1, 7, 64, 700):
        say(f"[case] route/permute T={T}")
        x = synth.make_tokens(shape, T, point=T)
        ids_ref, w_ref, _ = oracle.route(shape, x, r["w_router"], r["router_bias"])
        desc = moesd.make_desc(shape)
        xd, wr, b = gpu.to_dev_bf16(x), gpu.to_dev_bf16(r["w_router"]), gpu.to_dev(r["router_bias"])
        ids = torch.empty((T, 4), dtype=torch.int32, device="cuda")
        w = torch.empty((T, 4), dtype=torch.float32, device="cuda")
        ws = torch.empty(moesd.moesd_workspace_bytes(desc, T), dtype=torch.uint8, device="cuda")
        moesd.moesd_route(desc, xd, wr, b, T, ids, w, ws)
        assert np.array_equal(ids.cpu().numpy(), ids_ref)
        np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=2e-7, atol=1e-9)
        np.testing.assert_allclose(w.cpu().numpy().sum(1), 1.0, atol=1e-6)
        counts = torch.empty(60, dtype=torch.int32, device="cuda")
        offsets = torch.empty(61, dtype=torch.int32, device="cuda")
        perm = torch.empty(T * 4, dtype=torch.int32, device="cuda")
        inv = torch.empty(T * 4, dtype=torch.int32, device="cuda")
        na = torch.empty(1, dtype=torch.int32, device="cuda")
        for rep in range(3):                      # determinism: identical bytes every time
            moesd.moesd_permute(60, 4, T, ids, counts, offsets, perm, inv, na)
            pr = oracle.permute(60, 4, ids_ref)
            assert np.array_equal(counts.cpu().numpy(), pr["counts"])
            assert np.array_equal(offsets.cpu().numpy(), pr["offsets"])
            assert np.array_equal(perm.cpu().numpy(), pr["perm"])
            assert np.array_equal(inv.cpu().numpy(), pr["inv"])
            assert int(na.item()) == pr["n_active"]


@pytest.mark.parametrize("E,K,T", [(256, 8, 2560), (8, 2, 4096), (1024, 32, 300), (64, 8, 1), (5, 5, 64)])
def test_permute_large_and_extreme(gpu, oracle, E, K, T):
    import torch
    import paper_2505_19645_amd as moesd
    say(f"[case] permute E={E} K={K} T={T}")
    rng = np.random.default_rng(E + T)
    # Zipf-like expert popularity, K distinct experts per token
    p = 1.0 / np.arange(1, E + 1)
    p /= p.sum()
    ids = np.stack([rng.choice(E, size=K, replace=False, p=p) for _ in range(T)]).astype(np.int32)
    pr = oracle.permute(E, K, ids)
    idd = gpu.to_dev(ids)
    counts = torch.empty(E, dtype=torch.int32, device="cuda")
    offsets = torch.empty(E + 1, dtype=torch.int32, device="cuda")
    perm = torch.empty(T * K, dtype=torch.int32, device="cuda")
    inv = torch.empty(T * K, dtype=torch.int32, device="cuda")
    na = torch.empty(1, dtype=torch.int32, device="cuda")
    moesd.moesd_permute(E, K, T, idd, counts, offsets, perm, inv, na)
    assert np.array_equal(counts.cpu().numpy(), pr["counts"])
    assert np.array_equal(offsets.cpu().numpy(), pr["offsets"])
    assert np.array_equal(perm.cpu().numpy(), pr["perm"])
    assert np.array_equal(inv.cpu().numpy(), pr["inv"])
    assert int(na.item()) == pr["n_active"]


def full_case(gpu, oracle, name, T, point, skew=0.0, all_tokens=False):
    shape = PRESETS[name]
    w, layer = full_size_weights(name, gpu)
    if skew > 0.0:
        w = dict(w)
        w["router_bias"] = synth.make_router(shape, skew)["router_bias"]
        layer = layer.with_router_bias(w["router_bias"])
    x = synth.make_tokens(shape, T, point=point)
    tokens = None if all_tokens else tokens_from_permutation(oracle, shape, w, x)
    return run_case(gpu, oracle, shape, T, skew=skew, tokens=tokens, point=point, weights=w, layer=layer)


@pytest.mark.parametrize("T", [1, 4, 16])
def test_qwen15_shape_full_size_few_tokens(gpu, oracle, T):
    # benchmark config 1 at full size, T <= 16: shared expert in the small-tile class, top-K and permutation
    # fused in one workgroup; every token compared
    full_case(gpu, oracle, "qwen1.5-moe-a2.7b", T, point=150 + T, all_tokens=True)


def test_qwen15_shape_full_size_sampled_tokens(gpu, oracle):
    # benchmark config 1 at full size, T = 64 (B=16, gamma=3): all routing outputs bit-exact, every token compared
    full_case(gpu, oracle, "qwen1.5-moe-a2.7b", 64, point=163, all_tokens=True)
    # T = 256 (B=64, gamma=3): routed experts in 64-row wide tiles, the shared expert streamed in four token blocks;
    # from here on the compared tokens are chosen from the oracle's permutation (tile borders, every class)
    full_case(gpu, oracle, "qwen1.5-moe-a2.7b", 256, point=164)
    # T = 320: the shared expert still streamed (five token blocks); T = 640 (B=128, gamma=4, the largest of this
    # shape's sweep): routed experts in wide tiles, some beyond 64 rows, the shared expert in the MFMA-tiled kernels
    full_case(gpu, oracle, "qwen1.5-moe-a2.7b", 320, point=165)
    full_case(gpu, oracle, "qwen1.5-moe-a2.7b", 640, point=166)


@pytest.mark.parametrize("T", [1, 4, 16])
def test_qwen2_shape_full_size_few_tokens(gpu, oracle, T):
    # benchmark config 2 at full size, T <= 16 (the shared expert, 20480 wide, in small tiles), every token compared
    full_case(gpu, oracle, "qwen2-57b-a14b", T, point=250 + T, all_tokens=True)


def test_qwen2_shape_full_size_sampled_tokens(gpu, oracle):
    # benchmark config 2 at full size (3.5 GB of expert weights, 0.44 GB shared expert), T = 64
    shape = PRESETS["qwen2-57b-a14b"]
    got, _ = full_case(gpu, oracle, "qwen2-57b-a14b", 64, point=263)
    w, layer = full_size_weights("qwen2-57b-a14b", gpu)
    # At this size both streaming kernels hand out the tail of their small tiles from a counter, so which
    # workgroup computes which tile differs from launch to launch; the bytes of the result must not.
    x = synth.make_tokens(shape, 64, point=263)
    for rep in range(3):
        again = layer.forward(x)
        assert np.array_equal(again["out_f32"], got["out_f32"]) and np.array_equal(again["out_bf16"], got["out_bf16"])
        assert np.array_equal(again["perm"], got["perm"]) and again["n_active"] == got["n_active"]
    # the largest T of this shape's sweep (B=256, gamma=4): about 160 rows per expert, every kernel class at once
    full_case(gpu, oracle, "qwen2-57b-a14b", 1280, point=264)
    # the compute-bound points the benchmark times beyond the sweep: 256 and 512 rows per expert on average
    # (blocks split evenly, last blocks of a few rows, the shared expert in the tiled kernels without k-parts)
    full_case(gpu, oracle, "qwen2-57b-a14b", 2048, point=265)
    full_case(gpu, oracle, "qwen2-57b-a14b", 4096, point=266)


@pytest.mark.parametrize("T", [16, 64, 1280])
def test_qwen2_shape_full_size_skewed_routing(gpu, oracle, T):
    # the skewed variant of benchmark config 2: per-expert logit bias N(0, 1.5), Zipf-like expert loads (a few
    # experts with most of the rows, many with none): classes mixed inside one launch at every T
    got, _ = full_case(gpu, oracle, "qwen2-57b-a14b", T, point=270 + T, skew=1.5)
    uniform = PRESETS["qwen2-57b-a14b"]
    if T == 16:   # visibly fewer activated experts than uniform routing gives (Eq. N(t): 56.4 at T = 16)
        assert got["n_active"] < 50
    assert got["counts"].max() > 2 * T * uniform.top_k / uniform.E


@pytest.mark.parametrize("shape,T", [
    # d = 512: one 512-element block per gate/up tile, so a unit is three tiles and every step carries the extra
    # barrier of a one-slot tile; about 220 active experts x 52 row tiles = 11500 small tiles (45 per workgroup)
    (LayerShape("drawn-1slot", d=512, E=256, top_k=8, inter=832, shared_inter=0, seed=31), 64),
    # I = 1000: two blocks per down tile, the second ragged, units of two tiles (about 146 experts x 38 row tiles, 43 slots
    # per workgroup); gate/up: three blocks, the last ragged; shared expert with a gate in the wide class
    (LayerShape("drawn-2slot", d=1200, E=160, top_k=8, inter=1000, shared_inter=520, shared_gate=1, seed=32), 48),
])
def test_drawn_units_with_short_tiles(gpu, oracle, shape, T):
    # Lines of small tiles long enough for the streaming kernels to hand out their tail from a counter (at least
    # 12 tiles and 40 slots per workgroup on 256 CUs), with tiles of one and of two slots: the unit sizes, the
    # mailbox between the multiplying and the loading waves and the one-slot tiles' extra barrier all take part.
    w = synth.make_layer(shape, threads=16)
    tokens = [0, T // 3, T - 1]
    got, _ = run_case(gpu, oracle, shape, T, tokens=tokens, point=77, weights=w)
    again = gpu.GpuLayer(shape, w).forward(synth.make_tokens(shape, T, point=77))
    assert np.array_equal(again["out_f32"], got["out_f32"])


@pytest.mark.parametrize("T", [1, 4, 16])
def test_mixtral_shape_full_size_few_tokens(gpu, oracle, T):
    # benchmark config 3 at full size, T <= 16 (no shared expert, 8 experts of 352 MB), every token compared
    full_case(gpu, oracle, "mixtral-8x7b", T, point=350 + T, all_tokens=True)


def test_mixtral_shape_full_size_tiled_sampled_tokens(gpu, oracle):
    # benchmark config 3 at full size and its largest T (4096: about 1024 rows per expert, the MFMA-tiled
    # kernels with the persistent schedule the benchmark's compute-bound point times); routing bit-exact on
    # all tokens, output on tokens chosen from the permutation (first / last rows, 64- and 256-row borders)
    full_case(gpu, oracle, "mixtral-8x7b", 4096, point=363)
    # T = 128 (about 32 rows per expert): every expert in wide tiles, several thousand of them
    full_case(gpu, oracle, "mixtral-8x7b", 128, point=364)
    # T = 256 and 1024 of this shape's sweep: 64 and 256 rows per expert
    full_case(gpu, oracle, "mixtral-8x7b", 256, point=365)
    full_case(gpu, oracle, "mixtral-8x7b", 1024, point=366)
    # T = 2048 and 8192, the other compute-bound points of the benchmark: 512 and 2048 rows per expert
    full_case(gpu, oracle, "mixtral-8x7b", 2048, point=367)
    full_case(gpu, oracle, "mixtral-8x7b", 8192, point=368)


@pytest.mark.parametrize("T", [1, 4, 16])
def test_deepseek_shape_full_size_few_tokens(gpu, oracle, T):
    # benchmark config 4 at full size (sigmoid scores, 256 experts, ungated shared expert), every token compared
    full_case(gpu, oracle, "deepseek-v3", T, point=450 + T, all_tokens=True)


def test_deepseek_shape_full_size_sampled_tokens(gpu, oracle):
    # benchmark config 4 at full size (22.6 GB of expert weights): T = 64 (the benchmark's headline point) and the
    # largest T of its sweep (2560: about 80 rows per expert, shared expert through the tiled kernels)
    full_case(gpu, oracle, "deepseek-v3", 64, point=463)
    full_case(gpu, oracle, "deepseek-v3", 2560, point=464)
