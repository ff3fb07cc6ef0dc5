"""CPU-side checks of the C-ABI library: it loads, exports what the header
declares, its closed forms agree with the paper-pinned oracle, and argument
validation returns the documented codes before anything touches a GPU."""
import ctypes as C
import math
import os
import re

import pytest

import paper_2505_19645_amd as moesd
from paper_2505_19645_amd import binding
from paper_2505_19645_amd.synth import PRESETS, LayerShape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "moesd.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(moesd_[a-z_0-9]+)\s*\(", hdr))
    assert {"moesd_route", "moesd_permute", "moesd_moe_forward",
            "moesd_expected_active_experts"} <= declared
    L = binding.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(binding.EXPORTS)


def test_closed_forms_match_oracle(oracle):
    for E, K in [(8, 2), (60, 4), (64, 8), (256, 8), (62, 6), (16, 16), (1024, 1)]:
        for t in [0, 1, 2, 3, 16, 64, 257, 4096, 10**6]:
            a = moesd.moesd_expected_active_experts(E, K, t)
            b = oracle.expected_active_experts(E, K, t)
            assert a == pytest.approx(b, rel=1e-12, abs=1e-12), (E, K, t)
            a = moesd.moesd_expected_tokens_per_expert(E, K, t)
            b = oracle.expected_tokens_per_expert(E, K, t)
            assert a == pytest.approx(b, rel=1e-12, abs=1e-12), (E, K, t)
        for tau in [0.0, 0.5, 0.9, 0.95, 0.99, 0.999999]:
            assert moesd.moesd_token_threshold(E, K, tau) == oracle.token_threshold(E, K, tau)
    assert math.isnan(moesd.moesd_expected_active_experts(0, 0, 1))
    assert math.isnan(moesd.moesd_expected_active_experts(8, 9, 1))
    assert math.isnan(moesd.moesd_expected_tokens_per_expert(8, 2, -1))
    assert moesd.moesd_token_threshold(8, 0, 0.95) == -1
    assert moesd.moesd_token_threshold(8, 2, 1.0) == -1
    # the benchmark shapes (tau = 0.95) and N(1) = K
    assert [moesd.moesd_token_threshold(E, K, 0.95) for E, K in [(8, 2), (60, 4), (64, 8), (256, 8)]] \
        == [11, 44, 23, 95]
    assert moesd.moesd_expected_active_experts(60, 4, 1) == pytest.approx(4.0, abs=1e-12)


def test_workspace_bytes_and_descriptor_validation():
    for name, shape in PRESETS.items():
        d = moesd.make_desc(shape)
        b1 = moesd.moesd_workspace_bytes(d, 1)
        b64 = moesd.moesd_workspace_bytes(d, 64)
        assert 0 < b1 < b64 and b64 % 256 == 0
        # lower bound: the fp32 per-slot outputs of the down projection
        assert b64 >= 64 * shape.top_k * shape.d * 4
    assert moesd.moesd_workspace_bytes(moesd.make_desc(LayerShape("b", 12, 8, 2, 16)), 4) == 0   # d % 8
    assert moesd.moesd_workspace_bytes(moesd.make_desc(LayerShape("b", 16, 8, 9, 16)), 4) == 0   # K > E
    assert moesd.moesd_workspace_bytes(moesd.make_desc(PRESETS["tiny"]), -1) == 0


def _fwd(desc, T, ws_bytes=1 << 20, wt=None, x=0x1000, out=0x1000, ws=0x1000):
    # fake, never dereferenced: every case below is rejected before any launch
    w = binding.Weights()
    for n, _ in binding.Weights._fields_:
        setattr(w, n, 0x1000)
    if wt:
        for k, v in wt.items():
            setattr(w, k, v)
    return binding.moesd_moe_forward(desc, w, x, T, out, ws, workspace_bytes=ws_bytes, stream=0,
                                     check=False)


def test_forward_argument_errors_need_no_gpu():
    tiny = PRESETS["tiny"]
    d = moesd.make_desc(tiny)
    assert _fwd(d, -1) == binding.INVALID_ARG
    assert _fwd(d, 16, ws_bytes=16) == binding.WORKSPACE_TOO_SMALL
    assert _fwd(d, 16, ws=0x1010) == binding.INVALID_ARG                       # misaligned workspace
    assert _fwd(d, 16, x=None) == binding.INVALID_ARG
    assert _fwd(d, 16, out=None) == binding.INVALID_ARG
    assert _fwd(d, 16, wt={"w_gate": None}) == binding.INVALID_ARG
    bad = moesd.make_desc(LayerShape("b", 256, 8, 0, 512))
    assert _fwd(bad, 16) == binding.INVALID_ARG
    bad = moesd.make_desc(LayerShape("b", 256, 2048, 2, 512))
    assert _fwd(bad, 16) == binding.UNSUPPORTED                                 # E > MOESD_MAX_E
    bad = moesd.make_desc(LayerShape("b", 256, 8, 2, 512, score_func=7))
    assert _fwd(bad, 16) == binding.UNSUPPORTED
    bad = moesd.make_desc(LayerShape("b", 256, 8, 2, 516))
    assert _fwd(bad, 16) == binding.INVALID_ARG                                 # inter % 8
    for G, Gk in ((3, 1), (4, 0), (4, 5), (8, 1)):                              # E % G; no group; > G; K > Gk*E/G
        bad = moesd.make_desc(LayerShape("b", 256, 8, 2, 512, n_group=G, topk_group=Gk))
        assert _fwd(bad, 16) == binding.INVALID_ARG, (G, Gk)
    bad = moesd.make_desc(LayerShape("b", 256, 256, 2, 512, n_group=128, topk_group=4))
    assert _fwd(bad, 16) == binding.UNSUPPORTED                                 # more than 64 groups
    ok = moesd.make_desc(LayerShape("b", 256, 8, 2, 512, n_group=4, topk_group=2))
    assert moesd.moesd_workspace_bytes(ok, 16) > 0
    sh = moesd.make_desc(PRESETS["qwen1.5-moe-a2.7b"])
    assert _fwd(sh, 16, ws_bytes=1 << 30, wt={"ws_down": None}) == binding.INVALID_ARG
    assert _fwd(sh, 16, ws_bytes=1 << 30, wt={"w_shared_gate": None}) == binding.INVALID_ARG
    assert _fwd(d, 2**30) == binding.INVALID_ARG                                # T*K >= 2^31
    big = moesd.make_desc(PRESETS["deepseek-v3"])
    assert _fwd(big, 300000, ws_bytes=1 << 46) == binding.UNSUPPORTED           # T*d*2 >= 2^32, before any launch
    assert moesd.moesd_workspace_bytes(big, 300000) == 0
    assert binding.moesd_permute(8, 9, 4, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, stream=0,
                                 check=False) == binding.INVALID_ARG
    assert binding.moesd_permute(8, 2, 4, 0x1000, None, 0x1000, 0x1000, 0x1000, 0x1000, stream=0,
                                 check=False) == binding.INVALID_ARG
    assert binding.moesd_route(d, None, 0x1000, None, 4, 0x1000, 0x1000, 0x1000, 1 << 20, stream=0,
                               check=False) == binding.INVALID_ARG
    # 8-bit expert weights: unknown format, sizes that are not multiples of 16, missing row scales
    bad = moesd.make_desc(LayerShape("b", 256, 8, 2, 512, weight_format=2))
    assert _fwd(bad, 16) == binding.UNSUPPORTED
    bad = moesd.make_desc(LayerShape("b", 264, 8, 2, 512, weight_format=1))
    assert _fwd(bad, 16) == binding.INVALID_ARG
    bad = moesd.make_desc(LayerShape("b", 256, 8, 2, 520, weight_format=1))
    assert _fwd(bad, 16) == binding.INVALID_ARG
    q = moesd.make_desc(LayerShape("q", 256, 8, 2, 512, shared_inter=64, weight_format=1))
    assert _fwd(q, 16, ws_bytes=1 << 30, wt={"w_up_scale": None}) == binding.INVALID_ARG
    assert _fwd(q, 16, ws_bytes=1 << 30, wt={"ws_down_scale": None}) == binding.INVALID_ARG
    # the MFMA-tiled kernels (and their partial-sum space) come in above 128 tokens, whatever the weight format
    assert moesd.moesd_workspace_bytes(q, 128) < (64 << 20) < (128 << 20) <= moesd.moesd_workspace_bytes(q, 129)
    # the entry point on the library's static scratch array: the same checks, and sizes beyond the array
    wq = binding.Weights()
    for n, _ in binding.Weights._fields_:
        setattr(wq, n, 0x1000)
    assert binding.moesd_moe_forward_static(sh, wq, 0x1000, 2000, 0x1000, stream=0, check=False) == binding.WORKSPACE_TOO_SMALL
    assert binding.moesd_moe_forward_static(sh, wq, None, 16, 0x1000, stream=0, check=False) == binding.INVALID_ARG
    assert binding.moesd_moe_forward_static(sh, wq, 0x1000, -1, 0x1000, stream=0, check=False) == binding.INVALID_ARG
    assert moesd.moesd_workspace_bytes(sh, 64) <= binding.STATIC_SCRATCH_BYTES < moesd.moesd_workspace_bytes(sh, 2000)
    hdr = open(os.path.join(ROOT, "include", "moesd.h")).read()
    assert int(re.search(r"MOESD_STATIC_SCRATCH_BYTES \((\d+)u << 20\)", hdr).group(1)) << 20 == binding.STATIC_SCRATCH_BYTES
    assert binding.status_string(binding.WORKSPACE_TOO_SMALL) == "workspace too small"
    with pytest.raises(binding.MoesdError):
        binding.moesd_moe_forward(d, binding.Weights(), 0x1000, -1, 0x1000, 0x1000,
                                  workspace_bytes=1 << 20, stream=0)


def test_nonuniform_activation_count_against_the_oracle(oracle):
    import numpy as np
    rng = np.random.default_rng(4)
    for E, K, t in ((60, 4, 64), (256, 8, 1), (8, 8, 5), (40, 3, 0), (16, 2, 100000)):
        p = rng.random(E) ** 3
        p *= K / p.sum()
        p = np.minimum(p, 1.0)
        a = moesd.moesd_expected_active_experts_p(p.tolist(), t)
        b = oracle.expected_active_experts_p(p, t)
        assert abs(a - b) <= 1e-12 * max(1.0, b)
        u = moesd.moesd_expected_active_experts_p([K / E] * E, t)
        assert abs(u - moesd.moesd_expected_active_experts(E, K, t)) <= 1e-10 * max(1.0, u)
        if t > 1 and K < E:
            assert a < u                                    # any other p with the same sum activates fewer
    assert math.isnan(moesd.moesd_expected_active_experts_p([0.5, 1.5], 2))
    assert moesd.moesd_expected_active_experts_p([1.0, 0.0], 0) == 0.0
    assert moesd.moesd_expected_active_experts_p([1.0, 0.0], 3) == 1.0
