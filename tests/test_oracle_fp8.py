"""Pins for the low-precision expert weights of the oracle (oracle/moe_oracle.c): the E4M3 decoder
against a table of all 256 code points written with rational arithmetic (tests/golden/fp8_e4m3_values.txt,
OCP OFP8 specification Sec. 5) and against a library cast; the fp8 layer against the (separately pinned)
bf16 layer on weights that both formats hold exactly, and against numpy matrix products for general
scales.  The paper itself only says that the floor of the expert-loading term scales with the weights'
bit width (Appendix C.2); the format is the public OFP8 one.  CPU only."""
import dataclasses
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2505_19645_amd import synth
from paper_2505_19645_amd.synth import LayerShape, bf16_bits_to_f32, f32_to_bf16_bits

HERE = os.path.dirname(os.path.abspath(__file__))


def golden_table():
    vals = {}
    for line in open(os.path.join(HERE, "golden", "fp8_e4m3_values.txt")):
        if line.startswith("#"):
            continue
        code, v = line.split()
        vals[int(code, 16)] = None if v == "nan" else Fraction(v)
    assert len(vals) == 256
    return vals


def test_decoder_matches_the_table_of_all_code_points(oracle):
    dec = oracle.fp8_decode(np.arange(256, dtype=np.uint8))
    for code, want in golden_table().items():
        if want is None:
            assert np.isnan(dec[code]), code
        else:
            assert Fraction(float(dec[code])) == want, (code, dec[code], want)


def test_decoder_matches_a_library_cast(oracle):
    torch = pytest.importorskip("torch")
    if not hasattr(torch, "float8_e4m3fn"):
        pytest.skip("this torch has no float8_e4m3fn")
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    dec = oracle.fp8_decode(codes)
    assert np.array_equal(np.isnan(dec), np.isnan(lib))
    assert np.array_equal(dec[~np.isnan(dec)], lib[~np.isnan(lib)])


def test_decoder_properties(oracle):
    dec = oracle.fp8_decode(np.arange(256, dtype=np.uint8))
    pos, neg = dec[:128], dec[128:]
    assert np.isnan(pos[127]) and np.isnan(neg[127]) and np.isnan(dec).sum() == 2      # no infinities, two NaNs
    assert np.array_equal(neg[:127], -pos[:127]) and pos[0] == 0.0
    assert (np.diff(pos[:127]) > 0).all()                         # code order is value order
    assert pos[126] == 448.0 and pos[1] == 2.0 ** -9 and pos[8] == 2.0 ** -6          # max, smallest subnormal, smallest normal
    assert np.array_equal(pos[8:119] * 2, pos[16:127])            # one exponent step doubles every value
    assert np.array_equal(np.diff(pos[:9]), np.full(8, 2.0 ** -9))  # subnormals and the first binade: equal spacing


def random_fp8_layer(shape, rng, pow2_scales):
    """Random finite E4M3 codes and row scales (powers of two, or arbitrary positive fp32)."""
    d, E, I, S = shape.d, shape.E, shape.inter, shape.shared_inter
    w = synth.make_router(shape, 0.7)
    w["w_shared_gate"] = synth.make_shared(shape)["w_shared_gate"]

    def codes(*dims):
        c = rng.integers(0, 256, size=dims, dtype=np.uint8)
        c[(c & 0x7F) == 0x7F] = 0x38                              # never a NaN code
        return c

    def scales(*dims):
        if pow2_scales:
            return (2.0 ** rng.integers(-9, -3, size=dims)).astype(np.float32)
        return rng.uniform(2e-4, 3e-3, size=dims).astype(np.float32)

    for name, dims in (("w_gate", (E, I, d)), ("w_up", (E, I, d)), ("w_down", (E, d, I)),
                       ("ws_gate", (S, d)), ("ws_up", (S, d)), ("ws_down", (d, S))):
        if name.startswith("ws_") and S == 0:
            w[name] = w[name + "_scale"] = None
            continue
        w[name] = codes(*dims)
        w[name + "_scale"] = scales(*dims[:-1])
    return w


def dequantized_bf16(oracle, w):
    """The same layer as bf16 words; exact when every scale is a power of two (E4M3 has 4 significant
    bits, bf16 has 8)."""
    out = {k: v for k, v in w.items() if not k.endswith("_scale")}
    for k in ("w_gate", "w_up", "w_down", "ws_gate", "ws_up", "ws_down"):
        if w.get(k) is None:
            continue
        val = oracle.fp8_decode(w[k]) * w[k + "_scale"].astype(np.float64)[..., None]
        bits = f32_to_bf16_bits(val.astype(np.float32))
        assert np.array_equal(bf16_bits_to_f32(bits).astype(np.float64), val)   # nothing was rounded
        out[k] = bits
    return out


@pytest.mark.parametrize("shape", [
    LayerShape("fp8-a", d=64, E=6, top_k=2, inter=48, shared_inter=32, shared_gate=1, weight_format=1, seed=61),
    LayerShape("fp8-b", d=48, E=5, top_k=3, inter=80, score_func=1, weight_format=1, seed=62),
])
def test_fp8_layer_equals_the_bf16_layer_on_weights_both_formats_hold(oracle, shape):
    rng = np.random.default_rng(shape.seed)
    w8 = random_fp8_layer(shape, rng, pow2_scales=True)
    w16 = dequantized_bf16(oracle, w8)
    x = synth.make_tokens(shape, 11, point=3)
    a = oracle.moe_forward(shape, w8, x)
    b = oracle.moe_forward(dataclasses.replace(shape, weight_format=0), w16, x)
    for k in ("ids", "perm", "counts"):
        assert np.array_equal(a[k], b[k])
    assert np.array_equal(a["out"], b["out"])          # same real weights, same sums: the same doubles
    assert np.array_equal(a["out_bf16"], b["out_bf16"])
    assert np.abs(a["out"]).max() > 0


def test_fp8_dense_case_against_matrix_products(oracle):
    # one expert, one slot: out = W_down . (silu(W_gate x) * (W_up x)) with W = decode(code) * scale[row]
    shape = LayerShape("fp8-dense", d=40, E=1, top_k=1, inter=56, weight_format=1, seed=63)
    rng = np.random.default_rng(63)
    w = random_fp8_layer(shape, rng, pow2_scales=False)
    x = synth.make_tokens(shape, 7, point=1)
    got = oracle.moe_forward(shape, w, x)["out"]
    X = bf16_bits_to_f32(x).astype(np.float64)
    tab = {c: (None if v is None else float(v)) for c, v in golden_table().items()}
    deq = lambda k: np.vectorize(tab.get, otypes=[np.float64])(w[k][0]) * w[k + "_scale"][0].astype(np.float64)[:, None]
    g, u = X @ deq("w_gate").T, X @ deq("w_up").T
    want = (g / (1.0 + np.exp(-g)) * u) @ deq("w_down").T
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)
    # scales are per output row: using a matrix's scales along its columns is a different layer
    wrong = (g / (1.0 + np.exp(-g)) * u) @ (np.vectorize(tab.get, otypes=[np.float64])(w["w_down"][0])
                                             * w["w_up_scale"][0].astype(np.float64)[None, :]).T
    assert not np.allclose(got, wrong, rtol=1e-3)


def test_input_preparation_rounds_to_the_nearest_code(oracle):
    # the generator's encoder (inputs only): nearest code, ties to the even code, saturation at 448
    rng = np.random.default_rng(5)
    v = np.concatenate([rng.normal(size=20000) * 100, rng.normal(size=20000) * 0.01, [448.0, 500.0, -1e9, 0.0, 2.0 ** -10]])
    codes = synth.encode_e4m3(v)
    dec = oracle.fp8_decode(codes)
    assert not np.isnan(dec).any()
    grid = oracle.fp8_decode(np.arange(127, dtype=np.uint8))
    clipped = np.clip(np.abs(v), 0, 448.0)
    best = np.abs(grid[None, :] - clipped[:, None]).min(axis=1)
    assert np.array_equal(np.abs(np.abs(dec) - clipped), best)
    assert dec[-1] == 0.0 and dec[-5] == 448.0 and dec[-4] == 448.0 and dec[-3] == -448.0   # 2^-10: tie, even code 0
    torch = pytest.importorskip("torch")
    if hasattr(torch, "float8_e4m3fn"):
        inside = np.abs(v) <= 448.0
        lib = torch.from_numpy(v[inside]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(codes[inside] & 0x7F, lib & 0x7F)
    # row-wise quantisation: the largest entry of a row lands on +-448, the scale is max / 448
    wb = synth.normal_bf16(9, "w_gate", 0, (5, 64), 0.05)
    c, s = synth.quantize_rows_e4m3(wb)
    assert (np.abs(oracle.fp8_decode(c)).max(axis=1) == 448.0).all()
    np.testing.assert_allclose(s, np.abs(bf16_bits_to_f32(wb)).max(axis=1) / 448.0, rtol=1e-6)
