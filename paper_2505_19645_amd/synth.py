"""Seeded synthetic inputs for the MoE layer: shapes, tokens and weights.

This module is the only code shared by the GPU path and the CPU oracle.  It
holds no arithmetic of the method itself: it draws Gaussian numbers, rounds them
to bf16 and hands out the raw 16-bit words, nothing more.

The paper evaluates on trained checkpoints and on prompts from two public
benchmarks (Experiments, "Models and datasets"); neither is needed for the MoE
layer, whose cost depends on the data only through which experts the T rows
activate.  The stand-in is i.i.d. Gaussian data with the layer shapes of the
models the paper names, which gives the near-uniform routing that Sec. 3.2
assumes, plus one variant with a per-expert logit bias for skewed loads.

Every tensor is generated block by block from a counter-based generator
(Philox) keyed by (seed, tensor id, block index), so any expert's slice can be
produced on its own and two callers always get identical bits.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np

# tensor ids: part of the generator key, never renumber
_TID = {
    "x": 1, "w_router": 2, "router_bias": 3, "w_gate": 4, "w_up": 5, "w_down": 6,
    "ws_gate": 7, "ws_up": 8, "ws_down": 9, "w_shared_gate": 10,
}

SCORE_SOFTMAX = 0
SCORE_SIGMOID = 1
WEIGHTS_BF16 = 0
WEIGHTS_FP8_E4M3 = 1


@dataclasses.dataclass(frozen=True)
class LayerShape:
    """Shape of one MoE layer (paper notation: E experts, K per token)."""
    name: str
    d: int
    E: int
    top_k: int
    inter: int
    shared_inter: int = 0
    score_func: int = SCORE_SOFTMAX
    renormalize: int = 1
    shared_gate: int = 0
    routed_scale: float = 1.0
    seed: int = 0
    n_group: int = 0      # > 1: group-limited selection (E experts in n_group consecutive groups)
    topk_group: int = 0   # groups kept per token
    weight_format: int = 0  # 0: bf16 expert weights; 1: E4M3 codes with one fp32 scale per output row

    @property
    def weight_bytes_per_element(self) -> int:
        return 1 if self.weight_format == WEIGHTS_FP8_E4M3 else 2

    @property
    def expert_bytes(self) -> int:
        """Bytes of one routed expert's three matrices (and of their row scales, if any)."""
        scales = (2 * self.inter + self.d) * 4 if self.weight_format == WEIGHTS_FP8_E4M3 else 0
        return 3 * self.d * self.inter * self.weight_bytes_per_element + scales

    @property
    def shared_bytes(self) -> int:
        scales = (2 * self.shared_inter + self.d) * 4 if (self.weight_format == WEIGHTS_FP8_E4M3 and self.shared_inter) else 0
        return 3 * self.d * self.shared_inter * self.weight_bytes_per_element + scales \
            + (self.d * 2 if self.shared_gate else 0)

    @property
    def router_bytes(self) -> int:
        return self.E * self.d * 2


# The five benchmark shapes (index = position in the benchmark's config list).
PRESETS = {
    "tiny": LayerShape("tiny", d=256, E=8, top_k=2, inter=512, seed=0),
    "qwen1.5-moe-a2.7b": LayerShape("qwen1.5-moe-a2.7b", d=2048, E=60, top_k=4, inter=1408,
                                    shared_inter=5632, shared_gate=1, seed=1000),
    "qwen2-57b-a14b": LayerShape("qwen2-57b-a14b", d=3584, E=64, top_k=8, inter=2560,
                                 shared_inter=20480, shared_gate=1, seed=2000),
    "mixtral-8x7b": LayerShape("mixtral-8x7b", d=4096, E=8, top_k=2, inter=14336, seed=3000),
    "deepseek-v3": LayerShape("deepseek-v3", d=7168, E=256, top_k=8, inter=2048,
                              shared_inter=2048, score_func=SCORE_SIGMOID, seed=4000),
}
PRESET_ORDER = ["tiny", "qwen1.5-moe-a2.7b", "qwen2-57b-a14b", "mixtral-8x7b", "deepseek-v3"]


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 words."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 words to fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---- 8-bit weights: preparing the inputs (the layer itself only ever decodes) -------------------
# E4M3 of the OCP OFP8 specification: s eeee mmm, bias 7, subnormals, no infinities, largest finite
# value 448.  The 127 positive finite values in code order:
_E4M3_POS = np.array([(m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
                      for e in range(16) for m in range(8)][:127], dtype=np.float64)
E4M3_MAX = 448.0


def encode_e4m3(a: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of each value (ties to the even code, magnitudes above 448 saturate).
    Works on the fp32 bit patterns: above 2^-6 the fp32 mantissa is rounded to 3 bits (nearest even,
    the carry runs into the exponent by itself); below, the codes are multiples of 2^-9."""
    x = np.ascontiguousarray(a, dtype=np.float32)
    u = x.view(np.uint32)
    sign = ((u >> np.uint32(24)) & np.uint32(0x80)).astype(np.uint8)
    mag = u & np.uint32(0x7FFFFFFF)
    r = mag + np.uint32(0x7FFFF) + ((mag >> np.uint32(20)) & np.uint32(1))   # round to 3 mantissa bits
    code = ((r >> np.uint32(20)).astype(np.int32) - np.int32((127 - 7) << 3))  # rebias: (e - 127 + 7) << 3 | m
    sub = mag < np.uint32(0x3C800000)                                         # |x| < 2^-6: subnormal codes
    if sub.any():
        code[sub] = np.rint(np.abs(x[sub]) * np.float32(512.0)).astype(np.int32)
    np.clip(code, 0, 0x7E, out=code)
    return code.astype(np.uint8) | sign


def quantize_rows_e4m3(w_bits: np.ndarray):
    """bf16 words [..., rows, cols] -> (E4M3 codes, fp32 scales [..., rows]): each row is divided by
    max|row| / 448 (rounded to fp32) and rounded to the nearest code."""
    w = bf16_bits_to_f32(w_bits)
    amax = np.abs(w).max(axis=-1)
    scale = np.where(amax > 0, amax / np.float32(E4M3_MAX), np.float32(1.0)).astype(np.float32)
    w /= scale[..., None]
    return encode_e4m3(w), scale


def _rng(seed: int, tensor: str, block: int) -> np.random.Generator:
    ss = np.random.SeedSequence([int(seed), _TID[tensor], int(block)])
    return np.random.Generator(np.random.Philox(ss))


def normal_f32(seed: int, tensor: str, block: int, shape, std: float) -> np.ndarray:
    g = _rng(seed, tensor, block)
    a = g.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(std)
    return a


def normal_bf16(seed: int, tensor: str, block: int, shape, std: float) -> np.ndarray:
    return f32_to_bf16_bits(normal_f32(seed, tensor, block, shape, std))


def make_tokens(shape: LayerShape, T: int, point: int = 0, zero: bool = False) -> np.ndarray:
    """X[T, d] ~ N(0,1) as bf16 words.  `point` selects an independent batch
    (one per (B, gamma) sweep point); rows are i.i.d., so row b*(gamma+1)+i is
    simply request b, position i."""
    if zero:
        return np.zeros((T, shape.d), dtype=np.uint16)
    return normal_bf16(shape.seed, "x", point, (T, shape.d), 1.0)


def expert_block(shape: LayerShape, tensor: str, e: int) -> np.ndarray:
    """One routed expert's slice of w_gate / w_up ([I, d]) or w_down ([d, I])."""
    d, I = shape.d, shape.inter
    if tensor in ("w_gate", "w_up"):
        return normal_bf16(shape.seed, tensor, e, (I, d), 1.0 / np.sqrt(d))
    if tensor == "w_down":
        return normal_bf16(shape.seed, tensor, e, (d, I), 1.0 / np.sqrt(I))
    raise KeyError(tensor)


def make_router(shape: LayerShape, skew_std: float = 0.0) -> dict:
    """Router weights (std 0.02) and, for the skewed variant, a per-expert fp32
    logit bias ~ N(0, skew_std)."""
    out = {"w_router": normal_bf16(shape.seed, "w_router", 0, (shape.E, shape.d), 0.02),
           "router_bias": None}
    if skew_std > 0.0:
        out["router_bias"] = normal_f32(shape.seed, "router_bias", 0, (shape.E,), skew_std)
    return out


def make_shared(shape: LayerShape) -> dict:
    d, S = shape.d, shape.shared_inter
    out = {"ws_gate": None, "ws_up": None, "ws_down": None, "w_shared_gate": None}
    if S > 0:
        out["ws_gate"] = normal_bf16(shape.seed, "ws_gate", 0, (S, d), 1.0 / np.sqrt(d))
        out["ws_up"] = normal_bf16(shape.seed, "ws_up", 0, (S, d), 1.0 / np.sqrt(d))
        out["ws_down"] = normal_bf16(shape.seed, "ws_down", 0, (d, S), 1.0 / np.sqrt(S))
        if shape.shared_gate:
            out["w_shared_gate"] = normal_bf16(shape.seed, "w_shared_gate", 0, (d,), 0.02)
    return out


def make_layer(shape: LayerShape, skew_std: float = 0.0, threads: int = 8) -> dict:
    """All weights of one layer as numpy arrays of bf16 words (bias: fp32).
    Expert tensors are filled one expert per task so the host cores share the
    work; the result does not depend on `threads`.  With shape.weight_format ==
    WEIGHTS_FP8_E4M3 the expert matrices (routed and shared) are the same Gaussian
    draws quantised row by row: uint8 codes under the same keys plus fp32 scales
    under "<key>_scale"."""
    d, E, I = shape.d, shape.E, shape.inter
    fp8 = shape.weight_format == WEIGHTS_FP8_E4M3
    w = {}
    w.update(make_router(shape, skew_std))
    w.update(make_shared(shape))
    wdt = np.uint8 if fp8 else np.uint16
    w["w_gate"] = np.empty((E, I, d), dtype=wdt)
    w["w_up"] = np.empty((E, I, d), dtype=wdt)
    w["w_down"] = np.empty((E, d, I), dtype=wdt)
    if fp8:
        w["w_gate_scale"] = np.empty((E, I), dtype=np.float32)
        w["w_up_scale"] = np.empty((E, I), dtype=np.float32)
        w["w_down_scale"] = np.empty((E, d), dtype=np.float32)
        for k in ("ws_gate", "ws_up", "ws_down"):
            if w[k] is not None:
                w[k], w[k + "_scale"] = quantize_rows_e4m3(w[k])

    def fill(job):
        name, e = job
        if fp8:
            w[name][e], w[name + "_scale"][e] = quantize_rows_e4m3(expert_block(shape, name, e))
        else:
            w[name][e] = expert_block(shape, name, e)

    jobs = [(n, e) for e in range(E) for n in ("w_gate", "w_up", "w_down")]
    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    return w


def sweep_points(shape_name: str):
    """(B, gamma) grid of the benchmark sweep for a preset; T = B*(gamma+1)."""
    if shape_name == "tiny":
        return [(4, 3)]
    if shape_name == "mixtral-8x7b":
        return [(t, 0) for t in (1, 4, 16, 64, 256, 1024, 4096)]
    bmax = {"qwen1.5-moe-a2.7b": 128, "qwen2-57b-a14b": 256, "deepseek-v3": 512}[shape_name]
    bs = []
    b = 1
    while b <= bmax:
        bs.append(b)
        b *= 2
    return [(b, g) for b in bs for g in range(5)]
