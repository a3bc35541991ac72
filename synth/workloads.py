"""Seeded synthetic gate workloads (inputs only; none of the router's arithmetic).

Both the CPU oracle's tests and the GPU path's tests/bench draw their inputs from
here, so that the two sides consume identical bits.  Nothing in this module
computes a logit, a score, a routing decision or a dispatch index.

The shapes follow the two models the paper evaluates (Evaluation section,
"Models and Datasets": Mixtral-8x7B with k=2 of 8 experts, DeepSeek-MoE-16b with
k=6 of 64 routed experts).  Their weights and the evaluation datasets are not
available, so hidden states and gate weights are random with a controllable
logit bias; the threshold presets are the paper's (appendix table "Thresholds
used per model and dataset").

Recipe.  W ~ N(0, 0.02^2) [E,H];  hidden_t = sigma_t * g_t + pinv(W) b_t with
g_t ~ N(0, I_H), so that the gate logits are approximately sigma_t * (W g_t) + b_t:
a chosen per-token logit bias b_t on top of natural noise of standard deviation
sigma_t * 0.02 * sqrt(H).  bf16 tensors are produced by round-to-nearest-even of
the fp32 values and handed out as uint16 bit patterns.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

BASE_SEED = 20251003

DTYPE_F32 = 0
DTYPE_BF16 = 1


@dataclasses.dataclass(frozen=True)
class GateShape:
    name: str
    index: int          # position in the list of benchmark configurations
    T: int
    H: int
    E: int
    k: int
    c: int
    dtype: int          # DTYPE_F32 / DTYPE_BF16
    layers: int         # number of MoE layers (or decode steps for the decode shape)
    persist_loads: bool # True: load counters carry over between consecutive calls


SHAPES = {
    "tiny":     GateShape("tiny",     0, 256,    128,  8,  2, 4, DTYPE_F32,  1,   False),
    "mixtral":  GateShape("mixtral",  1, 16384,  4096, 8,  2, 4, DTYPE_BF16, 32,  False),
    "deepseek": GateShape("deepseek", 2, 16384,  2048, 64, 6, 8, DTYPE_BF16, 27,  False),
    "decode":   GateShape("decode",   3, 64,     2048, 64, 6, 8, DTYPE_BF16, 512, True),
    "prefill":  GateShape("prefill",  4, 131072, 4096, 64, 6, 8, DTYPE_BF16, 1,   False),
}


def thresholds(shape_name: str, layer: int, preset: str = "paper") -> tuple[float, float]:
    """(eps_high, t_fix) for one layer.

    preset "paper": appendix threshold table -- Mixtral rows ARC (t_fix 0.60,
    eps_high 0.7159/0.6419/0.6285 for early/middle/final layers), DeepSeek rows
    ARC-Challenge/MMLU (0.80 / 0.40).  The paper does not say where the bands
    start; thirds of the layer stack are used (first third early, last third
    final, the rest middle).
    preset "gsm8k": DeepSeek GSM8K row (t_fix 0.25/0.45/0.55, eps_high 0.30).
    preset "stress": eps_high = 2 and t_fix = 1e-30, so that every token takes the
    load-aware branch with a full working set of c experts (the longest possible
    chain of load-dependent decisions).
    preset "topk": eps_high tiny, every token keeps its top-k.
    """
    s = SHAPES[shape_name]
    n = s.layers if not s.persist_loads else 1
    third = n // 3
    band = 0 if layer < third else (2 if layer >= n - third else 1)
    if n < 3:
        band = 1
    mixtral_like = s.E == 8
    if preset == "paper":
        if mixtral_like:
            return (0.7159, 0.6419, 0.6285)[band], 0.60
        return 0.40, 0.80
    if preset == "gsm8k":
        if mixtral_like:
            return (0.72, 0.75, 0.80)[band], 0.60
        return 0.30, (0.25, 0.45, 0.55)[band]
    if preset == "stress":
        return 2.0, 1e-30
    if preset == "topk":
        return 1e-6, (0.60 if mixtral_like else 0.80)
    raise ValueError(preset)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def _store(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == DTYPE_BF16:
        return f32_to_bf16_bits(x)
    return np.ascontiguousarray(x, dtype=np.float32)


def _as_f64(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == DTYPE_BF16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


def make_gate(rng: np.random.Generator, T: int, H: int, E: int, dtype: int,
              bias: np.ndarray | None = None, sigma: np.ndarray | float = 1.0,
              w: np.ndarray | None = None):
    """One (hidden, w_gate) pair with an optional target logit bias.

    bias: None, [E] (same for every token) or [T,E]; sigma: scalar or [T].
    w: reuse a given stored gate matrix instead of drawing a new one.
    Returns (hidden, w_gate) in the storage dtype (uint16 bits for bf16).
    """
    if w is None:
        w = _store(rng.standard_normal((E, H), dtype=np.float32) * np.float32(0.02), dtype)
    g = rng.standard_normal((T, H), dtype=np.float32)
    if np.ndim(sigma) > 0:
        g *= np.asarray(sigma, dtype=np.float32)[:, None]
    elif float(sigma) != 1.0:
        g *= np.float32(sigma)
    if bias is not None:
        w64 = _as_f64(w, dtype)
        pinv_t = np.linalg.solve(w64 @ w64.T, w64)          # [E,H] = (W W^T)^-1 W
        b = np.asarray(bias, dtype=np.float64)
        if b.ndim == 1:
            g += (b @ pinv_t).astype(np.float32)[None, :]
        else:
            g += (b @ pinv_t).astype(np.float32)
    return _store(g, dtype), w


def layer_inputs(shape_name: str, layer: int = 0, T: int | None = None,
                 w: np.ndarray | None = None):
    """Inputs of one routing call of a benchmark configuration.

    Returns a dict with hidden, w_gate (storage dtype), loads_in (int32 zeros), and
    the GateShape.  `T` overrides the token count (same distribution, fewer or
    more tokens).  Seed = BASE_SEED + 1000 * configuration index + layer.
    """
    s = SHAPES[shape_name]
    T = s.T if T is None else T
    rng = np.random.default_rng(BASE_SEED + 1000 * s.index + layer)
    E, H = s.E, s.H
    bias = None
    sigma: np.ndarray | float = 1.0
    if shape_name == "tiny":
        pass
    elif shape_name == "mixtral":
        # half of the tokens: +3.0 on one random expert (peaked); the rest unbiased
        bias = np.zeros((T, E), dtype=np.float32)
        peaked = rng.permutation(T)[: T // 2]
        bias[peaked, rng.integers(0, E, size=peaked.size)] = 3.0
    elif shape_name in ("deepseek", "decode"):
        # Zipf(s=1.1) expert popularity: bias -1.1 ln(rank) under a random expert->rank map
        rank_of = rng.permutation(E) + 1
        bias = (-1.1 * np.log(rank_of)).astype(np.float32)
        if shape_name == "decode":
            # the expert->rank map belongs to the model: fixed over decode steps
            rank_of = np.random.default_rng(BASE_SEED + 1000 * s.index).permutation(E) + 1
            bias = (-1.1 * np.log(rank_of)).astype(np.float32)
            theta = rng.choice(np.array([0.3, 1.0, 3.0], dtype=np.float32), size=T)
            sigma = (1.0 / theta).astype(np.float32)
            bias = bias[None, :] * sigma[:, None]
    elif shape_name == "prefill":
        rank_of = rng.permutation(E) + 1
        zipf = (-1.3 * np.log(rank_of)).astype(np.float32)
        flat = rng.random(T) < 0.10
        bias = np.where(flat[:, None], np.float32(0.0), zipf[None, :]).astype(np.float32)
        natural = 0.02 * math.sqrt(H)
        sigma = np.where(flat, np.float32(0.05 / natural), np.float32(1.0)).astype(np.float32)
    else:
        raise ValueError(shape_name)
    hidden, w_gate = make_gate(rng, T, H, E, s.dtype, bias=bias, sigma=sigma, w=w)
    return {
        "shape": s, "T": T, "hidden": hidden, "w_gate": w_gate,
        "loads_in": np.zeros(E, dtype=np.int32),
    }


def decode_gate_weight() -> np.ndarray:
    """The single gate matrix shared by all steps of the decode configuration."""
    s = SHAPES["decode"]
    rng = np.random.default_rng(BASE_SEED + 1000 * s.index + 999_983)
    return _store(rng.standard_normal((s.E, s.H), dtype=np.float32) * np.float32(0.02), s.dtype)


def random_logits(seed: int, T: int, E: int, kind: str = "normal", scale: float = 1.0,
                  tie_levels: int = 0) -> np.ndarray:
    """fp32 logits for tests that start after the gate projection.

    kind "normal": N(0, scale^2); "ties": values drawn from `tie_levels` distinct
    levels so that equal logits (and equal scores) are frequent.
    """
    rng = np.random.default_rng(seed)
    if kind == "normal":
        return (rng.standard_normal((T, E)) * scale).astype(np.float32)
    if kind == "ties":
        levels = (rng.standard_normal(max(tie_levels, 1)) * scale).astype(np.float32)
        return levels[rng.integers(0, levels.size, size=(T, E))]
    raise ValueError(kind)
