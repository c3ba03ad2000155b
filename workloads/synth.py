"""Seeded generators for logits, activations, expert weights and the batch split.

Everything is drawn with NumPy's PCG64 from `SeedSequence([cfg.seed, stream, index])`
in fp32; bf16 tensors are the fp32 draws rounded to nearest-even and are returned as
raw uint16 bit patterns (NumPy has no bf16 type).  Nothing here routes, dispatches or
plans: those are the method, and live elsewhere.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .configs import LayerConfig

_STREAM_LOGITS = 11
_STREAM_X = 12
_STREAM_PERM = 13
_STREAM_ZIPF_S = 14
_STREAM_BIAS = 15
_STREAM_RATIO = 16
_STREAM_W1 = 21
_STREAM_W2 = 22

WEIGHT_STD = 0.02


def _rng(seed: int, stream: int, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream, index])))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to the fp32 values they denote."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def rank_token_offsets(T: int, N: int) -> np.ndarray:
    """Data-parallel batch split: rank i owns tokens [floor(i*T/N), floor((i+1)*T/N))."""
    return np.array([(i * T) // N for i in range(N + 1)], dtype=np.int32)


def zipf_exponent(cfg: LayerConfig, step: int) -> float:
    if cfg.s_range is None:
        return float(cfg.bias_param)
    lo, hi = cfg.s_range
    return float(_rng(cfg.seed, _STREAM_ZIPF_S, step).uniform(lo, hi))


def popularity_bias(cfg: LayerConfig, step: int = 0) -> np.ndarray:
    """Per-expert logit bias b[E] (fp32).

    "normal": b ~ N(0, bias_param) drawn once.  "zipf": a seeded ranking pi of the
    experts and b[e] = -s*ln(pi(e)+1), so softmax(b) is the Zipf(s) pmf over the
    ranking; the ranking is redrawn every `reshuffle_every` steps when that is set, and is
    drawn from `ranking_seed` instead of `seed` when that is set (a post-failure workload
    keeps the ranking of the configuration it re-plans).
    """
    if cfg.bias == "normal":
        return (_rng(cfg.seed, _STREAM_BIAS).standard_normal(cfg.E, dtype=np.float32)
                * np.float32(cfg.bias_param)).astype(np.float32)
    epoch = step // cfg.reshuffle_every if cfg.reshuffle_every else 0
    perm_seed = cfg.seed if cfg.ranking_seed is None else cfg.ranking_seed
    pi = _rng(perm_seed, _STREAM_PERM, epoch).permutation(cfg.E)
    s = zipf_exponent(cfg, step)
    return (-s * np.log(pi.astype(np.float64) + 1.0)).astype(np.float32)


def step_inputs(cfg: LayerConfig, step: int = 0, with_x: bool = True) -> dict:
    """Inputs of one layer pass: gating logits [T,E] fp32 and activations x [T,d].

    x is fp32 for an fp32 config, else bf16 bit patterns (uint16).
    """
    z = _rng(cfg.seed, _STREAM_LOGITS, step).standard_normal((cfg.T, cfg.E), dtype=np.float32)
    logits = (z + popularity_bias(cfg, step)[None, :]).astype(np.float32)
    out = {"logits": logits, "rank_tok_off": rank_token_offsets(cfg.T, cfg.N)}
    if with_x:
        x = _rng(cfg.seed, _STREAM_X, step).standard_normal((cfg.T, cfg.d), dtype=np.float32)
        out["x"] = x if cfg.dtype == "f32" else f32_to_bf16_bits(x)
    return out


def ratio_logits(T: int, E: int, ratio: float, seed: int) -> np.ndarray:
    """Gating logits [T,E] fp32 whose expert popularity rises linearly from 1 (expert 0) to
    `ratio` (expert E-1): logit = ln(popularity) + standard Gumbel noise, so that taking the
    largest logits draws experts in proportion to their popularity (the single-layer
    load-ratio workloads of the paper's ablation, most popular : least popular = ratio : 1)."""
    pop = 1.0 + (float(ratio) - 1.0) * np.arange(E) / max(1, E - 1)
    u = _rng(seed, _STREAM_RATIO, int(round(ratio * 1000))).random((T, E))
    gumbel = -np.log(-np.log(np.clip(u, 1e-12, 1.0 - 1e-12)))
    return (np.log(pop)[None, :] + gumbel).astype(np.float32)


def _one_weight(cfg: LayerConfig, stream: int, e: int, shape) -> np.ndarray:
    w = _rng(cfg.seed, stream, e).standard_normal(shape, dtype=np.float32)
    w *= np.float32(WEIGHT_STD)
    return w if cfg.dtype == "f32" else f32_to_bf16_bits(w)


def expert_weights(cfg: LayerConfig, threads: int = 8) -> dict:
    """Per-expert FFN weights, N(0, 0.02), no biases.

    w1[E, n1, d]: first projection, rows are output features (n1 = ffn for GELU; for
    SwiGLU n1 = 2*ffn with the gate projection in rows [0,ffn) and the up projection
    in rows [ffn,2ffn)).  w2[E, d, ffn]: second (down) projection, rows are output
    features.  All replicas of an expert carry these same values.
    """
    n1 = cfg.ffn * (2 if cfg.act == "swiglu" else 1)
    dt = np.float32 if cfg.dtype == "f32" else np.uint16
    w1 = np.empty((cfg.E, n1, cfg.d), dtype=dt)
    w2 = np.empty((cfg.E, cfg.d, cfg.ffn), dtype=dt)

    def fill(e):
        w1[e] = _one_weight(cfg, _STREAM_W1, e, (n1, cfg.d))
        w2[e] = _one_weight(cfg, _STREAM_W2, e, (cfg.d, cfg.ffn))

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(fill, range(cfg.E)))
    return {"w1": w1, "w2": w2}
