"""Seeded synthetic inputs for the smoothed W8A8 expert-FFN path.

This module only draws random tensors of the shapes and value structure the
workloads need (hidden states with a few fixed outlier channels, Gaussian
full-precision weights, a router gate and router logits).  It contains none of
the quantization method's arithmetic: smoothing vectors, int8 codes and scales
are derived from these tensors separately by the CPU oracle and by the HIP
library, each with its own code.

Everything is a pure function of its seed (numpy Philox counter-based streams),
so the CPU oracle and the GPU path are always fed the same bytes.

The tensors stand in for OPT / Mixtral activations and weights, which are not
available offline: hidden states are N(0,1) with a small set of channels whose
magnitude is tens of times larger and stable across tokens (the outlier
structure the paper's Section I and Section III.B.1 describe), weights are
N(0, 0.02^2).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

# Mixtral-8x7B expert geometry used by the MoE workloads.
MIXTRAL_H = 4096
MIXTRAL_I = 14336
MIXTRAL_E = 8

ZIPF_S = 1.1
OFFLOAD_POPULARITY = (0.3, 0.2, 0.15, 0.1, 0.1, 0.07, 0.05, 0.03)


def _rng(seed: int, stream: int) -> np.random.Generator:
    """Independent counter-based stream `stream` of seed `seed`."""
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


# Stream ids (one per tensor kind so that shapes can change independently).
_S_X, _S_OUTLIER_IDX, _S_OUTLIER_MUL, _S_GATE, _S_GUMBEL = 1, 2, 3, 4, 5
_S_W_BASE = 100


def outlier_channels(seed: int, K: int, n_outlier: int) -> np.ndarray:
    """Indices of the fixed outlier channels: first entries of a seeded permutation."""
    return np.sort(_rng(seed, _S_OUTLIER_IDX).permutation(K)[:n_outlier]).astype(np.int64)


def hidden_states(seed: int, T: int, K: int, n_outlier: int | None = None,
                  mult: float | tuple[float, float] = (20.0, 80.0),
                  channel_seed: int | None = None) -> tuple[np.ndarray, np.ndarray, np.ndarray]:
    """fp16 activations [T, K] ~ N(0,1) with fixed outlier channels scaled up.

    n_outlier defaults to ceil(0.5% of K).  `mult` is either one multiplier for
    every outlier channel or a (lo, hi) range from which one multiplier per
    outlier channel is drawn uniformly.  The multiplier is applied in fp32
    before the single rounding to fp16.  Returns (X, channel_idx, channel_mult).
    The outlier channels and their multipliers belong to the layer, not to the
    batch: `channel_seed` (default: `seed`) selects them, `seed` the token values.
    """
    if n_outlier is None:
        n_outlier = int(math.ceil(0.005 * K))
    cs = seed if channel_seed is None else channel_seed
    idx = outlier_channels(cs, K, n_outlier)
    if isinstance(mult, tuple):
        m = _rng(cs, _S_OUTLIER_MUL).uniform(mult[0], mult[1], size=n_outlier).astype(np.float32)
    else:
        m = np.full(n_outlier, mult, dtype=np.float32)
    x = _rng(seed, _S_X).standard_normal(size=(T, K), dtype=np.float32)
    x[:, idx] *= m[None, :]
    return x.astype(np.float16), idx, m


def gaussian_weight(seed: int, which: int, K: int, N: int, std: float = 0.02) -> np.ndarray:
    """fp32 weight [K, N] (input channel major) ~ N(0, std^2); `which` selects the matrix."""
    w = _rng(seed, _S_W_BASE + which).standard_normal(size=(K, N), dtype=np.float32)
    w *= np.float32(std)
    return w


def router_gate(seed: int, H: int, E: int, std: float = 0.02) -> np.ndarray:
    """fp16 router gate [H, E] ~ N(0, std^2)."""
    g = _rng(seed, _S_GATE).standard_normal(size=(H, E), dtype=np.float32) * np.float32(std)
    return g.astype(np.float16)


def gate_logits(X: np.ndarray, gate: np.ndarray, bias: np.ndarray | None = None) -> np.ndarray:
    """Router logits fp16 [T, E] = X @ gate (+ bias), accumulated in fp64, rounded once."""
    l = X.astype(np.float64) @ gate.astype(np.float64)
    if bias is not None:
        l = l + bias[None, :].astype(np.float64)
    return l.astype(np.float16)


def _top2_shares(logits_f16: np.ndarray) -> np.ndarray:
    """Share of the 2T (token, slot) assignments that lands on each expert."""
    l = logits_f16.astype(np.float32)
    E = l.shape[1]
    order = np.argsort(-l, axis=1, kind="stable")[:, :2]
    cnt = np.bincount(order.ravel(), minlength=E).astype(np.float64)
    return cnt / cnt.sum()


def zipf_shares(E: int, s: float = ZIPF_S) -> np.ndarray:
    p = 1.0 / np.arange(1, E + 1, dtype=np.float64) ** s
    return p / p.sum()


def fit_router_bias(X: np.ndarray, gate: np.ndarray, target: np.ndarray, iters: int = 50) -> np.ndarray:
    """Router bias (fp64 [E]) that makes expert popularity follow `target`.

    Fixed-length deterministic iteration b += log(target / observed); observed
    shares are clipped away from zero so the update stays finite.
    """
    E = gate.shape[1]
    b = np.zeros(E, dtype=np.float64)
    base = X.astype(np.float64) @ gate.astype(np.float64)
    for _ in range(iters):
        obs = _top2_shares((base + b[None, :]).astype(np.float16))
        b += 0.5 * np.log(target / np.clip(obs, 1e-4, None))
        b -= b.mean()
    return b


def gumbel_logits(seed: int, T: int, popularity=OFFLOAD_POPULARITY) -> np.ndarray:
    """fp16 logits [T, E] = log(popularity) + Gumbel noise: top-2 samples two
    distinct experts in proportion to popularity."""
    p = np.asarray(popularity, dtype=np.float64)
    u = _rng(seed, _S_GUMBEL).uniform(1e-12, 1.0, size=(T, p.size))
    return (np.log(p)[None, :] - np.log(-np.log(u))).astype(np.float16)


# --------------------------------------------------------------------------
# Workload descriptions (shapes only; tensors are drawn lazily by the callers)
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class LinearWorkload:
    name: str
    seed: int
    T: int
    K: int
    N: int
    n_outlier: int
    mult: float | tuple[float, float]
    act: str  # "relu" | "none"


@dataclass(frozen=True)
class FfnWorkload:
    name: str
    seed: int
    T: int
    H: int
    F: int
    n_outlier: int
    mult: tuple[float, float] = (20.0, 80.0)


@dataclass(frozen=True)
class MoeWorkload:
    name: str
    seed: int
    T: int
    H: int = MIXTRAL_H
    I: int = MIXTRAL_I
    E: int = MIXTRAL_E
    routing: str = "gate"  # "gate" | "zipf" | "popularity"
    resident: tuple[int, ...] = field(default_factory=tuple)  # empty = all resident
    layer_seed: int | None = None  # seed of the layer (weights, gate, outlier channels); default: seed


OPT125M_LINEAR = LinearWorkload("opt125m_linear", 0, 16, 768, 3072, 4, 50.0, "relu")
OPT67B_FFN = FfnWorkload("opt6.7b_ffn", 1, 2048, 4096, 16384, 20)
# One Mixtral-shaped layer (weights, router gate, outlier channels: seed 2) serves the
# decode, prefill and offload workloads; each workload draws its own tokens.
MIXTRAL_LAYER_SEED = 2
MIXTRAL_DECODE = tuple(MoeWorkload(f"mixtral_decode_b{b}", 2, b, layer_seed=MIXTRAL_LAYER_SEED) for b in (1, 8, 64))
MIXTRAL_PREFILL = MoeWorkload("mixtral_prefill_zipf", 3, 4096, routing="zipf", layer_seed=MIXTRAL_LAYER_SEED)
MIXTRAL_OFFLOAD = MoeWorkload("mixtral_offload_b256", 4, 256, routing="popularity", resident=(0, 1, 2, 3),
                              layer_seed=MIXTRAL_LAYER_SEED)
MIXTRAL_CALIB = MoeWorkload("mixtral_calibration", 2, 256, layer_seed=MIXTRAL_LAYER_SEED)


def _layer_seed(wl: MoeWorkload) -> int:
    return wl.seed if wl.layer_seed is None else wl.layer_seed


def moe_hidden_states(wl: MoeWorkload) -> np.ndarray:
    """The workload's token batch: its own values, the layer's outlier channels."""
    return hidden_states(wl.seed, wl.T, wl.H, channel_seed=_layer_seed(wl))[0]


def moe_logits(wl: MoeWorkload, X: np.ndarray) -> np.ndarray:
    """Router logits for a MoE workload, following its routing recipe."""
    if wl.routing == "popularity":
        assert wl.E == len(OFFLOAD_POPULARITY)
        return gumbel_logits(wl.seed, wl.T)
    gate = router_gate(_layer_seed(wl), wl.H, wl.E)
    if wl.routing == "zipf":
        bias = fit_router_bias(X, gate, zipf_shares(wl.E))
        return gate_logits(X, gate, bias)
    return gate_logits(X, gate)


def moe_weight(wl: MoeWorkload, e: int, which: str) -> np.ndarray:
    """fp32 weight of expert e; which in {"w1","w3"} -> [H, I], "w2" -> [I, H]."""
    j = {"w1": 0, "w3": 1, "w2": 2}[which]
    if which == "w2":
        return gaussian_weight(_layer_seed(wl), 3 * e + j, wl.I, wl.H)
    return gaussian_weight(_layer_seed(wl), 3 * e + j, wl.H, wl.I)
