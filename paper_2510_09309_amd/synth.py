"""Seeded synthetic inputs for the MaskKV hot path (shared by tests, oracle checks and bench).

This module only draws random numbers and rounds them to the storage dtype; it holds
none of the method's arithmetic (no softmax, no scoring, no selection).  Both the CPU
oracle's tests and the GPU path consume the arrays produced here, so the two sides
always see the same rounded bits.

Recipe (stand-in for LLaDA-8B-shaped activations, no model weights or benchmark text):
for every head, Q, K and V components are N(0,1) * sigma / sqrt(d); a per-head unit
vector u_h is added to every mask query; ``n_planted`` random prompt positions get
``amplitude * u_h`` added to their key, so that mask queries attend to them more than
to the background.  Values are then rounded (round-to-nearest-even) to the storage
dtype and returned as float32 arrays holding exactly representable values.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "round_to_bf16",
    "bf16_bits",
    "LayerInputs",
    "make_layer",
    "make_response_step",
    "budgets_two_level",
    "budgets_log_uniform",
    "CONFIGS",
    "config_layer",
    "config_budgets",
    "c5_prompt_lengths",
]


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); return the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 and widen back: float32 values exactly representable in bf16."""
    bits = bf16_bits(x).astype(np.uint32) << np.uint32(16)
    return bits.view(np.float32).reshape(np.shape(x))


@dataclass
class LayerInputs:
    """One layer's (one sequence's) Q/K/V, all heads.  Arrays are float32 holding dtype-exact values."""
    H: int
    d: int
    P: int                 # prompt length
    n_m: int               # mask / response-span length
    dtype: str             # "f32" or "bf16"
    Q: np.ndarray          # [H, n_m, d]  queries of the response span (= mask queries at the first step)
    K: np.ndarray          # [H, P + n_m, d]  prompt rows then response rows
    V: np.ndarray          # [H, P + n_m, d]
    planted: np.ndarray    # [H, n_planted] prompt positions whose key carries the planted direction
    u: np.ndarray = field(repr=False, default=None)  # [H, d] per-head unit direction

    @property
    def N(self) -> int:
        return self.P + self.n_m


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    assert dtype == "f32"
    return np.ascontiguousarray(x, dtype=np.float32)


def make_layer(seed: int, H: int, d: int, P: int, n_m: int, dtype: str = "bf16",
               n_planted: int = 0, amplitude: float = 0.0, sigma: float = 1.0,
               query_shift: float = 1.0) -> LayerInputs:
    """Draw one layer of inputs.  See the module docstring for the recipe."""
    rng = np.random.default_rng(seed)
    N = P + n_m
    s = np.float32(sigma / np.sqrt(d))
    Q = rng.standard_normal((H, n_m, d), dtype=np.float32) * s
    K = rng.standard_normal((H, N, d), dtype=np.float32) * s
    V = rng.standard_normal((H, N, d), dtype=np.float32) * s
    u = rng.standard_normal((H, d), dtype=np.float32)
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    planted = np.zeros((H, n_planted), dtype=np.int64)
    for h in range(H):
        Q[h] += np.float32(query_shift) * u[h]
        if n_planted > 0:
            pos = np.sort(rng.choice(P, size=n_planted, replace=False))
            planted[h] = pos
            K[h, pos] += np.float32(amplitude) * u[h]
    return LayerInputs(H=H, d=d, P=P, n_m=n_m, dtype=dtype,
                       Q=_store(Q, dtype), K=_store(K, dtype), V=_store(V, dtype),
                       planted=planted, u=u)


def make_response_step(seed: int, H: int, d: int, n_m: int, dtype: str = "bf16", sigma: float = 1.0):
    """Fresh response-span Q, K, V for one denoising step: three [H, n_m, d] arrays."""
    rng = np.random.default_rng(seed)
    s = np.float32(sigma / np.sqrt(d))
    out = []
    for _ in range(3):
        out.append(_store(rng.standard_normal((H, n_m, d), dtype=np.float32) * s, dtype))
    return tuple(out)


def make_hidden_states(seed: int, n: int, hidden: int, dtype: str, drift: float):
    """Stand-ins for an attention sub-layer's input and output hidden states [n, hidden]: Gaussian rows, the
    output being the input plus `drift` times fresh Gaussian noise (so the rows' cosine similarity is about
    1/sqrt(1 + drift^2)); rounded to the storage dtype.  Returns float32 arrays holding the rounded values."""
    rng = np.random.default_rng(seed)
    h_in = rng.standard_normal((n, hidden)).astype(np.float32)
    h_out = h_in + np.float32(drift) * rng.standard_normal((n, hidden)).astype(np.float32)
    if dtype == "bf16":
        return round_to_bf16(h_in), round_to_bf16(h_out)
    return h_in, h_out


def make_value_steps(seed: int, n: int, width: int, dtype: str, drift_lo: float, drift_hi: float):
    """Stand-ins for one layer's value features of the n response tokens at two consecutive denoising steps,
    [n, width] each: the earlier step is Gaussian, the later one adds Gaussian noise whose size is drawn per
    token uniformly in [drift_lo, drift_hi], so the per-token cosine similarities spread over a range (about
    1/sqrt(1 + drift^2)).  Returns (V_now, V_prev) as float32 arrays holding the rounded values."""
    rng = np.random.default_rng(seed)
    v_prev = rng.standard_normal((n, width)).astype(np.float32)
    drift = rng.uniform(drift_lo, drift_hi, size=(n, 1)).astype(np.float32)
    v_now = v_prev + drift * rng.standard_normal((n, width)).astype(np.float32)
    if dtype == "bf16":
        return round_to_bf16(v_now), round_to_bf16(v_prev)
    return v_now, v_prev


def make_grouped_queries(seed: int, base: LayerInputs, q_per_kv: int, sigma: float = 1.0,
                         query_shift: float = 1.0) -> np.ndarray:
    """Queries for a grouped-query layer: [H * q_per_kv, n_m, d], query heads h*g .. h*g+g-1 reading KV head h of
    `base`.  Same recipe as make_layer's queries; the heads of a group share their KV head's planted direction."""
    rng = np.random.default_rng(seed)
    s = np.float32(sigma / np.sqrt(base.d))
    Q = rng.standard_normal((base.H * q_per_kv, base.n_m, base.d), dtype=np.float32) * s
    for hq in range(base.H * q_per_kv):
        Q[hq] += np.float32(query_shift) * base.u[hq // q_per_kv]
    return _store(Q, base.dtype)


def budgets_two_level(H: int, avg: int, seed: int, ratio: int = 2) -> np.ndarray:
    """Per-head integer budgets summing to H*avg: half the heads (seeded choice) get ``ratio`` x the others.

    Largest-remainder rounding keeps the total exact.
    """
    rng = np.random.default_rng(seed)
    heavy = np.zeros(H, dtype=bool)
    heavy[rng.choice(H, size=H // 2, replace=False)] = True
    w = np.where(heavy, float(ratio), 1.0)
    total = H * avg
    exact = w / w.sum() * total
    base = np.floor(exact).astype(np.int64)
    rem = total - int(base.sum())
    order = np.argsort(-(exact - base), kind="stable")
    base[order[:rem]] += 1
    return base.astype(np.int32)


def budgets_log_uniform(n: int, lo: int, hi: int, seed: int) -> np.ndarray:
    """n integer budgets, log-uniform in [lo, hi]."""
    rng = np.random.default_rng(seed)
    x = np.exp(rng.uniform(np.log(lo), np.log(hi), size=n))
    return np.clip(np.rint(x), lo, hi).astype(np.int32)


# The five benchmark configurations (shape, dtype, planting, pooling, budgets).
CONFIGS = {
    "C1": dict(layers=1, B=1, H=4, d=64, dtype="f32", P=512, n_m=64, n_planted=10, amplitude=3.0,
               window=7, budget_avg=32, budget_kind="uniform", seed=0),
    "C2": dict(layers=1, B=1, H=32, d=128, dtype="bf16", P=4096, n_m=256, n_planted=82, amplitude=2.5,
               window=7, budget_avg=256, budget_kind="two_level", seed=0),
    "C3": dict(layers=32, B=1, H=32, d=128, dtype="bf16", P=8192, n_m=256, n_planted=164, amplitude=2.5,
               window=7, budget_avg=128, budget_boundary=512, budget_kind="two_level", seed=1000),
    "C4": dict(layers=32, B=1, H=32, d=128, dtype="bf16", P=32768, n_m=256, n_planted=655, amplitude=2.5,
               window=7, budget_avg=256, budget_kind="two_level", seed=2000),
    "C5": dict(layers=1, B=8, H=32, d=128, dtype="bf16", P_lo=4096, P_hi=16384, n_m=512, planted_frac=0.02,
               amplitude=2.5, window=7, budget_lo=64, budget_hi=1024, budget_kind="log_uniform", steps=64,
               seed=3000),
}


def c5_prompt_lengths(cfg: dict | None = None) -> np.ndarray:
    cfg = cfg or CONFIGS["C5"]
    rng = np.random.default_rng(cfg["seed"])
    return rng.integers(cfg["P_lo"], cfg["P_hi"] + 1, size=cfg["B"]).astype(np.int32)


def config_layer(name: str, layer: int = 0, b: int = 0, sigma: float = 1.0) -> LayerInputs:
    """Inputs of one layer (and, for the batched config, one sequence) of a named configuration."""
    cfg = CONFIGS[name]
    if name == "C5":
        P = int(c5_prompt_lengths(cfg)[b])
        n_planted = int(round(cfg["planted_frac"] * P))
        seed = cfg["seed"] + 100 + b
    else:
        P = cfg["P"]
        n_planted = cfg["n_planted"]
        seed = cfg["seed"] + layer
    return make_layer(seed, cfg["H"], cfg["d"], P, cfg["n_m"], cfg["dtype"],
                      n_planted=n_planted, amplitude=cfg["amplitude"], sigma=sigma)


def config_budgets(name: str, layer: int = 0) -> np.ndarray:
    """Per-(b, h) budgets of a named configuration, int32 [B*H]."""
    cfg = CONFIGS[name]
    H, B = cfg["H"], cfg["B"]
    kind = cfg["budget_kind"]
    if kind == "uniform":
        return np.full(B * H, cfg["budget_avg"], dtype=np.int32)
    if kind == "two_level":
        avg = cfg["budget_avg"]
        if "budget_boundary" in cfg and layer in (0, cfg["layers"] - 1):
            avg = cfg["budget_boundary"]
        return budgets_two_level(H, avg, seed=cfg["seed"] + 7)
    if kind == "log_uniform":
        return budgets_log_uniform(B * H, cfg["budget_lo"], cfg["budget_hi"], seed=cfg["seed"] + 7)
    raise ValueError(kind)
