"""Seeded synthetic MoE layers: shapes, seeds and value distributions only.

This module is the one piece shared by the CPU oracle and the HIP path. It draws
random tensors and converts number formats; it performs none of the MoE layer's
arithmetic (no gate product, no softmax, no top-k, no FFN).  Everything it
returns is a NumPy array on the host:

* fp32 layers: ``float32`` arrays.
* bf16 layers: ``uint16`` arrays holding bfloat16 bit patterns (fp32 normals
  rounded to nearest-even); both consumers read these same bytes.

The five named workloads follow the model shapes the paper serves (a
Mixtral-8x7B-like layer: 8 experts, 2 active, 16-bit experts of three d x F
matrices, Section 2.2 and Table 1) plus the fine-grained, skewed and
decode-shaped layers this build is measured on.  They stand in for the paper's
datasets and trained weights, which are not available offline.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
import math
import os

import numpy as np

F32 = 0
BF16 = 1


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int           # tokens
    d: int           # hidden size
    E: int           # experts
    k: int           # experts activated per token
    F: int           # SwiGLU FFN width
    dtype: int       # F32 or BF16 (storage type of x and all weights)
    renorm: int      # 1: top-k routing weights renormalised to sum to one
    seed: int
    x_std: float     # std of x; <0 means 1.0
    w_std: float     # std of all weights; <0 means 1/sqrt(d)
    zipf_alpha: float = 0.0   # >0: per-expert gate bias s*ln(Zipf rank probability)
    zipf_scale: float = 0.0   # the "s" above
    empty_tail: int = 0       # >0: the last `empty_tail` experts get bias -1e9 (never chosen)

    @property
    def A(self) -> int:
        return self.T * self.k

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == F32 else 2


# zipf_scale for "skew" was found by oracle/calibrate_skew.py (bisection with the
# oracle router so that the hottest expert is chosen by 95% of the tokens, i.e.
# holds 15.8% of the T*k assignments; a 20% share cannot be reached with k = 6
# because an expert receives at most one assignment per token, 1/k = 16.7%).
ZIPF_SCALE_SKEW = 0.9150390625

CONFIGS = {
    "tiny": LayerConfig("tiny", T=64, d=128, E=8, k=2, F=256, dtype=F32, renorm=1,
                        seed=1001, x_std=0.02, w_std=0.02),
    "mixtral": LayerConfig("mixtral", T=4096, d=4096, E=8, k=2, F=14336, dtype=BF16, renorm=1,
                           seed=2002, x_std=1.0, w_std=-1.0),
    "finegrained": LayerConfig("finegrained", T=8192, d=2048, E=64, k=6, F=1408, dtype=BF16,
                               renorm=0, seed=3003, x_std=1.0, w_std=-1.0),
    "skew": LayerConfig("skew", T=8192, d=2048, E=64, k=6, F=1408, dtype=BF16, renorm=0,
                        seed=4004, x_std=1.0, w_std=-1.0, zipf_alpha=1.2,
                        zipf_scale=ZIPF_SCALE_SKEW),
    "decode": LayerConfig("decode", T=32, d=4096, E=128, k=8, F=1536, dtype=BF16, renorm=1,
                          seed=5005, x_std=1.0, w_std=-1.0),
}
# The paper's other two evaluation models (its Table 1 gives experts per layer, active experts and
# parameter totals: Phi-3.5-MoE 2 of 16, 42 B; Llama-4-Scout 1 of 16, 109 B).  Hidden and FFN widths
# are not in the paper; they are the public model configurations, and with them 3*d*F*E per layer
# times the layer count reproduces the parameter totals the paper prints.  Synthetic weights.
CONFIGS["phi"] = LayerConfig("phi", T=4096, d=4096, E=16, k=2, F=6400, dtype=BF16, renorm=1,
                             seed=6006, x_std=1.0, w_std=-1.0)
CONFIGS["llama4"] = LayerConfig("llama4", T=4096, d=5120, E=16, k=1, F=8192, dtype=BF16, renorm=0,
                                seed=7007, x_std=1.0, w_std=-1.0)
# The skewed layer with its last four experts forced empty.
CONFIGS["skew_empty"] = replace(CONFIGS["skew"], name="skew_empty", empty_tail=4)


def small_config(name="small", **kw) -> LayerConfig:
    """A free-form config for tests (defaults: a bf16 layer spanning a few tiles)."""
    base = dict(T=300, d=256, E=8, k=2, F=384, dtype=BF16, renorm=1, seed=7, x_std=1.0,
                w_std=-1.0)
    base.update(kw)
    return LayerConfig(name, **base)


# ----------------------------------------------------------------------------- formats
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns.

    Inputs are finite normals here, so NaN handling is not needed.
    """
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(
        np.float32)


def _store(a32: np.ndarray, dtype: int) -> np.ndarray:
    return a32 if dtype == F32 else f32_to_bf16_bits(a32)


def _normal(seed_path, shape, std, dtype):
    rng = np.random.default_rng(list(seed_path))
    a = rng.standard_normal(shape, dtype=np.float32)
    a *= np.float32(std)
    return _store(a, dtype)


# ----------------------------------------------------------------------------- layers
def gate_bias(cfg: LayerConfig):
    """Per-expert additive gate bias (float32 [E]) or None for an unbiased router."""
    if cfg.zipf_alpha <= 0.0 and cfg.empty_tail <= 0:
        return None
    b = np.zeros(cfg.E, dtype=np.float64)
    if cfg.zipf_alpha > 0.0:
        ranks = np.arange(1, cfg.E + 1, dtype=np.float64)
        p = ranks ** (-cfg.zipf_alpha)
        p /= p.sum()
        b = cfg.zipf_scale * np.log(p)
    if cfg.empty_tail > 0:
        b[cfg.E - cfg.empty_tail:] = -1.0e9
    return b.astype(np.float32)


def make_layer(cfg: LayerConfig, parts=("x", "w_gate", "w1", "w3", "w2"), workers=None):
    """Draw the tensors of one layer.

    Each tensor (and each expert of a weight tensor) has its own child seed
    ``[seed, tensor_id, expert]`` so any subset can be drawn alone, in any order,
    and experts can be drawn in parallel.

    Layouts (all row-major): x [T,d]; w_gate [E,d]; w1, w3 [E,F,d]; w2 [E,d,F].
    """
    w_std = cfg.w_std if cfg.w_std > 0 else 1.0 / math.sqrt(cfg.d)
    x_std = cfg.x_std if cfg.x_std > 0 else 1.0
    out = {"cfg": cfg, "gate_bias": gate_bias(cfg)}
    if "x" in parts:
        out["x"] = _normal((cfg.seed, 0), (cfg.T, cfg.d), x_std, cfg.dtype)
    if "w_gate" in parts:
        out["w_gate"] = _normal((cfg.seed, 1), (cfg.E, cfg.d), w_std, cfg.dtype)
    big = [(n, tid, shp) for n, tid, shp in (("w1", 2, (cfg.F, cfg.d)), ("w3", 3, (cfg.F, cfg.d)),
                                             ("w2", 4, (cfg.d, cfg.F))) if n in parts]
    if big:
        np_dt = np.float32 if cfg.dtype == F32 else np.uint16
        for n, _, shp in big:
            out[n] = np.empty((cfg.E,) + shp, dtype=np_dt)

        def fill(job):
            n, tid, shp, e = job
            out[n][e] = _normal((cfg.seed, tid, e), shp, w_std, cfg.dtype)

        jobs = [(n, tid, shp, e) for n, tid, shp in big for e in range(cfg.E)]
        if workers is None:
            workers = min(8, os.cpu_count() or 1)
        if workers > 1 and cfg.E * cfg.F * cfg.d > (1 << 22):
            with ThreadPoolExecutor(max_workers=workers) as pool:
                list(pool.map(fill, jobs))
        else:
            for j in jobs:
                fill(j)
    return out


def residual_step(cfg: LayerConfig, x: np.ndarray, eps: float, step: int = 1) -> np.ndarray:
    """The hidden states one layer later under a residual-stream model: x + eps * x_std * n with
    n ~ N(0, 1) drawn from the child seed [seed, 5, step], stored in the layer's dtype.  Stands in
    for the slowly varying hidden states that make a later layer's gate usable as a predictor
    (paper, Section 4.1); eps is the relative size of one layer's update."""
    x_std = cfg.x_std if cfg.x_std > 0 else 1.0
    x32 = x if cfg.dtype == F32 else bf16_bits_to_f32(x)
    rng = np.random.default_rng([cfg.seed, 5, int(step)])
    n = rng.standard_normal(x32.shape, dtype=np.float32)
    return _store(x32 + np.float32(eps * x_std) * n, cfg.dtype)


def expert_weights(cfg: LayerConfig, e: int):
    """(w1_e [F,d], w3_e [F,d], w2_e [d,F]) of one expert, drawn alone."""
    w_std = cfg.w_std if cfg.w_std > 0 else 1.0 / math.sqrt(cfg.d)
    return (_normal((cfg.seed, 2, e), (cfg.F, cfg.d), w_std, cfg.dtype),
            _normal((cfg.seed, 3, e), (cfg.F, cfg.d), w_std, cfg.dtype),
            _normal((cfg.seed, 4, e), (cfg.d, cfg.F), w_std, cfg.dtype))


def zipf_loads(E: int, total: int, alpha: float, seed: int) -> np.ndarray:
    """Synthetic per-expert token counts of one layer (int64 [E], summing to `total`): a multinomial
    draw with expert probabilities proportional to rank^-alpha, ranks shuffled over the expert
    indices.  Stands in for the skewed expert loads of the paper's traces (its Section 3.1
    characterisation: a few stragglers carry most tokens)."""
    rng = np.random.default_rng([int(seed), 77, int(E)])
    p = np.arange(1, E + 1, dtype=np.float64) ** (-float(alpha))
    p /= p.sum()
    rng.shuffle(p)
    return rng.multinomial(int(total), p).astype(np.int64)
