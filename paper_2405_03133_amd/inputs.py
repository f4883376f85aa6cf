"""Seeded synthetic inputs for the Lory merged-MoE-FFN layer.

This module only draws random numbers and rounds them; it holds none of the
method's arithmetic (no means, softmax, merges or matmuls).  Both the HIP
path's tests and the CPU oracle's tests take their tensors from here so that
the two sides see bit-identical operands.

Shapes follow the paper's problem statement (Algorithm 1: x is B x L x d, the
router maps a hidden vector to E weights; Section 4.1: L = 4096, T = 256,
E in {8, 16, 32}).  Value distributions: hidden states N(0, 1), expert and
router weights N(0, sigma = 0.02), upstream gradient dY N(0, 1).

The "structured" variant imitates what the paper reports about its real
workload (Section 5.4: routing is peaked and stable within a domain;
Section 3.2: adjacent segments are similar by construction): every sequence
gets a domain offset vector added to all of its hidden states and the router
is drawn with sigma = 1/sqrt(d), which yields clearly non-uniform,
segment-correlated routing weights.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

import numpy as np


@dataclass(frozen=True)
class LoryConfig:
    name: str
    B: int
    L: int
    T: int
    d: int
    d_ff: int
    E: int
    dtype: str  # "f32" or "bf16"
    seed: int

    @property
    def N(self) -> int:
        return self.L // self.T

    @property
    def S(self) -> int:
        return self.B * self.N

    @property
    def tokens(self) -> int:
        return self.B * self.L

    def gemm_flops(self, backward: bool = True) -> float:
        """Dense SwiGLU FFN cost, 6*tokens*d*d_ff forward (Appendix B) and
        twice that again for the backward."""
        f = 6.0 * self.tokens * self.d * self.d_ff
        return 3.0 * f if backward else f

    def merge_flops(self, passes: int = 4) -> float:
        """Merge-class cost: 6*E*d*d_ff per segment and pass (Appendix B);
        forward merge, backward re-merge, gradient scatter and router-weight
        inner products are one pass each."""
        return passes * 6.0 * self.E * self.d * self.d_ff * self.S

    def with_(self, **kw) -> "LoryConfig":
        return replace(self, **kw)


_BASE_SEED = 0x10F7

CONFIGS: Dict[str, LoryConfig] = {
    "C1": LoryConfig("C1", B=2, L=512, T=128, d=64, d_ff=256, E=4, dtype="f32", seed=_BASE_SEED + 1),
    "C2": LoryConfig("C2", B=8, L=4096, T=256, d=1024, d_ff=2816, E=8, dtype="bf16", seed=_BASE_SEED + 2),
    "C3": LoryConfig("C3", B=8, L=4096, T=256, d=1024, d_ff=2816, E=32, dtype="bf16", seed=_BASE_SEED + 3),
    "C4": LoryConfig("C4", B=4, L=4096, T=256, d=2048, d_ff=5632, E=32, dtype="bf16", seed=_BASE_SEED + 4),
}
# One GPU's share of C4 under expert-wise model parallelism over 8 GPUs (paper Section 6): every
# expert cut along d_ff, the same slice of all experts on one device.
CONFIGS["C4_EP8"] = LoryConfig("C4_EP8", B=4, L=4096, T=256, d=2048, d_ff=704, E=32, dtype="bf16",
                               seed=_BASE_SEED + 6)
# The paper's own model shapes (Section 4.1 and its model table): 1.5B with 8/16/32 experts, 7B with 4.
for _E in (8, 16, 32):
    CONFIGS[f"P15_E{_E}"] = LoryConfig(f"P15_E{_E}", B=4, L=4096, T=256, d=1536, d_ff=4096, E=_E,
                                       dtype="bf16", seed=_BASE_SEED + 7)
CONFIGS["P7_E4"] = LoryConfig("P7_E4", B=4, L=4096, T=256, d=4096, d_ff=11008, E=4, dtype="bf16",
                              seed=_BASE_SEED + 8)
for _T in (64, 128, 256, 512, 1024):
    CONFIGS[f"C5_T{_T}"] = LoryConfig(f"C5_T{_T}", B=4, L=4096, T=_T, d=2048, d_ff=5632, E=16,
                                      dtype="bf16", seed=_BASE_SEED + 5)


# The headline shape with short segments (Appendix B's E/T overhead at its largest: E = 32, T = 64 and 128).
for _T in (64, 128):
    CONFIGS[f"C4_T{_T}"] = LoryConfig(f"C4_T{_T}", B=4, L=4096, T=_T, d=2048, d_ff=5632, E=32,
                                      dtype="bf16", seed=_BASE_SEED + 9)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even) and return
    them widened back to float32 (the widening is exact)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of already bf16-representable float32 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _normal(rng: np.random.Generator, shape, sigma: float) -> np.ndarray:
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        out *= np.float32(sigma)
    return out


def make_inputs(cfg: LoryConfig, structured: bool = False, with_dy: bool = True) -> Dict[str, np.ndarray]:
    """Return float32 arrays X[B,L,d], R[d,E], Wg/Wu[E,d,d_ff], Wd[E,d_ff,d]
    and dY[B,L,d].  For bf16 configs every value is already rounded to bf16,
    so widening to float64 (oracle) or narrowing to bf16 (GPU) is exact."""
    ss = np.random.SeedSequence([cfg.seed, 1 if structured else 0])
    kx, kr, kg, ku, kd, ky, km = [np.random.Generator(np.random.Philox(s)) for s in ss.spawn(7)]
    X = _normal(kx, (cfg.B, cfg.L, cfg.d), 1.0)
    if structured:
        mu = _normal(km, (cfg.B, 1, cfg.d), 1.0)
        X += mu
        R = _normal(kr, (cfg.d, cfg.E), 1.0 / np.sqrt(cfg.d))
    else:
        R = _normal(kr, (cfg.d, cfg.E), 0.02)
    out = {
        "X": X,
        "R": R,
        "Wg": _normal(kg, (cfg.E, cfg.d, cfg.d_ff), 0.02),
        "Wu": _normal(ku, (cfg.E, cfg.d, cfg.d_ff), 0.02),
        "Wd": _normal(kd, (cfg.E, cfg.d_ff, cfg.d), 0.02),
    }
    if with_dy:
        out["dY"] = _normal(ky, (cfg.B, cfg.L, cfg.d), 1.0)
    if cfg.dtype == "bf16":
        out = {k: round_to_bf16(v) for k, v in out.items()}
    return out


def make_routing_weights(cfg: LoryConfig, kind: str = "peaked") -> np.ndarray:
    """Routing-weight rows [S,E] to feed the FFN entry points directly
    (they take w as an input).  'uniform' = 1/E, 'onehot' = one expert per
    segment, 'peaked' = random simplex points with a dominant expert."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([cfg.seed, 99])))
    S, E = cfg.S, cfg.E
    if kind == "uniform":
        return np.full((S, E), 1.0 / E, dtype=np.float32)
    if kind == "onehot":
        w = np.zeros((S, E), dtype=np.float32)
        w[np.arange(S), rng.integers(0, E, size=S)] = 1.0
        return w
    if kind == "peaked":
        g = rng.gamma(shape=0.3, size=(S, E)).astype(np.float64) + 1e-6
        return (g / g.sum(axis=1, keepdims=True)).astype(np.float32)
    raise ValueError(kind)
