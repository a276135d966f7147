"""Seeded synthetic inputs for the APB layer forward pass.

This module only draws random tensors with the shapes, value distributions
and outlier structure of CNN layers lowered to matrix products (the paper's
efficiency evaluation multiplies im2col-shaped operands of ResNet-like
layers).  It holds none of the method's arithmetic: no partition rule, no
quantizer, no packing.  Both the CPU oracle's tests and the HIP path's tests
and benchmark take their inputs from here, so the two sides always see the
same numbers.

Notation: W is N x K (output channels x C_in*kh*kw), X is K x M (M = batch *
H_out * W_out im2col columns), delta is the half-width of the binarization
interval (the paper's alpha + delta in the definition of the APB operator).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

BASE_SEED = 230608960


@dataclass(frozen=True)
class LayerConfig:
    name: str
    index: int            # position in the benchmark's config list (seeds derive from it)
    N: int
    K: int
    M: int
    bits: int             # activation bits: 1 (sign) or 2 (uniform codes 0..3)
    rho: float            # fraction of weights outside the binarization interval
    weight_dist: str      # "normal" | "laplace" | "zipf_rows"
    weight_scale: float   # std (normal) or b (laplace)
    step: float           # activation step: beta (1-bit) or s (2-bit)
    note: str = ""


CONFIGS: Dict[str, LayerConfig] = {}


def _add(cfg: LayerConfig) -> None:
    CONFIGS[cfg.name] = cfg


_add(LayerConfig("C1", 0, 256, 256, 64, 1, 0.01, "normal", 0.05, 1.0,
                 "fully-connected 256x256, batch 64, 1-bit activations"))
_add(LayerConfig("C2", 1, 64, 576, 131072, 2, 0.02, "normal", 0.05, 0.75,
                 "3x3 conv 64->64 on 32x32 maps, batch 128"))
for _r, _tag in ((0.005, "r05"), (0.02, "r20"), (0.05, "r50")):
    for _b in (1, 2):
        _add(LayerConfig(f"C3_{_tag}_b{_b}", 2, 256, 2304, 8192, _b, _r, "normal", 0.05,
                         1.0 if _b == 1 else 0.75,
                         "3x3 conv 256->256 on 8x8 maps, batch 128"))
_add(LayerConfig("C4", 3, 128, 1152, 50176, 2, 0.01, "zipf_rows", 0.05, 0.75,
                 "3x3 conv 128->128 on 28x28 maps, batch 64, Zipf(1.1) outliers per row"))
_add(LayerConfig("C5a", 4, 4096, 4096, 256, 2, 0.03, "laplace", 0.02, 0.75,
                 "fully-connected 4096x4096, batch 256"))
_add(LayerConfig("C5b", 4, 512, 4608, 12544, 2, 0.03, "laplace", 0.02, 0.75,
                 "3x3 conv 512->512 on 7x7 maps, batch 256"))


def small_variant(cfg: LayerConfig, N: Optional[int] = None, K: Optional[int] = None,
                  M: Optional[int] = None) -> LayerConfig:
    """Same distributions, smaller shape (for parity cases the oracle finishes fast)."""
    return replace(cfg, name=cfg.name + "_small", N=N or cfg.N, K=K or cfg.K, M=M or cfg.M)


def _rng(cfg: LayerConfig, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=BASE_SEED + cfg.index + 1000 * stream))


def _delta_for_rate(W: np.ndarray, rho: float) -> np.float32:
    """Largest |w| that stays inside the interval when floor(rho*N*K) weights are left outside."""
    a = np.abs(W).ravel()
    n_out = int(np.floor(rho * a.size))
    if n_out <= 0:
        return np.float32(a.max())
    if n_out >= a.size:
        return np.float32(-1.0)
    kth = a.size - n_out - 1                      # index of the largest inlier in sorted order
    part = np.partition(a, kth)
    return np.float32(part[kth])


def make_weights(cfg: LayerConfig):
    """Return (W float32 [N,K], delta float32)."""
    N, K = cfg.N, cfg.K
    g = _rng(cfg, 1)
    if cfg.weight_dist == "normal":
        W = (g.standard_normal((N, K)) * cfg.weight_scale).astype(np.float32)
        return W, _delta_for_rate(W, cfg.rho)
    if cfg.weight_dist == "laplace":
        W = g.laplace(0.0, cfg.weight_scale, (N, K)).astype(np.float32)
        return W, _delta_for_rate(W, cfg.rho)
    if cfg.weight_dist == "zipf_rows":
        delta = np.float32(2.576 * cfg.weight_scale)
        W = (g.standard_normal((N, K)) * cfg.weight_scale).astype(np.float32)
        bad = np.abs(W) > delta
        while bad.any():                           # inliers: resample until inside the interval
            W[bad] = (g.standard_normal(int(bad.sum())) * cfg.weight_scale).astype(np.float32)
            bad = np.abs(W) > delta
        gs = _rng(cfg, 3)
        total = int(round(cfg.rho * N * K))
        ranks = gs.permutation(N) + 1              # rank 1 = heaviest row
        weight = ranks.astype(np.float64) ** -1.1
        counts = np.rint(total * weight / weight.sum()).astype(np.int64)
        counts = np.minimum(counts, K)
        for n in range(N):
            c = int(counts[n])
            if c == 0:
                continue
            cols = gs.choice(K, size=c, replace=False)
            mag = float(delta) * (1.0 + gs.exponential(1.0, c)) + 1e-4
            sgn = gs.integers(0, 2, c) * 2 - 1
            W[n, cols] = (mag * sgn).astype(np.float32)
        return W, delta
    raise ValueError(cfg.weight_dist)


def make_acts(cfg: LayerConfig) -> np.ndarray:
    """Return X float32 [K,M]: N(0,1) draws (1-bit) or their ReLU (2-bit), already in im2col layout."""
    g = _rng(cfg, 2)
    X = g.standard_normal((cfg.K, cfg.M), dtype=np.float32)
    if cfg.bits == 2:
        np.maximum(X, 0.0, out=X)
    return X


def make_layer(cfg: LayerConfig):
    """Return (W, delta, X, step)."""
    W, delta = make_weights(cfg)
    return W, delta, make_acts(cfg), np.float32(cfg.step)


def random_case(seed: int, N: int, K: int, M: int, bits: int, rho: float = 0.03,
                dist: str = "normal"):
    """Small free-form case for edge-shape tests: returns (W, delta, X, step)."""
    cfg = LayerConfig(f"rand{seed}", seed, N, K, M, bits, rho, dist,
                      0.05 if dist != "laplace" else 0.02, 1.0 if bits == 1 else 0.75)
    return make_layer(cfg)
