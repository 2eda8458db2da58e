"""Seeded synthetic inputs for the soft-k-means quantisation layer.

This module only *draws inputs*: weight tensors, initial codebooks and upstream
gradients.  It holds none of the method's arithmetic, so both the CPU oracle's
tests and the HIP path's tests can be fed from it without sharing any
computation.  numpy only.

The paper clusters the weights of a fine-tuned ResNet18 (Experiments, "Resnet18
on CIFAR10").  Those weights are not available offline; the stand-ins below take
only the layer *shapes* and draw values Kaiming-normal (std = sqrt(2/fan_in)).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

DIST_L2 = 0    # energy = ||w - c||      (the paper's attention, Eq. "aterms")
DIST_SQL2 = 1  # energy = ||w - c||^2    (the squared variant)
DIST_NAMES = {DIST_L2: "L2", DIST_SQL2: "SQL2"}


@dataclass(frozen=True)
class Config:
    name: str
    m: int
    d: int
    k: int
    std: float
    w_seed: int
    c0: str            # "quantile" | "rows"
    c0_seed: int
    tau: float
    tol: float
    max_iter: int
    g_seed: int
    g_kind: str        # "normal" (G ~ N(0, g_std^2)) | "target" (T ~ N(0, std^2); G = 2 (Wq - T))
    g_std: float = 1e-4
    note: str = ""


_STD_C3 = math.sqrt(2.0 / 4608.0)

CONFIGS = {
    "C1": Config("C1", 4096, 1, 4, 0.05, 1001, "quantile", 0, 1e-3, 1e-6, 100, 3001, "target",
                 note="tiny scalar case"),
    "C2": Config("C2", 589_824, 1, 16, math.sqrt(2.0 / 2304.0), 1002, "quantile", 0, 1e-4, 1e-6, 200,
                 3002, "normal", note="3x3x256x256 conv, 4 bits per weight"),
    "C3": Config("C3", 2_359_296, 1, 4, _STD_C3, 1003, "quantile", 0, 5e-5, 1e-7, 500,
                 3003, "normal", note="3x3x512x512 conv, 2 bits per weight"),
    "C4": Config("C4", 589_824, 4, 256, _STD_C3, 1003, "rows", 1004, 2e-4, 1e-6, 200,
                 3004, "normal", note="3x3x512x512 conv as 4-vectors, 8 bits per vector"),
    # the largest codebook of the paper's ResNet18 table (k = 16, d = 4: one bit per weight) on the same tensor;
    # temperature as C4's (same vectors, squared energy)
    "P16": Config("P16", 589_824, 4, 16, _STD_C3, 1003, "rows", 1006, 2e-4, 1e-6, 200,
                  3006, "normal", note="3x3x512x512 conv as 4-vectors, 4 bits per vector"),
    # beyond the paper's networks: a layer whose weights do not fit the chip's LDS (64 MiB), so every pass streams
    # W from memory; temperature tied to C3's as in the sweep (squared energy)
    "XL": Config("XL", 16_777_216, 1, 4, math.sqrt(2.0 / 4096.0), 1005, "quantile", 0,
                 5e-5 * (2.0 / 4096.0) / (2.0 / 4608.0), 1e-7, 200, 3005, "normal",
                 note="4096x4096 linear layer, 2 bits per weight"),
}

# ResNet18 tensors for the whole-network sweep: (number of weights, fan_in).
RESNET18_TENSORS = (
    [(7 * 7 * 3 * 64, 147)]
    + [(3 * 3 * 64 * 64, 576)] * 4
    + [(3 * 3 * 64 * 128, 576)] + [(3 * 3 * 128 * 128, 1152)] * 3 + [(1 * 1 * 64 * 128, 64)]
    + [(3 * 3 * 128 * 256, 1152)] + [(3 * 3 * 256 * 256, 2304)] * 3 + [(1 * 1 * 128 * 256, 128)]
    + [(3 * 3 * 256 * 512, 2304)] + [(3 * 3 * 512 * 512, 4608)] * 3 + [(1 * 1 * 256 * 512, 256)]
    + [(512 * 1000, 512)]
)


def sweep_config(idx: int, k: int, dist: int) -> Config:
    """Config of tensor `idx` of the ResNet18 sweep at k centroids.

    The sweep names no temperature; tau is tied to the 3x3x512x512 setting
    (5e-5 at std sqrt(2/4608)) and scaled with the layer's std (power 1 for
    the plain norm, 2 for the squared one) so every layer is equally soft.
    """
    n, fan_in = RESNET18_TENSORS[idx]
    std = math.sqrt(2.0 / fan_in)
    p = 1 if dist == DIST_L2 else 2
    tau = 5e-5 * (std / _STD_C3) ** p
    return Config(f"C5[{idx}]k{k}", n, 1, k, std, 2000 + idx, "quantile", 0, tau, 1e-6, 200,
                  4000 + idx, "normal")


@dataclass
class Problem:
    cfg: Config
    dist: int
    W: np.ndarray               # float32 [m, d]
    C0: np.ndarray              # float32 [k, d]
    G: Optional[np.ndarray]     # float32 [m, d], upstream dL/dWq ("normal" kind)
    T: Optional[np.ndarray]     # float32 [m, d], regression target ("target" kind)
    tau: float = field(init=False)
    tol: float = field(init=False)
    max_iter: int = field(init=False)

    def __post_init__(self):
        self.tau, self.tol, self.max_iter = self.cfg.tau, self.cfg.tol, self.cfg.max_iter


def draw_weights(n: int, std: float, seed: int) -> np.ndarray:
    """n values ~ N(0, std^2): float64 draws scaled, then rounded to float32."""
    return (np.random.default_rng(seed).standard_normal(n) * std).astype(np.float32)


def quantile_codebook(W: np.ndarray, k: int) -> np.ndarray:
    """Evenly spaced quantiles of the scalar weights: c_j = quantile((j + 1/2) / k)."""
    assert W.shape[1] == 1
    qs = (np.arange(k, dtype=np.float64) + 0.5) / k
    c = np.quantile(W[:, 0].astype(np.float64), qs)
    return c.astype(np.float32).reshape(k, 1)


def row_codebook(W: np.ndarray, k: int, seed: int) -> np.ndarray:
    """k distinct rows of W, in drawn order."""
    idx = np.random.default_rng(seed).choice(W.shape[0], size=k, replace=False)
    return W[idx].copy()


def make_problem(cfg, dist: int, m: Optional[int] = None) -> Problem:
    """Draw the inputs of one config.  `m` overrides the row count (reduced-size parity cases)."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    if m is not None and m != cfg.m:
        cfg = Config(**{**cfg.__dict__, "m": int(m), "name": f"{cfg.name}@m={m}"})
    W = draw_weights(cfg.m * cfg.d, cfg.std, cfg.w_seed).reshape(cfg.m, cfg.d)
    if cfg.c0 == "quantile":
        C0 = quantile_codebook(W, cfg.k)
    else:
        C0 = row_codebook(W, cfg.k, cfg.c0_seed)
    G = T = None
    if cfg.g_kind == "normal":
        G = draw_weights(cfg.m * cfg.d, cfg.g_std, cfg.g_seed).reshape(cfg.m, cfg.d)
    else:
        T = draw_weights(cfg.m * cfg.d, cfg.std, cfg.g_seed).reshape(cfg.m, cfg.d)
    return Problem(cfg, dist, W, C0, G, T)


def random_problem(m: int, d: int, k: int, seed: int, std: float = 1.0, spread: float = 1.0):
    """Small generic clustered problem for unit tests: k blobs of std `std` around centres ~ N(0, spread^2).

    Returns float64 W [m,d], C0 [k,d] (k distinct rows of W) and G [m,d].
    """
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((k, d)) * spread
    lab = rng.integers(0, k, size=m)
    W = centres[lab] + rng.standard_normal((m, d)) * std
    C0 = W[rng.choice(m, size=k, replace=False)].copy()
    G = rng.standard_normal((m, d))
    return W, C0, G
