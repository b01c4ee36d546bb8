"""Seeded synthetic inputs for the five benchmark configurations.

This module holds NO arithmetic of the method (no decode, no masking, no
product): it only draws random weights, activations and binary factors with
numpy and converts between storage dtypes.  Both the CPU oracle's tests and the
GPU path's tests / benchmark take their inputs from here, so neither depends on
the other's random numbers.

The configurations stand in for the layers the paper evaluates (LeNet-5 FC1,
AlexNet FC5/FC6, an LSTM, ResNet convolutions as matrix products, Sec. 2.2 and
Sec. 4); the trained weights and datasets themselves are not used.  Factors are
i.i.d. Bernoulli(p), which by Eq. 7 gives mask density 1 - (1 - p^2)^k.

Recipe: generator numpy.random.default_rng(seed); draw order W, Ip, Iz, X.
  W  ~ N(0, sigma_w) as float32, rounded (nearest-even) to the storage dtype
  Ip [T, r, k] = uniform < p,  Iz [T, k, c] = uniform < p   (uint8 0/1)
  X  ~ N(0, 1) as float32, rounded to the storage dtype
bfloat16 values are carried as uint16 bit patterns (numpy has no bfloat16).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    m: int          # rows of W (outputs)
    n: int          # columns of W (inputs)
    r: int          # tile rows
    c: int          # tile columns
    k: int          # rank of every tile
    p: float        # Bernoulli parameter of both factors
    N: int          # batch (columns of X)
    dtype: str      # "f32" | "f16" | "bf16"
    sigma_w: float
    seed: int = 0

    @property
    def tiles(self) -> int:
        return (-(-self.m // self.r)) * (-(-self.n // self.c))  # edge tiles are cut off at the matrix edge


CONFIGS = {
    # single FC layer (LeNet-5 FC1 shape)
    "C1": Config("C1", 500, 800, 100, 100, 4, 0.16, 1, "f32", 0.05),
    # AlexNet 9216 -> 4096 layer
    "C2": Config("C2", 4096, 9216, 256, 256, 16, 0.08, 128, "f16", 0.01),
    # AlexNet 4096 -> 4096 layer, batch 1 (GEMV) and batch 1024
    "C3a": Config("C3a", 4096, 4096, 512, 512, 32, 0.06, 1, "bf16", 0.015),
    "C3b": Config("C3b", 4096, 4096, 512, 512, 32, 0.06, 1024, "bf16", 0.015),
    # one LSTM layer's gate matrix (4 gates x 1500 rows, input + hidden columns)
    "C4": Config("C4", 6000, 3000, 300, 300, 8, 0.12, 20, "f16", 0.02),
    # 3x3 conv 256 -> 256 as an im2col product (He-normal: sqrt(2 / 2304))
    "C5": Config("C5", 256, 2304, 128, 128, 8, 0.2, 12544, "bf16", 0.029462782549439483),
}

LSTM_STEPS = 35
LSTM_LAYERS = 2
LSTM_HIDDEN = 1500


def scaled(cfg: Config, **kw) -> Config:
    """Same tile shape / rank / p, different matrix size or batch."""
    return replace(cfg, **kw)


# ----------------------------------------------------------------------------
# storage dtypes
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    out = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """float array -> array in the storage dtype (bf16 as uint16 bits)."""
    a = np.asarray(a)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(a.astype(np.float16))
    if dtype == "bf16":
        return f32_to_bf16_bits(a.astype(np.float32))
    raise ValueError(dtype)


def to_float64(s: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a storage array to float64."""
    if dtype == "bf16":
        return bf16_bits_to_f32(s).astype(np.float64)
    return np.asarray(s).astype(np.float64)


# ----------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------

def make_factors(rng, tiles: int, r: int, c: int, k: int, p: float):
    Ip01 = (rng.random((tiles, r, k), dtype=np.float32) < p).astype(np.uint8)
    Iz01 = (rng.random((tiles, k, c), dtype=np.float32) < p).astype(np.uint8)
    return Ip01, Iz01


def make(cfg: Config, want_w: bool = True, want_x: bool = True) -> dict:
    """Inputs of one configuration.  Returns storage-dtype arrays:
    W [m, n], X [n, N], Ip01 [T, r, k], Iz01 [T, k, c]."""
    rng = np.random.default_rng(cfg.seed)
    out = {"cfg": cfg}
    W = rng.standard_normal((cfg.m, cfg.n), dtype=np.float32) * np.float32(cfg.sigma_w)
    out["W"] = to_storage(W, cfg.dtype) if want_w else None
    del W
    out["Ip01"], out["Iz01"] = make_factors(rng, cfg.tiles, cfg.r, cfg.c, cfg.k, cfg.p)
    if want_x:
        X = rng.standard_normal((cfg.n, cfg.N), dtype=np.float32)
        out["X"] = to_storage(X, cfg.dtype)
    else:
        out["X"] = None
    return out


def make_real_factors(cfg: Config, seed_offset: int = 1000) -> dict:
    """Stand-ins for the real-valued non-negative factors that Algorithm 1 thresholds (Sec. 2.2 obtains
    them from an NMF library; none is used here).  Entries are i.i.d. Uniform(0, 1) float32, so that the
    threshold 1 - p turns each factor into Bernoulli(p) bits, the density of the benchmark configurations:
      Mp [T, r, k], Mz [T, k, c] ~ U(0, 1);  Tp = Tz = 1 - p for every tile (float32);
      w_threshold = the value below which W ~ N(0, sigma_w) falls with probability 0.9 in magnitude
      (1.6449 sigma_w: a 90 % magnitude-pruning target, the paper's usual setting)."""
    rng = np.random.default_rng(cfg.seed + seed_offset)
    T = cfg.tiles
    Mp = rng.random((T, cfg.r, cfg.k), dtype=np.float32)
    Mz = rng.random((T, cfg.k, cfg.c), dtype=np.float32)
    Tp = np.full(T, 1.0 - cfg.p, dtype=np.float32)
    Tz = np.full(T, 1.0 - cfg.p, dtype=np.float32)
    return {"Mp": Mp, "Mz": Mz, "Tp": Tp, "Tz": Tz, "w_threshold": float(np.float32(1.6449 * cfg.sigma_w))}


def make_factors_only(cfg: Config) -> dict:
    """Factors of a (possibly scaled) configuration without touching W / X.
    Uses its own stream so very large decode-only grids stay cheap."""
    rng = np.random.default_rng([cfg.seed, 0x1DB1])
    Ip01, Iz01 = make_factors(rng, cfg.tiles, cfg.r, cfg.c, cfg.k, cfg.p)
    return {"cfg": cfg, "Ip01": Ip01, "Iz01": Iz01}


def make_lstm(seed: int = 0, steps: int = LSTM_STEPS, layers: int = LSTM_LAYERS,
              hidden: int = LSTM_HIDDEN, batch: int = 20, r: int = 0, c: int = 0, k: int = 0, p: float = 0.0) -> dict:
    """C4: per layer a (4*hidden) x (2*hidden) fp16 gate matrix with 300x300
    tiles of rank 8 (or tiles r x c of rank k, factor density p), plus the input
    sequence x_t [hidden, batch] for every step."""
    base = CONFIGS["C4"]
    cfg = replace(base, m=4 * hidden, n=2 * hidden, N=batch, seed=seed)
    if r and c and k and p:
        cfg = replace(cfg, r=r, c=c, k=k, p=p)
    rng = np.random.default_rng(seed)
    Ws, Ips, Izs = [], [], []
    for _ in range(layers):
        W = rng.standard_normal((cfg.m, cfg.n), dtype=np.float32) * np.float32(cfg.sigma_w)
        Ws.append(to_storage(W, cfg.dtype))
        Ip01, Iz01 = make_factors(rng, cfg.tiles, cfg.r, cfg.c, cfg.k, cfg.p)
        Ips.append(Ip01)
        Izs.append(Iz01)
    xs = to_storage(rng.standard_normal((steps, hidden, batch), dtype=np.float32), cfg.dtype)
    return {"cfg": cfg, "W": Ws, "Ip01": Ips, "Iz01": Izs, "x": xs,
            "steps": steps, "layers": layers, "hidden": hidden, "batch": batch}
