"""Seeded synthetic workloads (inputs only -- none of the method's arithmetic lives here).

The paper measures on SIFT1M / Deep1M / GIST1M (Table 1), which are not available
offline.  The five configurations below take their shapes, value ranges and
rough statistics and stand in for them; both the CPU oracle's tests and the GPU
tests / benchmark draw their inputs from this one module.

Every array is produced by numpy's ``Generator(PCG64(seed))`` in fixed-size row
chunks, so a given (config, seed) always yields the same bytes for a given numpy
version; ``sha256_of`` lets a run record what it actually used.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass

import numpy as np

CHUNK = 65536  # rows generated per RNG call sequence; part of the recipe

BUILD_SEED = 2310


@dataclass(frozen=True)
class Config:
    name: str
    N: int
    d: int
    dtype: str      # "u8" or "f32"
    S: int
    R: int
    T1: int
    T2: int
    n_queries: int
    data_seed: int
    kind: str       # which generator

    @property
    def query_seed(self) -> int:
        return self.data_seed + 1000


CONFIGS = {
    "cfg1": Config("cfg1", 5_000, 32, "u8", 10, 32, 2, 4, 100, 20420, "gauss_u8"),
    "cfg2": Config("cfg2", 100_000, 128, "u8", 20, 96, 4, 15, 1_000, 20421, "heavy_u8"),
    "cfg3": Config("cfg3", 1_000_000, 128, "u8", 20, 96, 4, 15, 10_000, 20422, "heavy_u8"),
    "cfg4": Config("cfg4", 1_000_000, 96, "f32", 20, 96, 4, 15, 10_000, 20423, "unit_f32"),
    "cfg5": Config("cfg5", 1_000_000, 960, "f32", 20, 96, 4, 15, 1_000, 20424, "beta_f32"),
}


def sha256_of(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


# ------------------------------------------------------------------ generators
class _GaussU8:
    """16-component Gaussian mixture, means ~ U[32,224] per dim, sigma 20, rounded, clipped."""

    def __init__(self, d, seed):
        g = np.random.Generator(np.random.PCG64(seed))
        self.mu = g.uniform(32.0, 224.0, size=(16, d))

    def rows(self, g, n):
        k = g.integers(0, 16, size=n)
        x = self.mu[k] + g.normal(0.0, 20.0, size=(n, self.mu.shape[1]))
        return np.clip(np.rint(x), 0, 255).astype(np.uint8)


class _HeavyU8:
    """256 clusters of non-negative heavy-tailed features (local-descriptor-like).

    Centre c_k[j] ~ Gamma(0.5, 30); each cluster switches a feature on with
    probability P_ON; a sample is round(clip(on * c_k[j] + Gamma(0.5, 30) - 15, 0, 255)),
    which leaves about 40 % exact zeros.
    """
    P_ON = 0.5

    def __init__(self, d, seed):
        g = np.random.Generator(np.random.PCG64(seed))
        c = g.gamma(0.5, 30.0, size=(256, d))
        on = g.random(size=(256, d)) < self.P_ON
        self.centre = c * on + 12.0 * on

    def rows(self, g, n):
        k = g.integers(0, 256, size=n)
        x = self.centre[k] + g.gamma(0.5, 30.0, size=(n, self.centre.shape[1])) - 15.0
        return np.clip(np.rint(x), 0, 255).astype(np.uint8)


class _UnitF32:
    """1,024-component Gaussian mixture (centres ~ N(0, I), within-cluster sigma 0.5), L2-normalised."""

    def __init__(self, d, seed):
        g = np.random.Generator(np.random.PCG64(seed))
        self.mu = g.normal(0.0, 1.0, size=(1024, d))

    def rows(self, g, n):
        k = g.integers(0, 1024, size=n)
        x = self.mu[k] + g.normal(0.0, 0.5, size=(n, self.mu.shape[1]))
        x /= np.linalg.norm(x, axis=1, keepdims=True)
        return x.astype(np.float32)


class _BetaF32:
    """512 centres ~ Beta(2,5) per dim; x = 0.5 c_k + 0.25 f_group + 0.25 e, f per group of 32 dims."""

    def __init__(self, d, seed):
        assert d % 32 == 0
        g = np.random.Generator(np.random.PCG64(seed))
        self.c = g.beta(2.0, 5.0, size=(512, d)).astype(np.float32)
        self.d = d

    def rows(self, g, n):
        k = g.integers(0, 512, size=n)
        f = g.beta(2.0, 5.0, size=(n, self.d // 32)).astype(np.float32)
        e = g.beta(2.0, 5.0, size=(n, self.d)).astype(np.float32)
        x = 0.5 * self.c[k] + 0.25 * np.repeat(f, 32, axis=1) + 0.25 * e
        return x.astype(np.float32)


_KINDS = {"gauss_u8": _GaussU8, "heavy_u8": _HeavyU8, "unit_f32": _UnitF32, "beta_f32": _BetaF32}


def _generate(kind: str, d: int, model_seed: int, sample_seed: int, n: int) -> np.ndarray:
    model = _KINDS[kind](d, model_seed)
    g = np.random.Generator(np.random.PCG64(sample_seed))
    out = np.empty((n, d), np.uint8 if kind.endswith("u8") else np.float32)
    for lo in range(0, n, CHUNK):
        hi = min(n, lo + CHUNK)
        out[lo:hi] = model.rows(g, hi - lo)
    return out


def make_data(cfg: Config, N: int | None = None) -> np.ndarray:
    """Database vectors of a configuration (optionally only the first N rows' worth of draws)."""
    n = cfg.N if N is None else N
    return _generate(cfg.kind, cfg.d, cfg.data_seed, cfg.data_seed + 1, n)


def make_queries(cfg: Config, n: int | None = None) -> np.ndarray:
    """Queries from the same mixture (same centres), independent sample stream."""
    n = cfg.n_queries if n is None else n
    return _generate(cfg.kind, cfg.d, cfg.data_seed, cfg.query_seed, n)


def custom(kind: str, N: int, d: int, seed: int) -> np.ndarray:
    """Same generators at an arbitrary shape, for parity cases between the named configs."""
    return _generate(kind, d, seed, seed + 1, N)


def describe(X: np.ndarray) -> dict:
    x = X[: min(len(X), 20000)].astype(np.float64)
    return {
        "shape": list(X.shape), "dtype": str(X.dtype),
        "zero_frac": float((x == 0).mean()), "mean": float(x.mean()),
        "mean_sq_norm": float((x * x).sum(1).mean()),
    }
