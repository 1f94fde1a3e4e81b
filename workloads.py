"""Seeded synthetic rating matrices shaped like the paper's workloads (Table 1).

This module only *generates inputs*: index pairs, rating values, the train / holdout
split and the hyper-parameters of each named configuration.  It contains none of the
method's arithmetic (no SGD update, no partition, no RMSE) so that the CPU oracle and
the HIP library can both be fed from it without sharing any code of the method.

The public data sets the paper measures on (MovieLens, Netflix, Yahoo! R1,
Yahoo!Music; Table 1) are not reproduced here.  The generators below take only their
shapes, rating scales and degree skew and stand in for them: ratings come from a
planted low-rank model plus Gaussian noise, index pairs from a truncated-Zipf
Chung-Lu bipartite model.
"""
from __future__ import annotations

import dataclasses
import math
import os
import sys
import time
from typing import Optional

import numpy as np

BASE_SEED = 20061598
_T0 = time.time()


def _progress(msg: str) -> None:
    """Stage messages for the large configurations (MF_VERBOSE=1): generation takes minutes."""
    if os.environ.get("MF_VERBOSE", "0") == "1":
        print(f"[workloads +{time.time() - _T0:6.1f}s] {msg}", file=sys.stderr, flush=True)


@dataclasses.dataclass(frozen=True)
class Config:
    """One named workload.  ``alpha_*`` = Zipf exponent of the target degree sequence
    (0 means uniform).  ``rank``/``mean``/``std`` describe the planted model p*.q*;
    ``post_scale`` multiplies it before the noise is added.  ``step`` is the rounding
    grid of the ratings (0 = no rounding)."""

    name: str
    m: int
    n: int
    nnz_train: int
    nnz_test: int
    k: int
    storage: str          # "f32" or "f16": storage type of the factors on the device
    lr: float
    lam: float
    epochs: int
    alpha_row: float
    alpha_col: float
    rank: int
    mean: float
    std: float
    post_scale: float
    noise: float
    step: float
    lo: float
    hi: float
    uniform_pairs: bool = False   # config 1: pairs uniform without replacement
    sigma_override: Optional[float] = None
    seed: int = BASE_SEED


# Train / holdout sizes: percentage configs split the stated nnz, config 3 holds out
# 1.4 M ratings on top of its 99 M training ratings (as Table 1 lists them separately).
CONFIGS = {
    "tiny": Config("tiny", 2_000, 1_000, 90_000, 10_000, 32, "f32", 0.01, 0.05, 10,
                   0.0, 0.0, 8, 3.0, 0.0, 1.0, 0.1, 0.0, 1.0, 5.0,
                   uniform_pairs=True, sigma_override=1.0 / math.sqrt(8.0), seed=BASE_SEED + 1),
    "medium": Config("medium", 69_878, 10_677, 9_900_000, 100_000, 128, "f32", 0.005, 0.05, 20,
                     1.0, 1.0, 16, 3.5, 1.0, 1.0, 0.2, 0.5, 0.5, 5.0, seed=BASE_SEED + 2),
    "large": Config("large", 480_189, 17_770, 99_000_000, 1_400_000, 128, "f32", 0.005, 0.05, 20,
                    1.1, 0.9, 32, 3.6, 1.0, 1.0, 0.3, 1.0, 1.0, 5.0, seed=BASE_SEED + 3),
    "xlarge": Config("xlarge", 1_000_990, 624_961, 250_272_000, 2_528_000, 128, "f32", 0.001, 0.05, 20,
                     1.0, 1.0, 32, 2.0, 1.0, 25.0, 5.0, 1.0, 0.0, 100.0, seed=BASE_SEED + 4),
    "stress": Config("stress", 2_000_000, 1_000_000, 497_500_000, 2_500_000, 128, "f16", 0.005, 0.05, 10,
                     0.0, 1.2, 64, 3.5, 1.0, 1.0, 0.3, 1.0, 1.0, 5.0, seed=BASE_SEED + 5),
}


def scaled(cfg: Config, factor: float, k: Optional[int] = None) -> Config:
    """Shrink a configuration: nnz by ``factor`` and each axis by sqrt(factor), which
    keeps the density (and so the feasibility of the degree sequence) of the original.
    Used to keep CPU tests and quick GPU cases small."""
    if factor >= 1.0:
        return cfg
    ax = math.sqrt(factor)
    m = max(64, int(cfg.m * ax))
    n = max(64, int(cfg.n * ax))
    tr = max(1000, int(cfg.nnz_train * factor))
    te = max(100, int(cfg.nnz_test * factor))
    return dataclasses.replace(cfg, name=f"{cfg.name}@{factor:g}", m=m, n=n, nnz_train=tr,
                               nnz_test=te, k=k if k is not None else cfg.k)


@dataclasses.dataclass
class Dataset:
    cfg: Config
    rows: np.ndarray      # int32 [nnz_train]
    cols: np.ndarray      # int32 [nnz_train]
    vals: np.ndarray      # float32 [nnz_train]
    test_rows: np.ndarray
    test_cols: np.ndarray
    test_vals: np.ndarray
    max_row_degree: int
    max_col_degree: int
    median_row_degree: float
    median_col_degree: float


def _zipf_degrees(size: int, alpha: float, total: int, cap: float, rng: np.random.Generator) -> np.ndarray:
    """Target degree sequence proportional to rank^-alpha on a random relabelling of
    the ids, capped at ``cap`` and rescaled (bisection on the scale) to sum to total."""
    if alpha == 0.0:
        return np.full(size, total / size)
    base = np.arange(1, size + 1, dtype=np.float64) ** (-alpha)
    lo, hi = 0.0, float(total) * 4.0 / base.sum() * size
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        s = np.minimum(base * mid, cap).sum()
        if s < total:
            lo = mid
        else:
            hi = mid
    d = np.minimum(base * hi, cap)
    relabel = rng.permutation(size)
    out = np.empty(size, dtype=np.float64)
    out[relabel] = d
    return out


def _sample_axis(deg: np.ndarray, count: int, rng: np.random.Generator, what: str = "") -> np.ndarray:
    cdf = np.cumsum(deg)
    cdf /= cdf[-1]
    out = np.empty(count, dtype=np.int64)
    chunk = 1 << 24
    for s in range(0, count, chunk):
        e = min(count, s + chunk)
        out[s:e] = np.searchsorted(cdf, rng.random(e - s), side="right")
        if what and (s // chunk) % 8 == 7:
            _progress(f"{what}: {e} of {count} drawn")
    np.minimum(out, deg.size - 1, out=out)
    return out


def _pairs(cfg: Config, total: int, rng: np.random.Generator):
    m, n = cfg.m, cfg.n
    if cfg.uniform_pairs:
        keys = rng.choice(m * n, size=total, replace=False).astype(np.int64)
    else:
        drow = _zipf_degrees(m, cfg.alpha_row, total, 0.9 * n, rng)
        dcol = _zipf_degrees(n, cfg.alpha_col, total, 0.9 * m, rng)
        keys = np.empty(0, dtype=np.int64)
        want = total
        for rnd in range(64):
            draw = int(want * 1.05) + 1024
            _progress(f"{cfg.name}: pair round {rnd}, drawing {draw}")
            u = _sample_axis(drow, draw, rng, f"{cfg.name} rows")
            v = _sample_axis(dcol, draw, rng, f"{cfg.name} columns")
            _progress(f"{cfg.name}: removing duplicate pairs")
            keys = np.unique(np.concatenate([keys, u * n + v]))
            if keys.size >= total:
                break
            want = total - keys.size
        if keys.size < total:
            raise RuntimeError("pair generator did not reach the requested nnz")
        if keys.size > total:
            keep = rng.choice(keys.size, size=total, replace=False)
            keys = keys[keep]
        # the raw data order is not sorted: apply a seeded shuffle
        keys = keys[rng.permutation(keys.size)]
    u = (keys // n).astype(np.int32)
    v = (keys % n).astype(np.int32)
    return u, v


def _ratings(cfg: Config, u: np.ndarray, v: np.ndarray, rng: np.random.Generator) -> np.ndarray:
    rho = cfg.rank
    mu_e = math.sqrt(cfg.mean / rho)
    if cfg.sigma_override is not None:
        sigma = cfg.sigma_override
    else:
        # Var(p.q) = rho*sigma^4 + 2*mean*sigma^2 == std^2, solved for sigma^2
        sigma = math.sqrt((-cfg.mean + math.sqrt(cfg.mean ** 2 + rho * cfg.std ** 2)) / rho)
    pstar = rng.normal(mu_e, sigma, size=(cfg.m, rho)).astype(np.float32)
    qstar = rng.normal(mu_e, sigma, size=(cfg.n, rho)).astype(np.float32)
    out = np.empty(u.size, dtype=np.float32)
    chunk = 1 << 22
    for s in range(0, u.size, chunk):
        e = min(u.size, s + chunk)
        x = np.einsum("ij,ij->i", pstar[u[s:e]], qstar[v[s:e]]).astype(np.float64)
        x *= cfg.post_scale
        if cfg.noise > 0:
            x += rng.normal(0.0, cfg.noise, size=e - s)
        if cfg.step > 0:
            x = np.round(x / cfg.step) * cfg.step
        np.clip(x, cfg.lo, cfg.hi, out=x)
        out[s:e] = x
    return out


def generate(cfg: Config) -> Dataset:
    """Build the train and holdout COO sets of one configuration (deterministic in
    ``cfg.seed``; the same arrays are handed to the oracle and to the library)."""
    rng = np.random.Generator(np.random.Philox(cfg.seed))
    total = cfg.nnz_train + cfg.nnz_test
    u, v = _pairs(cfg, total, rng)
    _progress(f"{cfg.name}: pairs done, rating values")
    r = _ratings(cfg, u, v, rng)
    _progress(f"{cfg.name}: values done, holdout split")
    hold = np.zeros(total, dtype=bool)
    hold[rng.choice(total, size=cfg.nnz_test, replace=False)] = True
    tr = ~hold
    rd = np.bincount(u[tr], minlength=cfg.m)
    cd = np.bincount(v[tr], minlength=cfg.n)
    return Dataset(cfg, np.ascontiguousarray(u[tr]), np.ascontiguousarray(v[tr]),
                   np.ascontiguousarray(r[tr]), np.ascontiguousarray(u[hold]),
                   np.ascontiguousarray(v[hold]), np.ascontiguousarray(r[hold]),
                   int(rd.max()), int(cd.max()), float(np.median(rd)), float(np.median(cd)))


def planted_noiseless(m: int, n: int, nnz: int, rank: int, seed: int):
    """Exactly rank-``rank`` ratings with no noise, no rounding and no clipping, on
    distinct uniformly drawn pairs: the input of the convergence pin."""
    rng = np.random.Generator(np.random.Philox(seed))
    keys = rng.choice(m * n, size=nnz, replace=False).astype(np.int64)
    u = (keys // n).astype(np.int32)
    v = (keys % n).astype(np.int32)
    ps = rng.uniform(0.2, 1.0, size=(m, rank))
    qs = rng.uniform(0.2, 1.0, size=(n, rank))
    r = np.einsum("ij,ij->i", ps[u], qs[v]).astype(np.float32)
    return u, v, r
