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
RECIPE = 2                # names the cache files: a change of the recipe must not find old data
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


def _stream(seed: int, stage: int, piece: int = 0) -> np.random.Generator:
    """An independent random stream per (configuration seed, stage of the recipe, piece of that
    stage): Philox is keyed, so pieces can be drawn by any number of threads in any order and
    the data do not depend on how many threads there are."""
    return np.random.Generator(np.random.Philox(key=[seed, (stage << 40) | piece]))


def _threads() -> int:
    env = os.environ.get("MF_GEN_THREADS")
    if env:
        return max(1, int(env))
    return max(1, min(16, len(os.sched_getaffinity(0))))


def _parallel(fn, count: int):
    """[fn(0), ..., fn(count-1)], evaluated on a thread pool (numpy releases the interpreter lock
    in the sorts, gathers and generators these pieces consist of)."""
    if count <= 1 or _threads() == 1:
        return [fn(i) for i in range(count)]
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=_threads()) as pool:
        return list(pool.map(fn, range(count)))


_PIECE = 1 << 22          # draws per piece of a stage
_BUCKETS = 64             # key ranges that are de-duplicated independently
# stages of the recipe (first component of a stream's key)
_ST_RELABEL_ROW, _ST_RELABEL_COL, _ST_DRAW, _ST_TRIM, _ST_MIX, _ST_FACTORS, _ST_NOISE, _ST_HOLD = range(1, 9)


def _zipf_degrees(size: int, alpha: float, total: int, cap: float, rng: np.random.Generator) -> np.ndarray:
    """Target degree sequence proportional to rank^-alpha on a random relabelling of
    the ids, capped at ``cap`` and rescaled (bisection on the scale) to sum to total."""
    if alpha == 0.0:
        return np.full(size, total / size)
    base = np.arange(1, size + 1, dtype=np.float64) ** (-alpha)
    lo, hi = 0.0, float(total) * 4.0 / base.sum() * size
    for _ in range(100):
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


def _cdf(deg: np.ndarray) -> np.ndarray:
    cdf = np.cumsum(deg)
    cdf /= cdf[-1]
    return cdf


def _draw_sorted(cdf: np.ndarray, count: int, rng: np.random.Generator) -> np.ndarray:
    """``count`` ids drawn from the distribution with this cumulative table, in ascending order
    (sorted uniforms make the table look-up sequential)."""
    x = rng.random(count)
    x.sort()
    out = np.searchsorted(cdf, x, side="right")
    np.minimum(out, cdf.size - 1, out=out)
    return out


def _pairs_sorted(cfg: Config, total: int):
    """``total`` distinct (u, v) pairs as ascending keys u*n + v, in _BUCKETS consecutive key ranges."""
    m, n = cfg.m, cfg.n
    crow = _cdf(_zipf_degrees(m, cfg.alpha_row, total, 0.9 * n, _stream(cfg.seed, _ST_RELABEL_ROW)))
    ccol = _cdf(_zipf_degrees(n, cfg.alpha_col, total, 0.9 * m, _stream(cfg.seed, _ST_RELABEL_COL)))
    # key ranges of about equal mass: boundaries at the rows where the row table crosses j/_BUCKETS
    edges = np.searchsorted(crow, np.arange(1, _BUCKETS) / _BUCKETS, side="right").astype(np.int64) * n
    buckets = None                                     # round 0: ascending distinct keys per range
    extra = [np.empty(0, dtype=np.int64) for _ in range(_BUCKETS)]   # keys the later rounds add
    have, want, kept_share = 0, total, 1.0
    for rnd in range(64):
        # later rounds replace what the duplicates took away; many of their draws are duplicates
        # again (they fall on the dense corner of hot rows and hot columns), so they draw more by
        # the share of the previous round's draws that was kept
        draw = int(want * (1.05 if rnd == 0 else 1.02 / max(0.25, 0.8 * kept_share))) + 1024
        pieces = (draw + _PIECE - 1) // _PIECE
        _progress(f"{cfg.name}: pair round {rnd}, drawing {draw}")

        def one_piece(i, rnd=rnd, draw=draw):
            cnt = min(_PIECE, draw - i * _PIECE)
            rng = _stream(cfg.seed, _ST_DRAW, (rnd << 24) | i)
            u = _draw_sorted(crow, cnt, rng)
            v = _draw_sorted(ccol, cnt, rng)
            # rows ascending, columns in a random order: the two are drawn independently
            key = u * n + v[rng.permutation(cnt)]
            key.sort()
            return key, np.searchsorted(key, edges)

        drawn = _parallel(one_piece, pieces)
        _progress(f"{cfg.name}: removing duplicate pairs")

        def one_bucket(j, first_round=(rnd == 0)):
            parts = [] if first_round else [extra[j]]
            for key, cut in drawn:
                lo = cut[j - 1] if j > 0 else 0
                hi = cut[j] if j < _BUCKETS - 1 else key.size
                parts.append(key[lo:hi])
            keys = np.unique(np.concatenate(parts))
            if first_round:
                return keys
            # keep only keys that round 0 does not hold already
            main = buckets[j]
            at = np.minimum(np.searchsorted(main, keys), main.size - 1)
            return keys[main[at] != keys] if main.size else keys

        if rnd == 0:
            buckets = _parallel(one_bucket, _BUCKETS)
        else:
            extra = _parallel(one_bucket, _BUCKETS)
        del drawn
        before = have
        have = sum(b.size for b in buckets) + sum(x.size for x in extra)
        kept_share = (have - before) / draw
        if have >= total:
            break
        want = total - have
    if have < total:
        raise RuntimeError("pair generator did not reach the requested nnz")
    buckets = _parallel(lambda j: np.union1d(buckets[j], extra[j]) if extra[j].size else buckets[j], _BUCKETS)
    if have > total:
        # drop the surplus: every key range gives up its share (the remainder comes from the first
        # ranges), at seeded random positions
        surplus = have - total
        sizes = [b.size for b in buckets]
        quota = [surplus * sz // have for sz in sizes]
        left, j = surplus - sum(quota), 0
        while left > 0:
            if sizes[j % _BUCKETS] > quota[j % _BUCKETS]:
                quota[j % _BUCKETS] += 1
                left -= 1
            j += 1

        def trim(j):
            if quota[j] == 0:
                return buckets[j]
            gone = _stream(cfg.seed, _ST_TRIM, j).choice(sizes[j], size=quota[j], replace=False)
            return np.delete(buckets[j], gone)

        buckets = _parallel(trim, _BUCKETS)
    return buckets


def _planted(cfg: Config):
    rho = cfg.rank
    mu_e = math.sqrt(cfg.mean / rho)
    if cfg.sigma_override is not None:
        sigma = cfg.sigma_override
    else:
        # Var(p.q) = rho*sigma^4 + 2*mean*sigma^2 == std^2, solved for sigma^2
        sigma = math.sqrt((-cfg.mean + math.sqrt(cfg.mean ** 2 + rho * cfg.std ** 2)) / rho)
    pstar = _stream(cfg.seed, _ST_FACTORS, 0).normal(mu_e, sigma, size=(cfg.m, rho)).astype(np.float32)
    qstar = _stream(cfg.seed, _ST_FACTORS, 1).normal(mu_e, sigma, size=(cfg.n, rho)).astype(np.float32)
    return pstar, qstar


def _ratings(cfg: Config, pstar, qstar, u: np.ndarray, v: np.ndarray, rng: np.random.Generator) -> np.ndarray:
    out = np.empty(u.size, dtype=np.float32)
    step = 1 << 16          # temporaries of a step stay in the caches
    for s in range(0, u.size, step):
        e = min(u.size, s + step)
        x = np.einsum("ij,ij->i", pstar[u[s:e]], qstar[v[s:e]]).astype(np.float64)
        x *= cfg.post_scale
        if cfg.noise > 0:
            x += rng.normal(0.0, cfg.noise, size=e - s)
        if cfg.step > 0:
            x = np.round(x / cfg.step) * cfg.step
        np.clip(x, cfg.lo, cfg.hi, out=x)
        out[s:e] = x
    return out


def _coprime_stride(count: int) -> int:
    a = max(1, int(count * 0.6180339887498949))
    while math.gcd(a, count) != 1:
        a += 1
    return a


def generate(cfg: Config) -> Dataset:
    """Build the train and holdout COO sets of one configuration (deterministic in
    ``cfg.seed`` and independent of the number of threads; the same arrays are handed to the
    oracle and to the library)."""
    total = cfg.nnz_train + cfg.nnz_test
    m, n = cfg.m, cfg.n
    if cfg.uniform_pairs:
        keys = np.sort(_stream(cfg.seed, _ST_DRAW).choice(m * n, size=total, replace=False).astype(np.int64))
        cuts = [(total * j) // _BUCKETS for j in range(_BUCKETS + 1)]
        buckets = [keys[cuts[j]:cuts[j + 1]] for j in range(_BUCKETS)]
    else:
        buckets = _pairs_sorted(cfg, total)
    _progress(f"{cfg.name}: pairs done, rating values")
    pstar, qstar = _planted(cfg)

    # per key range: rating values (rows ascending, so the planted row factors are read in
    # order), then a seeded order inside the range
    def one_bucket(j):
        key = buckets[j]
        u, v = np.divmod(key, n)
        r = _ratings(cfg, pstar, qstar, u, v, _stream(cfg.seed, _ST_NOISE, j))
        order = _stream(cfg.seed, _ST_MIX, j).permutation(key.size)
        return key[order], r[order]

    mixed = _parallel(one_bucket, _BUCKETS)
    del buckets
    keys = np.concatenate([k for k, _ in mixed])
    vals = np.concatenate([r for _, r in mixed])
    del mixed
    _progress(f"{cfg.name}: values done, interleaving the key ranges")
    # the raw order of the data is not sorted: position i takes element (i*a + b) mod total of
    # the range-by-range arrays, a coprime to total (consecutive positions come from key ranges
    # far apart, and inside a range the order is random)
    a = _coprime_stride(total)
    b = int(_stream(cfg.seed, _ST_MIX, _BUCKETS).integers(0, total))
    # holdout: the first nnz_test distinct positions (of the interleaved order) of a seeded stream
    cand = _stream(cfg.seed, _ST_HOLD).integers(0, total, size=cfg.nnz_test + cfg.nnz_test // 4 + 1024)
    uniq, first = np.unique(cand, return_index=True)
    if uniq.size < cfg.nnz_test:
        raise RuntimeError("holdout stream too short")
    hold = np.sort(uniq[np.argsort(first, kind="stable")[:cfg.nnz_test]])
    u = np.empty(cfg.nnz_train, dtype=np.int32)
    v = np.empty(cfg.nnz_train, dtype=np.int32)
    r = np.empty(cfg.nnz_train, dtype=np.float32)
    tu = np.empty(cfg.nnz_test, dtype=np.int32)
    tv = np.empty(cfg.nnz_test, dtype=np.int32)
    tr_ = np.empty(cfg.nnz_test, dtype=np.float32)
    pieces = (total + _PIECE - 1) // _PIECE

    def one_piece(i):
        s, e = i * _PIECE, min(total, (i + 1) * _PIECE)
        src = (np.arange(s, e, dtype=np.int64) * a + b) % total
        key = keys[src]
        pu, pv = np.divmod(key, n)
        pr = vals[src]
        lo, hi = np.searchsorted(hold, [s, e])          # held-out positions of this piece
        held = np.zeros(e - s, dtype=bool)
        held[hold[lo:hi] - s] = True
        tu[lo:hi], tv[lo:hi], tr_[lo:hi] = pu[held], pv[held], pr[held]
        keep = ~held
        u[s - lo:e - hi], v[s - lo:e - hi], r[s - lo:e - hi] = pu[keep], pv[keep], pr[keep]

    _parallel(one_piece, pieces)
    del keys, vals
    _progress(f"{cfg.name}: degrees")
    groups = min(8, pieces)
    edges = [(cfg.nnz_train * g) // groups for g in range(groups + 1)]
    counts = _parallel(lambda g: (np.bincount(u[edges[g]:edges[g + 1]], minlength=m),
                                  np.bincount(v[edges[g]:edges[g + 1]], minlength=n)), groups)
    rd = sum(c[0] for c in counts)
    cd = sum(c[1] for c in counts)
    _progress(f"{cfg.name}: done")
    return Dataset(cfg, u, v, r, tu, tv, tr_,
                   int(rd.max()), int(cd.max()), float(np.median(rd)), float(np.median(cd)))


_FIELDS = ["rows", "cols", "vals", "test_rows", "test_cols", "test_vals", "max_row_degree",
           "max_col_degree", "median_row_degree", "median_col_degree"]
_mem = {}


def load(name: str, factor: float = 1.0, k: Optional[int] = None, keep: bool = True) -> Dataset:
    """generate(scaled(CONFIGS[name], factor, k)), remembered in this process and, for sets of
    1 M to 20 M ratings, in an .npz file under MF_DATA_CACHE (default: .cache beside this file)."""
    cfg = scaled(CONFIGS[name], factor, k)
    key = f"{name}_{factor:g}"
    if key in _mem:
        return Dataset(cfg, *[getattr(_mem[key], f) for f in _FIELDS])
    cache = os.environ.get("MF_DATA_CACHE", os.path.join(os.path.dirname(os.path.abspath(__file__)), ".cache"))
    path = os.path.join(cache, f"{key}_seed{cfg.seed}_recipe{RECIPE}.npz")
    on_disk = 1_000_000 <= cfg.nnz_train <= 20_000_000
    if on_disk and os.path.exists(path):
        z = np.load(path)
        ds = Dataset(cfg, *[z[f] if z[f].ndim else z[f].item() for f in _FIELDS])
    else:
        ds = generate(cfg)
        if on_disk:
            try:
                os.makedirs(cache, exist_ok=True)
                np.savez(path, **{f: getattr(ds, f) for f in _FIELDS})
            except OSError:
                pass
    if keep:
        _mem[key] = ds
    return ds


def forget(name: Optional[str] = None) -> None:
    """Drop remembered data sets (all, or those of one configuration): the large ones take GBs."""
    for key in list(_mem):
        if name is None or key.startswith(name + "_"):
            del _mem[key]


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
