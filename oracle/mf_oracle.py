"""ctypes front end of the C oracle (oracle/mf_oracle.c).  Test infrastructure only.

All factor state is held as float64 numpy arrays whatever the `arith` (see the C file's
header); index arrays are int32, ratings float32, perm / block_ptr int64.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

ARITH_F64, ARITH_F32, ARITH_F16 = 0, 1, 2
SPLIT_EQUAL_WIDTH, SPLIT_NNZ_BALANCED, SPLIT_NNZ_WIDTH_BALANCED = 0, 1, 2

__all__ = ["ARITH_F64", "ARITH_F32", "ARITH_F16", "SPLIT_EQUAL_WIDTH", "SPLIT_NNZ_BALANCED",
           "SPLIT_NNZ_WIDTH_BALANCED", "bounds_nnz_width_balanced",
           "round_f16", "init_factors", "partition", "blocks_independent", "sgd_step",
           "sgd_epoch", "sgd_epoch_omp", "sgd_sweep", "predict", "rating_loss", "rmse",
           "num_threads", "bounds_equal_width", "bounds_nnz_balanced", "mix64", "stratum_order",
           "sgd_epoch_ordered", "row_rank"]

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.mfo_round_f16.restype = C.c_double
        _lib.mfo_round_f16.argtypes = [C.c_double]
        _lib.mfo_predict.restype = C.c_double
        _lib.mfo_rating_loss.restype = C.c_double
        _lib.mfo_rmse.restype = C.c_double
    return _lib


def _p(a, dtype):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, (a.dtype, dtype)
    return a.ctypes.data_as(C.c_void_p)


def round_f16(x: float) -> float:
    return float(_load().mfo_round_f16(float(x)))


def init_factors(count: int, seed: int, stream: int, scale: float, arith: int = ARITH_F64) -> np.ndarray:
    x = np.empty(count, dtype=np.float64)
    _load().mfo_init_factors(_p(x, np.float64), C.c_int64(count), C.c_uint64(seed), C.c_uint64(stream),
                             C.c_float(scale), C.c_int(arith))
    return x


def bounds_equal_width(size: int, G: int) -> np.ndarray:
    b = np.empty(G + 1, dtype=np.int32)
    _load().mfo_bounds_equal_width(C.c_int64(size), C.c_int32(G), _p(b, np.int32))
    return b


def bounds_nnz_balanced(idx: np.ndarray, size: int, G: int) -> np.ndarray:
    b = np.empty(G + 1, dtype=np.int32)
    rc = _load().mfo_bounds_nnz_balanced(_p(idx, np.int32), C.c_int64(idx.size), C.c_int64(size),
                                         C.c_int32(G), _p(b, np.int32))
    assert rc == 0
    return b


def bounds_nnz_width_balanced(idx: np.ndarray, size: int, G: int) -> np.ndarray:
    b = np.empty(G + 1, dtype=np.int32)
    rc = _load().mfo_bounds_nnz_width_balanced(_p(idx, np.int32), C.c_int64(idx.size), C.c_int64(size),
                                               C.c_int32(G), _p(b, np.int32))
    assert rc == 0
    return b


def partition(rows, cols, m, n, G_r, G_c, split=SPLIT_EQUAL_WIDTH, row_seed=0):
    """-> (perm int64[nnz], block_ptr int64[G_r*G_c+1], row_bounds, col_bounds).
    row_seed != 0: the rows of every block in the seeded order of row_rank instead of ascending."""
    nnz = rows.size
    perm = np.empty(nnz, dtype=np.int64)
    bp = np.empty(G_r * G_c + 1, dtype=np.int64)
    rb = np.empty(G_r + 1, dtype=np.int32)
    cb = np.empty(G_c + 1, dtype=np.int32)
    rc = _load().mfo_partition_seeded(_p(rows, np.int32), _p(cols, np.int32), C.c_int64(nnz), C.c_int64(m),
                                      C.c_int64(n), C.c_int32(G_r), C.c_int32(G_c), C.c_int32(split),
                                      C.c_uint64(row_seed),
                                      _p(perm, np.int64), _p(bp, np.int64), _p(rb, np.int32), _p(cb, np.int32))
    if rc != 0:
        raise ValueError(f"mfo_partition failed with {rc}")
    return perm, bp, rb, cb


def row_rank(u: int, first: int, width: int, row_seed: int, a: int) -> int:
    f = _load().mfo_row_rank
    f.restype = C.c_int64
    return int(f(C.c_int32(u), C.c_int32(first), C.c_int32(width), C.c_uint64(row_seed), C.c_int32(a)))


def blocks_independent(a1, b1, a2, b2) -> bool:
    return bool(_load().mfo_blocks_independent(C.c_int32(a1), C.c_int32(b1), C.c_int32(a2), C.c_int32(b2)))


def sgd_step(p: np.ndarray, q: np.ndarray, r: float, lr: float, lam: float, arith: int = ARITH_F64):
    """In-place step on one (p, q) pair of float64 vectors."""
    _load().mfo_sgd_step(_p(p, np.float64), _p(q, np.float64), C.c_int32(p.size), C.c_float(r),
                         C.c_float(lr), C.c_float(lam), C.c_int(arith))


def sgd_epoch(P, Qt, rows, cols, vals, perm, block_ptr, G_r, G_c, lr, lam, arith=ARITH_F64,
              block_order=None, visits=None):
    k = P.shape[1]
    rc = _load().mfo_sgd_epoch(_p(P, np.float64), _p(Qt, np.float64), C.c_int32(k), _p(rows, np.int32),
                               _p(cols, np.int32), _p(vals, np.float32), _p(perm, np.int64),
                               _p(block_ptr, np.int64), C.c_int32(G_r), C.c_int32(G_c), C.c_float(lr),
                               C.c_float(lam), C.c_int(arith),
                               _p(block_order, np.int32) if block_order is not None else None,
                               _p(visits, np.int32) if visits is not None else None)
    assert rc == 0


def sgd_epoch_omp(P, Qt, rows, cols, vals, perm, block_ptr, G_r, G_c, lr, lam, arith=ARITH_F64):
    k = P.shape[1]
    rc = _load().mfo_sgd_epoch_omp(_p(P, np.float64), _p(Qt, np.float64), C.c_int32(k), _p(rows, np.int32),
                                   _p(cols, np.int32), _p(vals, np.float32), _p(perm, np.int64),
                                   _p(block_ptr, np.int64), C.c_int32(G_r), C.c_int32(G_c), C.c_float(lr),
                                   C.c_float(lam), C.c_int(arith))
    assert rc == 0


def mix64(z: int) -> int:
    f = _load().mfo_mix64
    f.restype = C.c_uint64
    return int(f(C.c_uint64(z & 0xFFFFFFFFFFFFFFFF)))


def stratum_order(seed: int, epoch: int, G_c: int) -> np.ndarray:
    """Per-epoch permutation of the strata (order[t] = stratum visited at step t)."""
    out = np.empty(G_c, np.int32)
    _load().mfo_stratum_order(C.c_uint64(seed), C.c_uint64(epoch), C.c_int32(G_c), _p(out, np.int32))
    return out


def sgd_epoch_ordered(P, Qt, rows, cols, vals, perm, block_ptr, G_r, G_c, lr, lam, order, arith=ARITH_F64,
                      parallel=True, visits=None):
    k = P.shape[1]
    order = np.ascontiguousarray(order, np.int32)
    assert order.size == G_c
    rc = _load().mfo_sgd_epoch_ordered(_p(P, np.float64), _p(Qt, np.float64), C.c_int32(k), _p(rows, np.int32),
                                       _p(cols, np.int32), _p(vals, np.float32), _p(perm, np.int64),
                                       _p(block_ptr, np.int64), C.c_int32(G_r), C.c_int32(G_c), C.c_float(lr),
                                       C.c_float(lam), C.c_int(arith), _p(order, np.int32),
                                       C.c_int(1 if parallel else 0),
                                       _p(visits, np.int32) if visits is not None else None)
    assert rc == 0


def sgd_sweep(P, Qt, rows, cols, vals, lr, lam, arith=ARITH_F64):
    _load().mfo_sgd_sweep(_p(P, np.float64), _p(Qt, np.float64), C.c_int32(P.shape[1]), _p(rows, np.int32),
                          _p(cols, np.int32), _p(vals, np.float32), C.c_int64(rows.size), C.c_float(lr),
                          C.c_float(lam), C.c_int(arith))


def predict(P, Qt, u: int, v: int) -> float:
    return float(_load().mfo_predict(_p(P, np.float64), _p(Qt, np.float64), C.c_int32(P.shape[1]),
                                     C.c_int64(u), C.c_int64(v)))


def rating_loss(p, q, r: float, lamP: float, lamQ: float) -> float:
    return float(_load().mfo_rating_loss(_p(p, np.float64), _p(q, np.float64), C.c_int32(p.size),
                                         C.c_double(r), C.c_double(lamP), C.c_double(lamQ)))


def rmse(P, Qt, rows, cols, vals) -> float:
    return float(_load().mfo_rmse(_p(P, np.float64), _p(Qt, np.float64), C.c_int32(P.shape[1]),
                                  _p(rows, np.int32), _p(cols, np.int32), _p(vals, np.float32),
                                  C.c_int64(rows.size)))


def num_threads() -> int:
    return int(_load().mfo_num_threads())
