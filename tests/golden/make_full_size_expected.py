"""Writes tests/golden/full_<config>.txt and full_<config>_groupsums.npy: what the CPU oracle gives on
a FULL-SIZE configuration, for the GPU parity test of that size (the oracle needs minutes to an hour
there, far more than a GPU test may take, so its results are stored; this script calls only oracle/
and the input generators).

    python tests/golden/make_full_size_expected.py <config> <grid_r> <grid_c> <split> <init_scale> <epochs>

Stored: the held-out RMSE after every epoch (canonical order, the configuration's storage
arithmetic: F64 for fp32 storage, F16 for binary16 storage); after the FIRST epoch the full rows of
P and Qt at a seeded sample of row / column indices (C99 hex floats, exact) and, so that every row
of both factors is covered, the sum of the elements of every group of 64 consecutive rows of P and
of Qt (float64, P's groups first).
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workloads  # noqa: E402
from tests.util import dataset, oracle_init  # noqa: E402

SAMPLE = 48          # sampled rows of P and of Qt
GROUP = 64           # rows per checksum group


def sample_ids(ds, axis_size, idx, seed):
    """Half of the sample from the ids with most ratings, half uniform."""
    deg = np.bincount(idx, minlength=axis_size)
    top = np.argsort(-deg, kind="stable")[:SAMPLE // 2]
    rng = np.random.Generator(np.random.Philox(seed))
    rest = rng.choice(axis_size, size=SAMPLE - top.size, replace=False)
    return np.unique(np.concatenate([top, rest])).astype(np.int64)


def group_sums(X):
    """Sum of all elements of every GROUP consecutive rows (the last group may be short)."""
    row = X.sum(axis=1)
    pad = (-row.size) % GROUP
    return np.concatenate([row, np.zeros(pad)]).reshape(-1, GROUP).sum(axis=1)


def main():
    name, gr, gc, split = sys.argv[1], int(sys.argv[2]), int(sys.argv[3]), int(sys.argv[4])
    scale, epochs = float(sys.argv[5]), int(sys.argv[6])
    t0 = time.time()
    ds = dataset(name, 1.0)
    cfg = ds.cfg
    arith = oracle.ARITH_F16 if cfg.storage == "f16" else oracle.ARITH_F64
    print(f"[{time.time() - t0:7.1f}s] data ready: {ds.rows.size} ratings", flush=True)
    perm, bp, _, _ = oracle.partition(ds.rows, ds.cols, cfg.m, cfg.n, gr, gc, split)
    print(f"[{time.time() - t0:7.1f}s] partition done", flush=True)
    P, Q = oracle_init(cfg.m, cfg.n, cfg.k, 1, scale, arith)
    rows_p = sample_ids(ds, cfg.m, ds.rows, 1)
    rows_q = sample_ids(ds, cfg.n, ds.cols, 2)
    lines = [f"# Oracle results on the full-size configuration '{name}' (written by make_full_size_expected.py;",
             "# inputs: workloads.generate, seed of the configuration; factors: init seed 1).",
             f"config {name}", f"recipe {workloads.RECIPE}", f"grid {gr} {gc}", f"split {split}",
             f"init_scale {scale!r}", f"arith {arith}", f"lr {cfg.lr!r}", f"lambda {cfg.lam!r}",
             f"nnz_train {ds.rows.size}", f"group {GROUP}"]
    head = len(lines)
    rmse = []
    for e in range(epochs):
        oracle.sgd_epoch_omp(P, Q, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, cfg.lr, cfg.lam, arith)
        rmse.append(oracle.rmse(P, Q, ds.test_rows, ds.test_cols, ds.test_vals))
        print(f"[{time.time() - t0:7.1f}s] epoch {e + 1}: held-out rmse {rmse[-1]:.6f}", flush=True)
        if e == 0:
            for tag, X, ids in (("P", P, rows_p), ("Q", Q, rows_q)):
                for i in ids:
                    lines.append(f"{tag}{int(i)} " + " ".join(float(x).hex() for x in X[i]))
            np.save(os.path.join(ROOT, "tests", "golden", f"full_{name}_groupsums.npy"),
                    np.concatenate([group_sums(P), group_sums(Q)]))
    lines.insert(head, "rmse " + " ".join(repr(float(x)) for x in rmse))
    out = os.path.join(ROOT, "tests", "golden", f"full_{name}.txt")
    with open(out, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print("wrote", out, flush=True)


if __name__ == "__main__":
    main()
