"""Helpers shared by the tests: cached synthetic data sets and oracle drivers."""
import os
import re

import numpy as np

import oracle
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def dataset(name: str, factor: float = 1.0, k=None) -> workloads.Dataset:
    """Generate (or take from the cache) one synthetic configuration."""
    return workloads.load(name, factor, k)


def oracle_init(m, n, k, seed, scale, arith=oracle.ARITH_F64):
    P = oracle.init_factors(m * k, seed, 0, scale, arith).reshape(m, k)
    Q = oracle.init_factors(n * k, seed, 1, scale, arith).reshape(n, k)
    return P, Q


def oracle_train(ds, gr, gc, split, epochs, seed=1, scale=0.1, arith=oracle.ARITH_F64, parallel=True, k=None):
    """Oracle factors after `epochs` epochs from the counter-based initial factors."""
    cfg = ds.cfg
    k = k or cfg.k
    perm, bp, rb, cb = oracle.partition(ds.rows, ds.cols, cfg.m, cfg.n, gr, gc, split)
    P, Q = oracle_init(cfg.m, cfg.n, k, seed, scale, arith)
    run = oracle.sgd_epoch_omp if parallel else oracle.sgd_epoch
    for _ in range(epochs):
        run(P, Q, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, cfg.lr, cfg.lam, arith)
    return P, Q, (perm, bp, rb, cb)


def declared_functions(header_path):
    """Names of the functions a C header declares (int / const char* returning)."""
    text = open(header_path).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mf_[a-z_0-9]+)\s*\(", text)))
