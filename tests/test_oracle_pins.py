"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage it pins.  A second group ("mutants") plants plausible
mistakes in a pure-Python copy of the step on the CPU and shows that the pins reject them,
so that the pins are known to be sensitive to a dropped term, a wrong sign, a transposed
operand or the sequential reading of Algorithm 1.
"""
import os

import numpy as np
import pytest

import oracle
import workloads


# --------------------------------------------------------------------------- helpers
def _read_golden(path):
    out = {}
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = vals
    return out


def _eq3_loss(p, q, r, lam_p, lam_q):
    """Eq. 3 typed independently of the oracle, in numpy float64."""
    return (r - p @ q) ** 2 + lam_p * (p @ p) + lam_q * (q @ q)


def _fd_grad(p, q, r, lam, h=1e-6):
    gp = np.zeros_like(p)
    gq = np.zeros_like(q)
    for f in range(p.size):
        d = np.zeros_like(p)
        d[f] = h
        gp[f] = (_eq3_loss(p + d, q, r, lam, lam) - _eq3_loss(p - d, q, r, lam, lam)) / (2 * h)
        gq[f] = (_eq3_loss(p, q + d, r, lam, lam) - _eq3_loss(p, q - d, r, lam, lam)) / (2 * h)
    return gp, gq


# --------------------------------------------------------------------------- Example 1
def test_example1_prediction_and_single_rating_rmse(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "example1_prediction.txt"))
    p = np.array([[float(x) for x in g["p"]]])
    q = np.array([[float(x) for x in g["q"]]])
    r = float(g["r"][0])
    est = float(g["estimate"][0])
    assert abs(oracle.predict(p, q, 0, 0) - est) < 5e-5          # printed to 4 decimals
    rm = oracle.rmse(p, q, np.zeros(1, np.int32), np.zeros(1, np.int32), np.array([r], np.float32))
    assert abs(rm - abs(r - est)) < 5e-5


# --------------------------------------------------------------------------- Example 2
def test_example2_independence_predicate(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "example2_blocks.txt"))
    ind = [tuple(int(x) for x in tok.split(",")) for tok in g["independent"]]
    for i in range(len(ind)):
        for j in range(len(ind)):
            if i != j:
                assert oracle.blocks_independent(*ind[i], *ind[j])
    (a1, b1), (a2, b2) = [tuple(int(x) for x in tok.split(",")) for tok in g["conflict"]]
    assert not oracle.blocks_independent(a1, b1, a2, b2)
    assert not oracle.blocks_independent(1, 2, 3, 2)            # same block column conflicts too


def test_every_stratum_is_a_set_of_independent_blocks():
    # the stratum rule s = (b - a) mod G_c, read back from the partition itself
    rng = np.random.default_rng(5)
    m, n, nnz = 50, 70, 3000
    rows = rng.integers(0, m, nnz).astype(np.int32)
    cols = rng.integers(0, n, nnz).astype(np.int32)
    for (gr, gc) in [(4, 4), (3, 7), (1, 5), (5, 5)]:
        perm, bp, rb, cb = oracle.partition(rows, cols, m, n, gr, gc)
        for s in range(gc):
            blocks = []
            for a in range(gr):
                L = s * gr + a
                idx = perm[bp[L]:bp[L + 1]]
                if idx.size == 0:
                    continue
                ra = np.searchsorted(rb, rows[idx], side="right") - 1
                ca = np.searchsorted(cb, cols[idx], side="right") - 1
                assert (ra == a).all() and (ca == ca[0]).all()
                blocks.append((a, int(ca[0])))
            for i in range(len(blocks)):
                for j in range(i + 1, len(blocks)):
                    assert oracle.blocks_independent(*blocks[i], *blocks[j])


# --------------------------------------------------------------------------- the step
@pytest.mark.parametrize("k", [1, 2, 7, 32])
def test_step_is_minus_half_gamma_times_gradient_of_eq3(k):
    # Algorithm 1 vs Eq. 4-6: step = -(gamma/2) * grad, both gradients at the same point
    rng = np.random.default_rng(100 + k)
    for _ in range(5):
        p = rng.normal(0, 0.5, k)
        q = rng.normal(0, 0.5, k)
        r = float(np.float32(rng.uniform(1, 5)))
        g = float(np.float32(0.1))
        lam = float(np.float32(0.3))
        gp, gq = _fd_grad(p, q, r, lam)
        p1, q1 = p.copy(), q.copy()
        oracle.sgd_step(p1, q1, r, g, lam, oracle.ARITH_F64)
        np.testing.assert_allclose(p1 - p, -0.5 * g * gp, rtol=0, atol=2e-9)
        np.testing.assert_allclose(q1 - q, -0.5 * g * gq, rtol=0, atol=2e-9)


def test_hand_case_k1_simultaneous_reading():
    # k=1, lambda=0, r=1, p=q=0.5, gamma=0.1: e = 0.75, p' = q' = 0.5 + 0.1*0.75*0.5 = 0.5375.
    # (Updating q with the already updated p would give 0.5403125 instead.)
    p = np.array([0.5])
    q = np.array([0.5])
    oracle.sgd_step(p, q, 1.0, float(np.float32(0.1)), 0.0, oracle.ARITH_F64)
    g = float(np.float32(0.1))
    assert abs(p[0] - (0.5 + g * 0.75 * 0.5)) < 1e-15
    assert abs(q[0] - (0.5 + g * 0.75 * 0.5)) < 1e-15
    assert abs(q[0] - 0.5403125) > 1e-3


def test_fixed_points():
    rng = np.random.default_rng(3)
    p = rng.uniform(0.1, 1, 8)
    q = rng.uniform(0.1, 1, 8)
    r = float(np.float32(p @ q))
    # make r exactly representable and equal to p.q: rescale p
    p *= r / (p @ q)
    p0, q0 = p.copy(), q.copy()
    oracle.sgd_step(p, q, r, 0.125, 0.0, oracle.ARITH_F64)       # e = 0, lambda = 0: nothing moves
    np.testing.assert_allclose(p, p0, atol=1e-15)
    np.testing.assert_allclose(q, q0, atol=1e-15)
    oracle.sgd_step(p, q, r, 0.125, 0.5, oracle.ARITH_F64)       # e = 0: pure shrink by (1 - g*lambda)
    np.testing.assert_allclose(p, p0 * (1 - 0.125 * 0.5), atol=1e-14)
    np.testing.assert_allclose(q, q0 * (1 - 0.125 * 0.5), atol=1e-14)


def test_small_step_lowers_the_rating_loss():
    rng = np.random.default_rng(4)
    for _ in range(20):
        p = rng.normal(0, 0.5, 16)
        q = rng.normal(0, 0.5, 16)
        r = float(np.float32(rng.uniform(1, 5)))
        lam = float(np.float32(0.05))
        before = oracle.rating_loss(p, q, r, lam, lam)
        assert abs(before - _eq3_loss(p, q, r, lam, lam)) < 1e-12
        oracle.sgd_step(p, q, r, float(np.float32(0.01)), lam, oracle.ARITH_F64)
        assert oracle.rating_loss(p, q, r, lam, lam) < before


def test_rows_and_columns_without_ratings_never_change():
    m, n, k = 6, 5, 4
    rows = np.array([0, 0, 2], np.int32)
    cols = np.array([1, 3, 1], np.int32)
    vals = np.array([3, 4, 5], np.float32)
    P = np.full((m, k), 0.3)
    Q = np.full((n, k), 0.2)
    oracle.sgd_sweep(P, Q, rows, cols, vals, 0.05, 0.05)
    assert (P[[1, 3, 4, 5]] == 0.3).all() and (Q[[0, 2, 4]] == 0.2).all()
    assert (P[[0, 2]] != 0.3).all() and (Q[[1, 3]] != 0.2).all()


# --------------------------------------------------------------------------- pure-Python brute force of the epoch
def _py_epoch(P, Q, rows, cols, vals, order, g, lam):
    g = float(np.float32(g))
    lam = float(np.float32(lam))
    for t in order:
        u, v = rows[t], cols[t]
        p, q = P[u].copy(), Q[v].copy()
        e = float(vals[t]) - p @ q
        P[u] = p + g * (e * q - lam * p)
        Q[v] = q + g * (e * p - lam * q)


def test_epoch_equals_python_loop_in_partition_order():
    rng = np.random.default_rng(11)
    m, n, k, nnz = 40, 30, 5, 600
    rows = rng.integers(0, m, nnz).astype(np.int32)
    cols = rng.integers(0, n, nnz).astype(np.int32)
    vals = rng.uniform(1, 5, nnz).astype(np.float32)
    perm, bp, _, _ = oracle.partition(rows, cols, m, n, 3, 4)
    P = rng.uniform(0, 0.3, (m, k))
    Q = rng.uniform(0, 0.3, (n, k))
    P2, Q2 = P.copy(), Q.copy()
    oracle.sgd_epoch(P, Q, rows, cols, vals, perm, bp, 3, 4, 0.05, 0.02)
    _py_epoch(P2, Q2, rows, cols, vals, perm, 0.05, 0.02)
    # same order, same formula: only the summation order of numpy's dot may differ
    np.testing.assert_allclose(P, P2, atol=1e-13)
    np.testing.assert_allclose(Q, Q2, atol=1e-13)


# --------------------------------------------------------------------------- exactly once
@pytest.mark.parametrize("split", [oracle.SPLIT_EQUAL_WIDTH, oracle.SPLIT_NNZ_BALANCED])
def test_every_rating_visited_exactly_once_and_partition_covers_all(split):
    ds = workloads.generate(workloads.scaled(workloads.CONFIGS["medium"], 0.002, k=8))
    m, n = ds.cfg.m, ds.cfg.n
    perm, bp, rb, cb = oracle.partition(ds.rows, ds.cols, m, n, 5, 9, split)
    nnz = ds.rows.size
    assert bp[0] == 0 and bp[-1] == nnz and (np.diff(bp) >= 0).all()
    assert np.array_equal(np.sort(perm), np.arange(nnz))
    P = np.full((m, 8), 0.1)
    Q = np.full((n, 8), 0.1)
    visits = np.zeros(nnz, np.int32)
    oracle.sgd_epoch(P, Q, ds.rows, ds.cols, ds.vals, perm, bp, 5, 9, 0.01, 0.05, visits=visits)
    assert (visits == 1).all()


# --------------------------------------------------------------------------- partition brute force
def _py_partition(rows, cols, m, n, gr, gc, rb, cb):
    keys = []
    for t, (u, v) in enumerate(zip(rows.tolist(), cols.tolist())):
        a = max(i for i in range(gr) if rb[i] <= u)
        b = max(i for i in range(gc) if cb[i] <= v)
        assert rb[a] <= u < rb[a + 1] and cb[b] <= v < cb[b + 1]
        s = (b - a) % gc
        keys.append((s * gr + a, u, v, t))
    keys.sort()
    perm = np.array([kk[3] for kk in keys], np.int64)
    cnt = np.zeros(gr * gc + 1, np.int64)
    for kk in keys:
        cnt[kk[0] + 1] += 1
    return perm, np.cumsum(cnt)


@pytest.mark.parametrize("gr,gc", [(1, 1), (2, 3), (4, 4), (7, 8)])
def test_partition_equal_width_matches_brute_force(gr, gc):
    rng = np.random.default_rng(gr * 10 + gc)
    m, n, nnz = 37, 29, 500
    rows = rng.integers(0, m, nnz).astype(np.int32)
    cols = rng.integers(0, n, nnz).astype(np.int32)
    rows[10:20] = rows[0]
    cols[10:20] = cols[0]                                      # duplicate (u, v) entries are legal
    perm, bp, rb, cb = oracle.partition(rows, cols, m, n, gr, gc, oracle.SPLIT_EQUAL_WIDTH)
    # uniform division, closed form: strip of id x is floor(x*G/size)
    assert np.array_equal(rb, [-(-a * m // gr) for a in range(gr + 1)])
    assert np.array_equal(cb, [-(-b * n // gc) for b in range(gc + 1)])
    for x in range(m):
        assert rb[x * gr // m] <= x < rb[x * gr // m + 1]
    perm2, bp2 = _py_partition(rows, cols, m, n, gr, gc, rb, cb)
    assert np.array_equal(perm, perm2) and np.array_equal(bp, bp2)


def test_partition_nnz_balanced_bounds_and_brute_force():
    rng = np.random.default_rng(77)
    m, n, nnz = 60, 45, 2000
    w = 1.0 / np.arange(1, m + 1)
    rows = rng.choice(m, nnz, p=w / w.sum()).astype(np.int32)
    cols = rng.integers(0, n, nnz).astype(np.int32)
    gr, gc = 4, 6
    perm, bp, rb, cb = oracle.partition(rows, cols, m, n, gr, gc, oracle.SPLIT_NNZ_BALANCED)
    deg = np.bincount(rows, minlength=m)
    S = np.concatenate([[0], np.cumsum(deg)])
    for a in range(1, gr):
        target = -(-a * nnz // gr)
        assert S[rb[a]] >= target and (rb[a] == 0 or S[rb[a] - 1] < target)
    assert rb[0] == 0 and rb[gr] == m and (np.diff(rb) >= 0).all()
    # no strip can exceed its fair share by more than the heaviest single row
    per_strip = np.add.reduceat(deg, rb[:-1][np.diff(rb) > 0])
    assert per_strip.max() <= nnz / gr + deg.max()
    perm2, bp2 = _py_partition(rows, cols, m, n, gr, gc, rb, cb)
    assert np.array_equal(perm, perm2) and np.array_equal(bp, bp2)


def test_partition_nnz_width_balanced_bounds_and_brute_force():
    rng = np.random.default_rng(78)
    m, n, nnz = 64, 50, 3000
    w = 1.0 / np.arange(1, n + 1) ** 1.3
    rows = rng.integers(0, m, nnz).astype(np.int32)
    cols = rng.choice(n, nnz, p=w / w.sum()).astype(np.int32)
    gr, gc = 4, 10
    perm, bp, rb, cb = oracle.partition(rows, cols, m, n, gr, gc, oracle.SPLIT_NNZ_WIDTH_BALANCED)
    for idx, size, G, bounds in ((rows, m, gr, rb), (cols, n, gc, cb)):
        deg = np.bincount(idx, minlength=size)
        S = np.concatenate([[0], np.cumsum(deg)])
        W = [int(S[x]) * size + x * nnz for x in range(size + 1)]        # python integers: exact
        assert W[size] == 2 * nnz * size
        for a in range(1, G):
            target = -(-a * W[size] // G)
            assert W[bounds[a]] >= target and (bounds[a] == 0 or W[bounds[a] - 1] < target)
        assert bounds[0] == 0 and bounds[G] == size and (np.diff(bounds) >= 0).all()
        # a strip is bounded in width and in ratings: twice the fair share plus one id
        widths = np.diff(bounds)
        per = np.array([deg[bounds[a]:bounds[a + 1]].sum() for a in range(G)])
        assert widths.max() <= 2 * size / G + 1
        assert per.max() <= 2 * nnz / G + deg.max()
    perm2, bp2 = _py_partition(rows, cols, m, n, gr, gc, rb, cb)
    assert np.array_equal(perm, perm2) and np.array_equal(bp, bp2)
    # without ratings the rule degenerates to the uniform division of the axis
    z = np.zeros(0, np.int32)
    assert np.array_equal(oracle.bounds_nnz_width_balanced(z, 20, 4), [0, 5, 10, 15, 20])


def test_partition_rejects_bad_arguments():
    rows = np.array([0, 1], np.int32)
    cols = np.array([0, 5], np.int32)
    with pytest.raises(ValueError):
        oracle.partition(rows, cols, 2, 5, 1, 1)               # column 5 out of range
    with pytest.raises(ValueError):
        oracle.partition(rows, cols, 2, 6, 2, 1)               # G_r > G_c


# --------------------------------------------------------------------------- independence => order inside a stratum is immaterial
def test_block_order_inside_strata_and_openmp_are_bit_identical():
    ds = workloads.generate(workloads.scaled(workloads.CONFIGS["medium"], 0.003, k=16))
    m, n, k = ds.cfg.m, ds.cfg.n, 16
    gr, gc = 6, 8
    perm, bp, _, _ = oracle.partition(ds.rows, ds.cols, m, n, gr, gc, oracle.SPLIT_NNZ_BALANCED)
    P0 = oracle.init_factors(m * k, 1, 0, 0.1).reshape(m, k)
    Q0 = oracle.init_factors(n * k, 1, 1, 0.1).reshape(n, k)
    rng = np.random.default_rng(0)
    order = np.concatenate([rng.permutation(gr) for _ in range(gc)]).astype(np.int32)
    for arith in (oracle.ARITH_F64, oracle.ARITH_F32, oracle.ARITH_F16):
        A = (P0.copy(), Q0.copy())
        B = (P0.copy(), Q0.copy())
        Cc = (P0.copy(), Q0.copy())
        oracle.sgd_epoch(*A, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, 0.01, 0.05, arith)
        oracle.sgd_epoch(*B, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, 0.01, 0.05, arith, block_order=order)
        oracle.sgd_epoch_omp(*Cc, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, 0.01, 0.05, arith)
        for X, Y in ((A, B), (A, Cc)):
            assert np.array_equal(X[0], Y[0]) and np.array_equal(X[1], Y[1])
        assert not np.array_equal(A[0], P0)


# --------------------------------------------------------------------------- randomised stratum order
def test_mixer_reproduces_the_published_splitmix64_stream(golden_dir):
    """The oracle's mixer is the SplitMix64 output function: fed with seed + i * increment it must
    give that generator's published first outputs for seed 1234567 (fixture with its source)."""
    g = _read_golden(os.path.join(golden_dir, "splitmix64_seed1234567.txt"))
    want = [int(g[f"x{i}"][0]) for i in range(5)]
    golden_ratio = 0x9E3779B97F4A7C15
    got = [oracle.mix64(1234567 + i * golden_ratio) for i in range(len(want))]
    assert got == want


def test_stratum_order_is_a_reproducible_permutation_sorted_by_its_keys():
    for gc in (1, 2, 7, 64, 333):
        o = oracle.stratum_order(5, 3, gc)
        assert sorted(o.tolist()) == list(range(gc))
        assert np.array_equal(o, oracle.stratum_order(5, 3, gc))
        # independent restatement: argsort of the keys, ties by index (keys via the pinned mixer)
        base = oracle.mix64(5 ^ ((3 * 0xD1B54A32D192ED03) & 0xFFFFFFFFFFFFFFFF))
        keys = [oracle.mix64((base + s) & 0xFFFFFFFFFFFFFFFF) for s in range(gc)]
        assert o.tolist() == sorted(range(gc), key=lambda s: (keys[s], s))
    a, b, c = oracle.stratum_order(5, 0, 64), oracle.stratum_order(5, 1, 64), oracle.stratum_order(6, 0, 64)
    assert not np.array_equal(a, b) and not np.array_equal(a, c)
    # no position is favoured: over many epochs stratum 0 lands everywhere about equally often
    gc = 8
    hits = np.zeros(gc)
    for e in range(4000):
        hits[oracle.stratum_order(11, e, gc).tolist().index(0)] += 1
    assert hits.min() > 400 and hits.max() < 600          # mean 500, sd 21


def test_ordered_epoch_is_the_blocks_swept_in_that_order_exactly_once():
    ds = workloads.generate(workloads.scaled(workloads.CONFIGS["medium"], 0.003, k=16))
    m, n, k = ds.cfg.m, ds.cfg.n, 16
    gr, gc = 5, 9
    perm, bp, _, _ = oracle.partition(ds.rows, ds.cols, m, n, gr, gc, oracle.SPLIT_NNZ_BALANCED)
    P0 = oracle.init_factors(m * k, 1, 0, 0.1).reshape(m, k)
    Q0 = oracle.init_factors(n * k, 1, 1, 0.1).reshape(n, k)
    order = oracle.stratum_order(9, 2, gc)
    assert not np.array_equal(order, np.arange(gc))
    for arith in (oracle.ARITH_F64, oracle.ARITH_F16):
        ident = (P0.copy(), Q0.copy())
        plain = (P0.copy(), Q0.copy())
        oracle.sgd_epoch_ordered(*ident, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, 0.01, 0.05, np.arange(gc), arith)
        oracle.sgd_epoch(*plain, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, 0.01, 0.05, arith)
        assert np.array_equal(ident[0], plain[0]) and np.array_equal(ident[1], plain[1])
        # the given order = plain sweeps (another entry point) over the blocks' ratings, stratum after stratum
        A = (P0.copy(), Q0.copy())
        B = (P0.copy(), Q0.copy())
        Cc = (P0.copy(), Q0.copy())
        visits = np.zeros(ds.rows.size, np.int32)
        oracle.sgd_epoch_ordered(*A, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, 0.01, 0.05, order, arith, parallel=False,
                                 visits=visits)
        oracle.sgd_epoch_ordered(*Cc, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, 0.01, 0.05, order, arith, parallel=True)
        for s in order:
            sel = perm[bp[s * gr]:bp[(s + 1) * gr]]
            oracle.sgd_sweep(*B, ds.rows[sel], ds.cols[sel], ds.vals[sel], 0.01, 0.05, arith)
        assert np.array_equal(visits, np.ones_like(visits))
        assert np.array_equal(A[0], B[0]) and np.array_equal(A[1], B[1])
        assert np.array_equal(A[0], Cc[0]) and np.array_equal(A[1], Cc[1])
        assert not np.array_equal(A[1], plain[1])          # the order does matter across strata


def test_seeded_row_order_is_a_permutation_of_every_strip_and_matches_brute_force():
    m, n, gr, gc, seed = 211, 97, 4, 6, 12345
    rng = np.random.default_rng(5)
    rows = rng.integers(0, m, 3000).astype(np.int32)
    cols = rng.integers(0, n, 3000).astype(np.int32)
    perm, bp, rb, cb = oracle.partition(rows, cols, m, n, gr, gc, oracle.SPLIT_NNZ_BALANCED, row_seed=seed)
    plain = oracle.partition(rows, cols, m, n, gr, gc, oracle.SPLIT_NNZ_BALANCED)
    assert np.array_equal(bp, plain[1]) and np.array_equal(rb, plain[2]) and np.array_equal(cb, plain[3])
    assert not np.array_equal(perm, plain[0])
    assert np.array_equal(oracle.partition(rows, cols, m, n, gr, gc, oracle.SPLIT_NNZ_BALANCED, row_seed=0)[0], plain[0])
    # the rank is the stated affine map (restated with Python integers and the pinned mixer) and a bijection
    rank = {}
    for a in range(gr):
        first, width = int(rb[a]), int(rb[a + 1] - rb[a])
        offset = oracle.mix64(seed + a) % width
        got = [oracle.row_rank(u, first, width, seed, a) for u in range(first, first + width)]
        assert got == [((u - first) * 2147483647 + offset) % width for u in range(first, first + width)]
        assert sorted(got) == list(range(width))
        for u, r in zip(range(first, first + width), got):
            rank[u] = r
    # brute force: block id, then rank of the row, column, original position
    strip = lambda bounds, x: int(np.searchsorted(bounds, x, side="right") - 1)
    def key(t):
        a, b = strip(rb, rows[t]), strip(cb, cols[t])
        return (((b - a) % gc) * gr + a, rank[int(rows[t])], int(cols[t]), t)
    assert perm.tolist() == sorted(range(rows.size), key=key)
    # all ratings of a row of a block stay together
    for L in range(gr * gc):
        blk_rows = rows[perm[bp[L]:bp[L + 1]]]
        changes = np.flatnonzero(np.diff(blk_rows)) + 1
        runs = np.split(blk_rows, changes)
        assert len({int(r[0]) for r in runs}) == len(runs)


# --------------------------------------------------------------------------- convergence on noiseless planted data
def test_noiseless_planted_low_rank_reaches_near_zero_rmse():
    m, n, rank = 150, 120, 3
    u, v, r = workloads.planted_noiseless(m, n, 9000, rank, seed=42)
    k = 8
    P = oracle.init_factors(m * k, 7, 0, 0.5).reshape(m, k)
    Q = oracle.init_factors(n * k, 7, 1, 0.5).reshape(n, k)
    perm, bp, _, _ = oracle.partition(u, v, m, n, 4, 4)
    first = oracle.rmse(P, Q, u, v, r)
    last = first
    hist = []
    for ep in range(400):
        oracle.sgd_epoch(P, Q, u, v, r, perm, bp, 4, 4, 0.03, 0.0)
        if ep % 20 == 19:
            hist.append(oracle.rmse(P, Q, u, v, r))
    assert all(b < a for a, b in zip([first] + hist, hist)), hist
    last = hist[-1]
    assert last < 2e-3 and last < first * 1e-2, (first, last)


# --------------------------------------------------------------------------- RMSE vs numpy
def test_rmse_reduces_to_numpy():
    rng = np.random.default_rng(9)
    m, n, k, cnt = 30, 20, 12, 500
    P = rng.normal(0, 1, (m, k))
    Q = rng.normal(0, 1, (n, k))
    rows = rng.integers(0, m, cnt).astype(np.int32)
    cols = rng.integers(0, n, cnt).astype(np.int32)
    vals = rng.uniform(1, 5, cnt).astype(np.float32)
    want = np.sqrt(np.mean((vals.astype(np.float64) - np.einsum("ik,ik->i", P[rows], Q[cols])) ** 2))
    assert abs(oracle.rmse(P, Q, rows, cols, vals) - want) < 1e-12


# --------------------------------------------------------------------------- binary16 rounding vs numpy
def test_round_f16_matches_numpy_binary16():
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        rng.normal(0, 1, 20000), rng.normal(0, 1e-5, 5000), rng.normal(0, 3e4, 2000),
        np.array([0.0, 65504.0, 65519.9, 65520.0, 7e4, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25, 2.0 ** -14,
                  1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -30, -0.1, -1e-7]),
        # every binary16 midpoint in [0.25, 0.5): ties must go to even
        (np.arange(0x3400, 0x3800, dtype=np.uint16).view(np.float16).astype(np.float64) + 2.0 ** -13),
    ])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).astype(np.float64)
    got = np.array([oracle.round_f16(float(x)) for x in xs])
    assert np.array_equal(got, want)


def test_f32_and_f16_arithmetic_stay_on_their_grids_and_close_to_f64():
    rng = np.random.default_rng(2)
    k = 32
    p = rng.uniform(0, 0.5, k).astype(np.float32).astype(np.float64)
    q = rng.uniform(0, 0.5, k).astype(np.float32).astype(np.float64)
    ref = (p.copy(), q.copy())
    oracle.sgd_step(*ref, 4.0, 0.01, 0.05, oracle.ARITH_F64)
    a = (p.copy(), q.copy())
    oracle.sgd_step(*a, 4.0, 0.01, 0.05, oracle.ARITH_F32)
    assert np.array_equal(a[0], a[0].astype(np.float32).astype(np.float64))
    np.testing.assert_allclose(a[0], ref[0], atol=1e-7)
    np.testing.assert_allclose(a[1], ref[1], atol=1e-7)
    ph = p.astype(np.float16).astype(np.float64)
    qh = q.astype(np.float16).astype(np.float64)
    refh = (ph.copy(), qh.copy())
    oracle.sgd_step(*refh, 4.0, 0.01, 0.05, oracle.ARITH_F64)
    b = (ph.copy(), qh.copy())
    oracle.sgd_step(*b, 4.0, 0.01, 0.05, oracle.ARITH_F16)
    assert np.array_equal(b[0], b[0].astype(np.float16).astype(np.float64))
    # result = binary16 rounding of the fp32 step, i.e. within half a binary16 ulp (+fp32 noise)
    np.testing.assert_allclose(b[0], refh[0], atol=2.0 ** -12 + 1e-6)
    np.testing.assert_allclose(b[1], refh[1], atol=2.0 ** -12 + 1e-6)


# --------------------------------------------------------------------------- initialiser
def test_init_is_uniform_on_the_24_bit_grid_and_streams_differ():
    x = oracle.init_factors(200000, 123, 0, 0.1)
    y = oracle.init_factors(200000, 123, 1, 0.1)
    z = oracle.init_factors(200000, 124, 0, 0.1)
    assert x.min() >= 0 and x.max() < 0.1
    assert abs(x.mean() - 0.05) < 3e-4 and abs(x.var() - 0.01 / 12) < 2e-5
    assert not np.array_equal(x, y) and not np.array_equal(x, z)
    assert np.array_equal(x, oracle.init_factors(200000, 123, 0, 0.1))
    assert np.array_equal(x[:1000], oracle.init_factors(1000, 123, 0, 0.1))     # counter-based
    u = oracle.init_factors(1000, 5, 0, 1.0)
    assert np.array_equal(u * 2 ** 24, np.round(u * 2 ** 24))                   # top 24 bits * 2^-24
    h = oracle.init_factors(1000, 5, 0, 0.1, oracle.ARITH_F16)
    assert np.array_equal(h, h.astype(np.float16).astype(np.float64))


# --------------------------------------------------------------------------- mutants: the pins must reject plausible mistakes
def _mutant_step(kind, p, q, r, g, lam):
    e = r - p @ q
    if kind == "sequential":            # q updated from the already updated p
        pn = p + g * (e * q - lam * p)
        return pn, q + g * (e * pn - lam * q)
    if kind == "no_reg":                # dropped regularisation term
        return p + g * e * q, q + g * e * p
    if kind == "wrong_sign":            # regulariser added instead of subtracted
        return p + g * (e * q + lam * p), q + g * (e * p + lam * q)
    if kind == "factor2":               # literal Eq. 6 with the factor 2 of Eq. 4-5
        return p + 2 * g * (e * q - lam * p), q + 2 * g * (e * p - lam * q)
    if kind == "swapped":               # p moved along p, q along q (transposed operands)
        return p + g * (e * p - lam * p), q + g * (e * q - lam * q)
    if kind == "err_sign":              # e = p.q - r
        return p + g * (-e * q - lam * p), q + g * (-e * p - lam * q)
    raise KeyError(kind)


@pytest.mark.parametrize("kind", ["sequential", "no_reg", "wrong_sign", "factor2", "swapped", "err_sign"])
def test_finite_difference_pin_rejects_planted_mistakes(kind):
    rng = np.random.default_rng(8)
    p = rng.normal(0, 0.5, 6)
    q = rng.normal(0, 0.5, 6)
    r, g, lam = 4.0, 0.1, 0.3
    gp, gq = _fd_grad(p, q, r, lam)
    pn, qn = _mutant_step(kind, p, q, r, g, lam)
    bad = max(np.abs(pn - p + 0.5 * g * gp).max(), np.abs(qn - q + 0.5 * g * gq).max())
    assert bad > 1e-4            # the FD pin's tolerance is 2e-9: each mutant fails it by far
