"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.

Bars (written out here):
  * integer work (partition, permutation, block pointers, bounds, initial factors' bit patterns):
    bit-exact;
  * deterministic mode, fp32 storage: max |dP|, |dQ| <= 1e-4 against the fp64 oracle after one
    epoch; final held-out RMSE within 1e-3 (absolute) after the configuration's epochs;
  * deterministic mode, binary16 storage: the rounding to binary16 is a decision taken from an
    fp32 value that both sides define operation by operation (dot product summed in double,
    then the same fp32 operations), so the result is the same binary16 value: the bar is
    bit-equality, allowing 1e-5 of the elements to differ (a double-precision dot product
    that rounds differently to fp32 on the two sides, probability about 1e-9 per step);
  * Hogwild mode: final held-out RMSE within 0.5 % (relative) of the oracle's;
  * RMSE kernel: relative 1e-9 against the fp64 oracle.
"""
import os

import numpy as np
import pytest

import oracle
from tests.util import dataset, oracle_init, oracle_train

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu



@pytest.fixture(scope="module")
def mfmod():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2006_15980_amd as mf
    mf.binding.lib()          # fails loudly when the HIP library is not built
    return mf


def _arith(storage):
    return oracle.ARITH_F16 if storage == "f16" else oracle.ARITH_F64


def _make(mf, ds, k, storage, gr, gc, split, seed=1, scale=0.1, options=None):
    model = mf.MatrixFactorization(ds.cfg.m, ds.cfg.n, k, storage, seed=seed, scale=scale, options=options)
    model.load_blocks(ds.rows, ds.cols, ds.vals, gr, gc, split)
    return model


def _one_heavy_block_row(mf, options):
    """A model on a 64 x 64 grid of equal-width strips in which block row 5 holds a hundred times
    the ratings of any other: the block row before it finishes each step long before block row 5
    has released the strip it needs, whatever the timing of the launch."""
    rng = np.random.default_rng(20061642)
    m, n, per_strip = 64 * 16, 640, 16
    light = rng.integers(0, m, 64 * 1000)
    heavy = rng.integers(5 * per_strip, 6 * per_strip, 100000)
    rows = np.concatenate([light, heavy]).astype(np.int32)
    cols = rng.integers(0, n, rows.size).astype(np.int32)
    vals = rng.uniform(1.0, 5.0, rows.size).astype(np.float32)
    model = mf.MatrixFactorization(m, n, 128, "f32", seed=1, scale=0.1, options=options)
    model.load_blocks(rows, cols, vals, 64, 64, 0)
    return model, rows, cols, vals


# ------------------------------------------------------------------------------- integer work
@pytest.mark.parametrize("storage", ["f32", "f16"])
def test_init_factors_bit_exact(mfmod, storage):
    m, n, k = 1000, 777, 64
    model = mfmod.MatrixFactorization(m, n, k, storage, seed=99, scale=0.1)
    P, Q = model.get_factors()
    Po, Qo = oracle_init(m, n, k, 99, 0.1, oracle.ARITH_F16 if storage == "f16" else oracle.ARITH_F32)
    assert np.array_equal(P, Po) and np.array_equal(Q, Qo)
    model.close()


@pytest.mark.parametrize("split", [0, 1])
def test_partition_through_the_device_path_is_bit_exact(mfmod, split):
    ds = dataset("tiny")
    model = _make(mfmod, ds, 32, "f32", 7, 9, split)
    perm, bp, rb, cb = model.partition()
    o = oracle.partition(ds.rows, ds.cols, ds.cfg.m, ds.cfg.n, 7, 9, split)
    for a, b in zip((perm, bp, rb, cb), o):
        assert np.array_equal(a, b)
    model.close()


def _device_load_matches(mfmod, rows, cols, vals, m, n, gr, gc, split, k=32):
    """mf_load_blocks_device against the oracle's partition (bit-exact) and against a model loaded
    through the host path (same bits after one deterministic epoch: the packed values too)."""
    dev = mfmod.MatrixFactorization(m, n, k, "f32", seed=3, scale=0.1)
    t = torch
    d = dev.P.device
    dev.load_blocks_device(t.from_numpy(rows).to(d), t.from_numpy(cols).to(d), t.from_numpy(vals).to(d), gr, gc, split)
    got = dev.partition()
    want = oracle.partition(rows, cols, m, n, gr, gc, split)
    for name, a, b in zip(("perm", "block_ptr", "row_bounds", "col_bounds"), got, want):
        assert np.array_equal(a, b), (name, gr, gc, split, rows.size)
    host = mfmod.MatrixFactorization(m, n, k, "f32", seed=3, scale=0.1)
    host.load_blocks(rows, cols, vals, gr, gc, split)
    for mode in (mfmod.MF_MODE_DET, mfmod.MF_MODE_DET):
        dev.sgd_epoch(0.01, 0.05, mode)
        host.sgd_epoch(0.01, 0.05, mode)
    for a, b in zip(dev.get_factors(), host.get_factors()):
        assert np.array_equal(a, b)
    dev.close()
    host.close()


@pytest.mark.parametrize("split", [0, 1, 2])
@pytest.mark.parametrize("grid", [(1, 1), (7, 9), (16, 16), (40, 333)])
def test_device_partitioner_is_bit_exact(mfmod, grid, split):
    ds = dataset("tiny")
    _device_load_matches(mfmod, ds.rows, ds.cols, ds.vals, ds.cfg.m, ds.cfg.n, grid[0], grid[1], split)


@pytest.mark.parametrize("count", [1, 63, 4095, 4096, 4097, 8193])
def test_device_partitioner_ragged_sizes_and_duplicates(mfmod, count):
    ds = dataset("tiny")
    rows, cols, vals = ds.rows[:count].copy(), ds.cols[:count].copy(), ds.vals[:count].copy()
    if count > 10:      # the same (row, column) several times: original order must be kept
        rows[count // 2:count // 2 + 5] = rows[0]
        cols[count // 2:count // 2 + 5] = cols[0]
        rows[-1], cols[-1] = rows[1], cols[1]
    _device_load_matches(mfmod, rows, cols, vals, ds.cfg.m, ds.cfg.n, 5, 6, 1)


def test_device_partitioner_skewed_matrix_many_tiles(mfmod):
    ds = dataset("medium", 0.2)     # 1.98 M ratings = 484 tiles, Zipf degrees
    _device_load_matches(mfmod, ds.rows, ds.cols, ds.vals, ds.cfg.m, ds.cfg.n, 64, 96, 2, k=32)
    _device_load_matches(mfmod, ds.rows, ds.cols, ds.vals, ds.cfg.m, ds.cfg.n, 224, 224, 1, k=32)


def test_device_partitioner_rejects_indices_outside_the_matrix_and_accepts_no_ratings(mfmod):
    m, n = 100, 50
    model = mfmod.MatrixFactorization(m, n, 32, "f32")
    d = model.P.device
    rows = torch.tensor([1, 2, 100], dtype=torch.int32, device=d)
    cols = torch.tensor([1, 2, 3], dtype=torch.int32, device=d)
    vals = torch.ones(3, dtype=torch.float32, device=d)
    with pytest.raises(mfmod.MFError) as err:
        model.load_blocks_device(rows, cols, vals, 2, 2, 1)
    assert err.value.code == mfmod.binding.MF_ERANGE
    model.load_blocks_device(rows[:0], cols[:0], vals[:0], 2, 2, 1)
    P0 = model.get_factors()[0]
    model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_DET)
    assert np.array_equal(model.get_factors()[0], P0)
    model.close()


@pytest.mark.parametrize("grid,split", [((7, 9), 1), ((16, 16), 0), ((40, 333), 2), ((1, 1), 1)])
def test_seeded_row_order_host_and_device_partitioners_match_the_oracle(mfmod, grid, split):
    """MF_OPT_ROW_ORDER_SEED: both partitioners give the oracle's seeded permutation bit for bit, and
    a deterministic epoch on it matches the oracle run on that permutation."""
    ds = dataset("tiny")
    cfg = ds.cfg
    gr, gc = grid
    seed = 987654321
    want = oracle.partition(ds.rows, ds.cols, cfg.m, cfg.n, gr, gc, split, row_seed=seed)
    plain = oracle.partition(ds.rows, ds.cols, cfg.m, cfg.n, gr, gc, split)
    if gr * gc < cfg.m:
        assert not np.array_equal(want[0], plain[0])
    Po, Qo = oracle_init(cfg.m, cfg.n, 32, 1, 0.1)
    oracle.sgd_epoch_omp(Po, Qo, ds.rows, ds.cols, ds.vals, want[0], want[1], gr, gc, cfg.lr, cfg.lam)
    for path in ("host", "device"):
        model = mfmod.MatrixFactorization(cfg.m, cfg.n, 32, "f32", seed=1, scale=0.1,
                                          options={mfmod.MF_OPT_ROW_ORDER_SEED: seed})
        if path == "host":
            model.load_blocks(ds.rows, ds.cols, ds.vals, gr, gc, split)
        else:
            d = model.P.device
            model.load_blocks_device(*(torch.from_numpy(x).to(d) for x in (ds.rows, ds.cols, ds.vals)), gr, gc, split)
        for name, a, b in zip(("perm", "block_ptr", "row_bounds", "col_bounds"), model.partition(), want):
            assert np.array_equal(a, b), (path, name)
        model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_DET)
        P, Q = model.get_factors()
        assert np.abs(P - Po).max() <= 1e-4 and np.abs(Q - Qo).max() <= 1e-4, path
        for _ in range(3):
            model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_HOGWILD)       # the work lists follow the new order
        assert np.isfinite(model.rmse())
        model.close()


# ------------------------------------------------------------------------------- RMSE kernel
@pytest.mark.parametrize("storage,k", [("f32", 32), ("f32", 128), ("f16", 128), ("f32", 256), ("f16", 64)])
def test_rmse_kernel_matches_oracle(mfmod, storage, k):
    ds = dataset("tiny")
    model = _make(mfmod, ds, k, storage, 4, 4, 1, seed=5, scale=0.6)
    P, Q = model.get_factors()              # exact: fp32 / binary16 values widen exactly
    tr, tc, tv = model.to_device(ds.test_rows, ds.test_cols, ds.test_vals)
    got = model.rmse(tr, tc, tv)
    want = oracle.rmse(P, Q, ds.test_rows, ds.test_cols, ds.test_vals)
    assert abs(got - want) <= 1e-9 * want
    got_tr = model.rmse()                   # over the loaded training ratings
    want_tr = oracle.rmse(P, Q, ds.rows, ds.cols, ds.vals)
    assert abs(got_tr - want_tr) <= 1e-9 * want_tr
    # ragged tail: 1, 63, 64, 65 entries
    for cnt in (1, 63, 64, 65):
        g = model.rmse(tr[:cnt], tc[:cnt], tv[:cnt])
        w = oracle.rmse(P, Q, ds.test_rows[:cnt], ds.test_cols[:cnt], ds.test_vals[:cnt])
        assert abs(g - w) <= 1e-9 * w
    model.close()


# ------------------------------------------------------------------------------- deterministic mode
def _det_options(mfmod, kernel):
    which = {"auto": mfmod.MF_KERNEL_AUTO, "global": mfmod.MF_KERNEL_GLOBAL, "lds": mfmod.MF_KERNEL_LDS}[kernel]
    return {mfmod.MF_OPT_DET_KERNEL: which}


def _det_one_epoch(mfmod, ds, k, storage, gr, gc, split, lr=None, lam=None, kernel="auto", scale=0.1):
    lr = ds.cfg.lr if lr is None else lr
    lam = ds.cfg.lam if lam is None else lam
    model = _make(mfmod, ds, k, storage, gr, gc, split, scale=scale, options=_det_options(mfmod, kernel))
    try:
        model.sgd_epoch(lr, lam, mfmod.MF_MODE_DET)
    except mfmod.MFError as err:
        model.close()
        if kernel == "lds" and err.code == mfmod.binding.MF_EINVAL:
            pytest.skip("the column strips of this grid do not fit the LDS")
        raise
    P, Q = model.get_factors()
    model.close()
    arith = _arith(storage)
    perm, bp, _, _ = oracle.partition(ds.rows, ds.cols, ds.cfg.m, ds.cfg.n, gr, gc, split)
    Po, Qo = oracle_init(ds.cfg.m, ds.cfg.n, k, 1, scale, arith)
    P0, Q0 = Po.copy(), Qo.copy()
    oracle.sgd_epoch_omp(Po, Qo, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, lr, lam, arith)
    assert not np.array_equal(Po, P0) and not np.array_equal(Qo, Q0)
    return P, Q, Po, Qo


@pytest.mark.parametrize("kernel", ["global", "lds"])
@pytest.mark.parametrize("k", [32, 64, 128, 256])
@pytest.mark.parametrize("grid,split", [((1, 1), 0), ((5, 7), 1), ((32, 32), 1), ((8, 64), 0)])
def test_det_one_epoch_fp32_within_1e4(mfmod, k, grid, split, kernel):
    ds = dataset("tiny")
    P, Q, Po, Qo = _det_one_epoch(mfmod, ds, k, "f32", grid[0], grid[1], split, kernel=kernel)
    assert np.abs(P - Po).max() <= 1e-4 and np.abs(Q - Qo).max() <= 1e-4, (np.abs(P - Po).max(), np.abs(Q - Qo).max())


@pytest.mark.parametrize("kernel", ["global", "lds"])
@pytest.mark.parametrize("k", [32, 128, 256])
def test_det_one_epoch_binary16_storage(mfmod, k, kernel):
    ds = dataset("tiny")
    P, Q, Po, Qo = _det_one_epoch(mfmod, ds, k, "f16", 6, 6, 1, kernel=kernel)
    for X, Xo in ((P, Po), (Q, Qo)):
        assert np.mean(X != Xo) <= 1e-5, float(np.mean(X != Xo))


def test_det_is_reproducible_and_both_kernels_give_the_same_bits(mfmod):
    ds = dataset("tiny")
    outs = []
    for kernel in ("lds", "lds", "global", "global"):
        model = _make(mfmod, ds, 32, "f32", 16, 16, 1, options=_det_options(mfmod, kernel))
        for _ in range(2):
            model.sgd_epoch(ds.cfg.lr, ds.cfg.lam, mfmod.MF_MODE_DET)
        outs.append(model.get_factors())
        model.close()
    for other in outs[1:]:
        assert np.array_equal(outs[0][0], other[0]) and np.array_equal(outs[0][1], other[1])


@pytest.mark.parametrize("storage", ["f32", "f16"])
@pytest.mark.parametrize("grid", [(5, 7), (16, 16), (8, 64), (33, 40)])
def test_one_launch_per_epoch_gives_the_same_bits_as_one_launch_per_stratum(mfmod, grid, storage):
    """Deterministic mode: the ring kernel (MF_OPT_RING = 1) hands the column strips from workgroup
    to workgroup inside one launch; any strip read too early or from a stale cache line would
    change bits."""
    ds = dataset("tiny")
    outs = []
    for ring in (0, 1):
        opts = {mfmod.MF_OPT_DET_KERNEL: mfmod.MF_KERNEL_LDS, mfmod.MF_OPT_RING: ring}
        model = _make(mfmod, ds, 64, storage, grid[0], grid[1], 2, options=opts)
        for _ in range(3):
            model.sgd_epoch(ds.cfg.lr, ds.cfg.lam, mfmod.MF_MODE_DET)
        model.sync()
        outs.append(model.get_factors())
        model.close()
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_ring_kernel_gives_up_cleanly_when_its_wait_limit_is_tiny(mfmod):
    """Failure handling forced from the host: with a wait limit of one poll and one block row far
    heavier than the others, the workgroup that needs its strips finds it not ready, raises the
    abort flag, every workgroup leaves, and the next synchronising call reports MF_EDEVICE (the
    kernel itself ends normally)."""
    ds = dataset("tiny")
    opts = {mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS, mfmod.MF_OPT_RING: 1,
            mfmod.MF_OPT_RING_SPIN_LIMIT: 1}
    model, rows, cols, vals = _one_heavy_block_row(mfmod, opts)
    assert model.epoch_plan(mfmod.MF_MODE_HOGWILD)["kernel"] == "sgd_ring_lds"
    model.sgd_epoch(ds.cfg.lr, ds.cfg.lam, mfmod.MF_MODE_HOGWILD)
    with pytest.raises(mfmod.MFError) as e:
        model.sync()
    assert e.value.code == mfmod.binding.MF_EDEVICE
    # reported once; the context then runs one launch per stratum, which needs no neighbour, and
    # trains on (from fresh factors: the abandoned epoch left them half-updated)
    model.sync()
    plan = model.epoch_plan(mfmod.MF_MODE_HOGWILD)
    assert plan["kernel"] == "sgd_block_lds" and "wait limit" in plan["note"], plan
    B = mfmod.binding
    B.mf_init(model.ctx, model.m, model.n, 128, B.MF_F32, model.P.data_ptr(), model.Qt.data_ptr(), 1, 0.1)
    B.mf_set_option(model.ctx, mfmod.MF_OPT_RING_SPIN_LIMIT, 1 << 22)
    model.load_blocks(rows, cols, vals, 64, 64, 0)                    # a new load may use the one-launch kernel again
    assert model.epoch_plan(mfmod.MF_MODE_HOGWILD)["kernel"] == "sgd_ring_lds"
    tr, tc, tv = model.to_device(rows[::7], cols[::7], vals[::7])
    before = model.rmse(tr, tc, tv)
    for _ in range(3):
        model.sgd_epoch(0.002, ds.cfg.lam, mfmod.MF_MODE_HOGWILD)
    assert model.rmse(tr, tc, tv) < before
    model.close()


# ------------------------------------------------------------------------------- divergence is reported, not wrapped round
@pytest.mark.parametrize("ring", [1, 0])
@pytest.mark.parametrize("case", ["value", "change", "sane"])
def test_hogwild_lds_kernel_reports_values_outside_its_fixed_point_range(mfmod, ring, case):
    """The Hogwild LDS kernel keeps Qt as 32-bit fixed point in [-128, 128).  Forced from the host:
    factors preset to 70 (value watch, limit 64), or ratings so large that one step changes an
    element by more than 4 (change watch).  Every kernel ends normally; the next synchronising
    call returns MF_ERANGE once.  Sane inputs raise nothing."""
    ds = dataset("tiny")
    cfg = ds.cfg
    B = mfmod.binding
    opts = {mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS, mfmod.MF_OPT_RING: ring}
    model = mfmod.MatrixFactorization(cfg.m, cfg.n, 32, "f32", seed=1, scale=0.1, options=opts)
    vals = ds.vals
    lr = 0.0
    if case == "value":
        model.Qt.fill_(70.0)
    elif case == "change":
        vals = np.full_like(ds.vals, 3.0e4)      # e ~ 3e4, lr*e*p ~ 0.01 * 3e4 * 0.05 = 15 > 4
        lr = 0.01
    model.load_blocks(ds.rows, ds.cols, vals, 16, 16, 1)
    model.sgd_epoch(lr, 0.0, mfmod.MF_MODE_HOGWILD)
    if case == "sane":
        model.sync()
    else:
        with pytest.raises(mfmod.MFError) as e:
            model.sync()
        assert e.value.code == B.MF_ERANGE, e.value
        model.sync()                               # reported once
        if case == "value":
            # the values themselves were inside +-128 and came back unchanged (lr = 0)
            assert float(model.Qt.min()) == 70.0 and float(model.Qt.max()) == 70.0
    model.close()


# ------------------------------------------------------------------------------- randomised stratum order
@pytest.mark.parametrize("grid", [(5, 7), (16, 16), (8, 64), (33, 40)])
def test_shuffled_strata_deterministic_mode_matches_oracle_on_every_kernel(mfmod, grid):
    """Two epochs with two different stratum permutations: every launch scheme (ring kernel with
    its generalised waits, one launch per stratum, global kernel) gives the same bits, and they
    agree with the oracle run in the same orders."""
    ds = dataset("tiny")
    gr, gc = grid
    cfg = ds.cfg
    orders = [mfmod.binding.mf_stratum_order(77, e, gc) for e in range(2)]
    assert all(np.array_equal(o, oracle.stratum_order(77, e, gc)) for e, o in enumerate(orders))
    outs = []
    for kernel, ring in (("lds", 1), ("lds", 0), ("global", 0)):
        opts = dict(_det_options(mfmod, kernel))
        opts[mfmod.MF_OPT_RING] = ring
        model = _make(mfmod, ds, 32, "f32", gr, gc, 1, options=opts)
        for o in orders:
            model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_DET, stratum_order=o)
        outs.append(model.get_factors())
        model.close()
    for other in outs[1:]:
        assert np.array_equal(outs[0][0], other[0]) and np.array_equal(outs[0][1], other[1])
    perm, bp, _, _ = oracle.partition(ds.rows, ds.cols, cfg.m, cfg.n, gr, gc, 1)
    Po, Qo = oracle_init(cfg.m, cfg.n, 32, 1, 0.1)
    for o in orders:
        oracle.sgd_epoch_ordered(Po, Qo, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, cfg.lr, cfg.lam, o)
    assert np.abs(outs[0][0] - Po).max() <= 1e-4 and np.abs(outs[0][1] - Qo).max() <= 1e-4
    # and the order does change the result (natural order differs by far more than the tolerance)
    Pn, Qn = oracle_init(cfg.m, cfg.n, 32, 1, 0.1)
    for _ in orders:
        oracle.sgd_epoch_omp(Pn, Qn, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, cfg.lr, cfg.lam)
    assert np.abs(Qn - Qo).max() > 1e-3


@pytest.mark.parametrize("ring", [1, 0])
def test_shuffled_strata_hogwild_final_rmse(mfmod, ring):
    ds = dataset("tiny")
    cfg = ds.cfg
    gr = gc = 32
    opts = {mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS, mfmod.MF_OPT_RING: ring}
    model = _make(mfmod, ds, cfg.k, "f32", gr, gc, 1, options=opts)
    perm, bp, _, _ = oracle.partition(ds.rows, ds.cols, cfg.m, cfg.n, gr, gc, 1)
    Po, Qo = oracle_init(cfg.m, cfg.n, cfg.k, 1, 0.1)
    for e in range(cfg.epochs):
        o = oracle.stratum_order(3, e, gc)
        model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_HOGWILD, stratum_order=o)
        oracle.sgd_epoch_ordered(Po, Qo, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, cfg.lr, cfg.lam, o)
    tr, tc, tv = model.to_device(ds.test_rows, ds.test_cols, ds.test_vals)
    got = model.rmse(tr, tc, tv)
    want = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
    model.close()
    assert abs(got - want) <= 5e-3 * want, (got, want)


def test_stratum_order_must_be_a_permutation(mfmod):
    ds = dataset("tiny")
    model = _make(mfmod, ds, 32, "f32", 4, 6, 1)
    for bad in ([0, 1, 2, 3, 4, 4], [0, 1, 2, 3, 4, 6], [-1, 1, 2, 3, 4, 5]):
        with pytest.raises(mfmod.MFError) as e:
            model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_DET, stratum_order=np.array(bad, np.int32))
        assert e.value.code == mfmod.binding.MF_EINVAL
    model.close()


def test_ring_kernel_with_an_order_gives_up_cleanly_when_its_wait_limit_is_tiny(mfmod):
    ds = dataset("tiny")
    opts = {mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS, mfmod.MF_OPT_RING: 1,
            mfmod.MF_OPT_RING_SPIN_LIMIT: 1}
    model = _one_heavy_block_row(mfmod, opts)[0]
    assert model.epoch_plan(mfmod.MF_MODE_HOGWILD)["kernel"] == "sgd_ring_lds"
    model.sgd_epoch(ds.cfg.lr, ds.cfg.lam, mfmod.MF_MODE_HOGWILD, stratum_order=oracle.stratum_order(1, 0, 64))
    with pytest.raises(mfmod.MFError) as e:
        model.sync()
    assert e.value.code == mfmod.binding.MF_EDEVICE
    model.close()


# ------------------------------------------------------------------------------- every rating exactly once, in every Hogwild kernel
@pytest.mark.parametrize("kernel,ring,grid", [("lds", 1, (16, 16)), ("lds", 1, (8, 40)), ("lds", 1, (33, 40)),
                                              ("lds", 1, (8, 37)), ("lds", 1, (3, 40)),
                                              ("lds", 0, (16, 16)), ("lds", 0, (8, 40)),
                                              ("global_atomics", 0, (8, 8))])
def test_hogwild_visits_every_rating_exactly_once(mfmod, kernel, ring, grid):
    """With a tiny step and no regularisation an epoch is, to first order, a sum over the ratings
    that does not depend on their order: P' = P + lr * sum_v e0_uv q_v.  At lr = 1e-5 the order
    changes an element by at most 2.6e-7 (measured with the oracle: canonical against reversed
    strata and against one unblocked sweep, on these grids), the 2^-24 grid of the strip moves an
    element of Qt by up to 7e-7, while a rating that is missed or applied twice moves its row of
    P by up to 2.7e-6 and a block whose strip is not written back moves its columns by 1.6e-5.
    Every launch scheme (ring kernel on square and rectangular grids, one launch per stratum, L2
    atomics) must agree with the oracle's canonical order to 6e-7 in P and 1.2e-6 in Qt."""
    ds = dataset("tiny")
    cfg = ds.cfg
    gr, gc = grid
    lr, lam = 1e-5, 0.0
    which = {"lds": mfmod.MF_HOGWILD_LDS, "global_atomics": mfmod.MF_HOGWILD_GLOBAL_ATOMICS}[kernel]
    model = _make(mfmod, ds, 32, "f32", gr, gc, 1, options={mfmod.MF_OPT_HOGWILD_KERNEL: which, mfmod.MF_OPT_RING: ring})
    model.sgd_epoch(lr, lam, mfmod.MF_MODE_HOGWILD)
    P, Q = model.get_factors()
    model.close()
    perm, bp, _, _ = oracle.partition(ds.rows, ds.cols, cfg.m, cfg.n, gr, gc, 1)
    P0, Q0 = oracle_init(cfg.m, cfg.n, 32, 1, 0.1)
    Po, Qo = P0.copy(), Q0.copy()
    oracle.sgd_epoch_omp(Po, Qo, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, lr, lam)
    assert np.abs(Po - P0).max() > 5e-5                      # the epoch does move the factors
    assert np.abs(P - Po).max() <= 6e-7 and np.abs(Q - Qo).max() <= 1.2e-6, (np.abs(P - Po).max(), np.abs(Q - Qo).max())


@pytest.mark.parametrize("ring,waves,gc,load", [(1, 0, 6, "host"), (0, 0, 6, "host"), (1, 5, 6, "device"),
                                                (1, 0, 13, "host"), (0, 0, 6, "streamed")])
def test_hogwild_visits_the_pieces_of_cut_rows_exactly_once(mfmod, ring, waves, gc, load):
    """The same first-order argument for rows so long that the LDS kernel shares them out over
    several wavefronts and keeps their p_u in LDS while the block runs: two rows with 20 000 and
    12 000 ratings move by about 3e-3 at lr = 1e-6; the order of their ratings matters to about
    6e-6 and the 2^-24 grid of the LDS copy to about 4e-6, while a piece that is skipped or applied
    twice (a fourteenth of the row or more) moves the row by 2e-4."""
    ds = dataset("tiny")
    cfg = ds.cfg
    rows = ds.rows.copy()
    rows[:20000] = 7
    rows[20000:32000] = 1500
    gr, lr, lam = 4, 1e-6, 0.0
    options = {mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS, mfmod.MF_OPT_RING: ring}
    if waves:
        options[mfmod.MF_OPT_LDS_WAVES] = waves
    model = mfmod.MatrixFactorization(cfg.m, cfg.n, 32, "f32", seed=1, scale=0.1, options=options)
    if load == "device":
        d = model.P.device
        model.load_blocks_device(*(torch.from_numpy(x).to(d) for x in (rows, ds.cols, ds.vals)), gr, gc, 1)
    elif load == "streamed":
        model.load_blocks_streamed(rows, ds.cols, ds.vals, gr, gc, 1)
    else:
        model.load_blocks(rows, ds.cols, ds.vals, gr, gc, 1)
    model.sgd_epoch(lr, lam, mfmod.MF_MODE_HOGWILD)
    P, Q = model.get_factors()
    model.close()
    perm, bp, _, _ = oracle.partition(rows, ds.cols, cfg.m, cfg.n, gr, gc, 1)
    P0, Q0 = oracle_init(cfg.m, cfg.n, 32, 1, 0.1)
    Po, Qo = P0.copy(), Q0.copy()
    oracle.sgd_epoch_omp(Po, Qo, rows, ds.cols, ds.vals, perm, bp, gr, gc, lr, lam)
    long_rows = np.array([7, 1500])
    others = np.setdiff1d(np.arange(cfg.m), long_rows)
    assert np.abs(Po[long_rows] - P0[long_rows]).max() > 1e-3
    d_long = float(np.abs(P[long_rows] - Po[long_rows]).max())
    d_rest = float(np.abs(P[others] - Po[others]).max())
    d_q = float(np.abs(Q - Qo).max())
    print("cut rows exactly once, ring=%d waves=%d: long rows %.2e, other rows %.2e, Qt %.2e" % (ring, waves, d_long, d_rest, d_q),
          flush=True)
    assert d_long <= 3e-5 and d_rest <= 6e-7 and d_q <= 2e-6, (d_long, d_rest, d_q)


def test_suggested_grids_train_to_the_oracle_result(mfmod):
    """mf_suggest_grid's answer for both modes is a grid the kernels accept and train on."""
    ds = dataset("tiny")
    cfg = ds.cfg
    for mode in (mfmod.MF_MODE_HOGWILD, mfmod.MF_MODE_DET):
        gr, gc, split = mfmod.binding.mf_suggest_grid(cfg.m, cfg.n, ds.rows.size, cfg.k, mode)
        Po, Qo, _ = oracle_train(ds, gr, gc, split, cfg.epochs)
        want = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
        got = _train_gpu(mfmod, ds, cfg.k, "f32", gr, gc, split, mode, cfg.epochs)
        tol = 5e-3 * want if mode == mfmod.MF_MODE_HOGWILD else 1e-3
        assert abs(got - want) <= tol, (mode, gr, gc, got, want)


# ------------------------------------------------------------------------------- ratings streamed from the host
@pytest.mark.parametrize("kernel", ["lds", "global"])
@pytest.mark.parametrize("grid", [(5, 7), (16, 16), (1, 1)])
def test_streamed_ratings_deterministic_mode_is_bit_identical_to_resident(mfmod, grid, kernel):
    """mf_load_blocks_streamed keeps the ratings in pinned host memory and copies every stratum in
    while the one before is computed: over several epochs (the two device buffers are reused) and
    with a shuffled stratum order the deterministic result must equal the resident path's bits."""
    ds = dataset("tiny")
    cfg = ds.cfg
    gr, gc = grid
    opts = dict(_det_options(mfmod, kernel))
    opts[mfmod.MF_OPT_RING] = 0
    outs = []
    for streamed in (False, True):
        model = mfmod.MatrixFactorization(cfg.m, cfg.n, 32, "f32", seed=1, scale=0.1, options=opts)
        (model.load_blocks_streamed if streamed else model.load_blocks)(ds.rows, ds.cols, ds.vals, gr, gc, 1)
        for e in range(3):
            model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_DET)
        model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_DET, stratum_order=oracle.stratum_order(5, 0, gc))
        outs.append(model.get_factors())
        if streamed:
            with pytest.raises(mfmod.MFError):
                model.rmse()                      # the training ratings are not on the device
            model.load_blocks(ds.rows, ds.cols, ds.vals, gr, gc, 1)       # back to the resident path
            assert np.isfinite(model.rmse())
        model.close()
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])
    perm, bp, _, _ = oracle.partition(ds.rows, ds.cols, cfg.m, cfg.n, gr, gc, 1)
    Po, Qo = oracle_init(cfg.m, cfg.n, 32, 1, 0.1)
    for e in range(3):
        oracle.sgd_epoch_omp(Po, Qo, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, cfg.lr, cfg.lam)
    oracle.sgd_epoch_ordered(Po, Qo, ds.rows, ds.cols, ds.vals, perm, bp, gr, gc, cfg.lr, cfg.lam, oracle.stratum_order(5, 0, gc))
    assert np.abs(outs[1][0] - Po).max() <= 1e-4 and np.abs(outs[1][1] - Qo).max() <= 1e-4


def test_streamed_ratings_hogwild_final_rmse(mfmod):
    ds = dataset("medium", 0.05)
    cfg = ds.cfg
    gr = gc = 48
    epochs = 6
    Po, Qo, _ = oracle_train(ds, gr, gc, 1, epochs)
    want = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
    model = mfmod.MatrixFactorization(cfg.m, cfg.n, cfg.k, "f32", seed=1, scale=0.1,
                                      options={mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS})
    model.load_blocks_streamed(ds.rows, ds.cols, ds.vals, gr, gc, 1)
    tr, tc, tv = model.to_device(ds.test_rows, ds.test_cols, ds.test_vals)
    for _ in range(epochs):
        model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_HOGWILD)
    got = model.rmse(tr, tc, tv)
    model.close()
    assert abs(got - want) <= 5e-3 * want, (got, want)


def test_det_edge_cases(mfmod):
    rng = np.random.default_rng(3)
    # duplicates of one (u, v), a single long row, a single long column, and empty strata
    m, n, k = 70, 90, 32
    rows = np.concatenate([np.full(300, 5), rng.integers(0, m, 300), np.full(130, 9), np.full(40, 11)]).astype(np.int32)
    cols = np.concatenate([rng.integers(0, n, 300), np.full(300, 17), np.full(130, 21), np.full(40, 21)]).astype(np.int32)
    vals = rng.uniform(1, 5, rows.size).astype(np.float32)
    for gr, gc, kernel in [(1, 1, "global"), (1, 1, "lds"), (3, 3, "global"), (3, 3, "lds"), (7, 30, "global"),
                           (7, 30, "lds")]:
        model = mfmod.MatrixFactorization(m, n, k, "f32", seed=4, scale=0.1, options=_det_options(mfmod, kernel))
        model.load_blocks(rows, cols, vals, gr, gc, 0)
        model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_DET)
        P, Q = model.get_factors()
        model.close()
        perm, bp, _, _ = oracle.partition(rows, cols, m, n, gr, gc, 0)
        Po, Qo = oracle_init(m, n, k, 4, 0.1)
        oracle.sgd_epoch(Po, Qo, rows, cols, vals, perm, bp, gr, gc, 0.01, 0.05)
        assert np.abs(P - Po).max() <= 1e-4 and np.abs(Q - Qo).max() <= 1e-4
        untouched = np.setdiff1d(np.arange(m), rows)
        P0, _ = oracle_init(m, n, k, 4, 0.1, oracle.ARITH_F32)
        assert np.array_equal(P[untouched], P0[untouched])          # rows without ratings never change


def test_empty_rating_set_is_a_valid_epoch(mfmod):
    model = mfmod.MatrixFactorization(50, 40, 32, "f32", seed=2, scale=0.1)
    z = np.zeros(0, np.int32)
    model.load_blocks(z, z, np.zeros(0, np.float32), 4, 4, 1)
    before = model.get_factors()
    model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_DET)
    model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_HOGWILD)
    after = model.get_factors()
    assert np.array_equal(before[0], after[0]) and np.array_equal(before[1], after[1])
    with pytest.raises(mfmod.MFError) as e:
        model.rmse()
    assert e.value.code == mfmod.binding.MF_EINVAL
    model.close()


def test_zero_learning_rate_changes_nothing_in_either_mode(mfmod):
    ds = dataset("tiny")
    model = _make(mfmod, ds, 128, "f32", 8, 8, 1,
                  options={mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_GLOBAL_ATOMICS})
    before = model.get_factors()
    model.sgd_epoch(0.0, 0.05, mfmod.MF_MODE_DET)
    model.sgd_epoch(0.0, 0.05, mfmod.MF_MODE_HOGWILD)
    after = model.get_factors()
    assert np.array_equal(before[0], after[0]) and np.array_equal(before[1], after[1])
    model.close()
    # the LDS kernel holds the strip of Qt as fixed point with 24 fraction bits: a pass with a
    # zero step puts Qt on that grid (at most half a step away) and a second pass changes nothing
    model = _make(mfmod, ds, 128, "f32", 8, 8, 1, options={mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS})
    before = model.get_factors()
    model.sgd_epoch(0.0, 0.05, mfmod.MF_MODE_HOGWILD)
    once = model.get_factors()
    model.sgd_epoch(0.0, 0.05, mfmod.MF_MODE_HOGWILD)
    twice = model.get_factors()
    assert np.array_equal(before[0], once[0]) and np.abs(before[1] - once[1]).max() <= 2.0 ** -25
    assert np.array_equal(once[1] * 2.0 ** 24, np.round(once[1] * 2.0 ** 24))
    assert np.array_equal(once[0], twice[0]) and np.array_equal(once[1], twice[1])
    model.close()


# ------------------------------------------------------------------------------- full runs of configuration 1
def _train_gpu(mfmod, ds, k, storage, gr, gc, split, mode, epochs, options=None, scale=0.1):
    model = _make(mfmod, ds, k, storage, gr, gc, split, scale=scale, options=options)
    tr, tc, tv = model.to_device(ds.test_rows, ds.test_cols, ds.test_vals)
    for _ in range(epochs):
        model.sgd_epoch(ds.cfg.lr, ds.cfg.lam, mode)
    out = model.rmse(tr, tc, tv)
    model.close()
    return out


def test_tiny_config_det_final_rmse_within_1e3(mfmod):
    ds = dataset("tiny")
    gr, gc = 16, 16
    Po, Qo, _ = oracle_train(ds, gr, gc, 1, ds.cfg.epochs)
    want = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
    got = _train_gpu(mfmod, ds, ds.cfg.k, "f32", gr, gc, 1, mfmod.MF_MODE_DET, ds.cfg.epochs)
    assert abs(got - want) <= 1e-3, (got, want)


@pytest.mark.parametrize("kernel", ["lds", "lds_per_stratum", "global_atomics"])
@pytest.mark.parametrize("storage", ["f32", "f16"])
def test_tiny_config_hogwild_final_rmse_within_half_percent(mfmod, kernel, storage):
    ds = dataset("tiny")
    Po, Qo, _ = oracle_train(ds, 8, 8, 1, ds.cfg.epochs, arith=_arith(storage))
    want = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
    which = mfmod.MF_HOGWILD_GLOBAL_ATOMICS if kernel == "global_atomics" else mfmod.MF_HOGWILD_LDS
    got = _train_gpu(mfmod, ds, ds.cfg.k, storage, 8, 8, 1, mfmod.MF_MODE_HOGWILD, ds.cfg.epochs,
                     options={mfmod.MF_OPT_HOGWILD_CHUNK: 32, mfmod.MF_OPT_LDS_CHUNK: 16,
                              mfmod.MF_OPT_HOGWILD_KERNEL: which,
                              mfmod.MF_OPT_RING: 0 if kernel == "lds_per_stratum" else 1})
    print("tiny HOGWILD %s %s: rmse gpu %.6f oracle %.6f" % (kernel, storage, got, want), flush=True)
    assert abs(got - want) <= 0.005 * want, (got, want)


@pytest.mark.parametrize("k,storage", [(32, "f32"), (64, "f16"), (256, "f32"), (256, "f16")])
def test_hogwild_lds_kernel_other_shapes_and_long_rows(mfmod, k, storage):
    """LDS kernel on a matrix with two very long rows (cut into pieces that share p_u) and a
    ragged strip width; checked against the oracle's held-out RMSE once both have converged."""
    rng = np.random.default_rng(17)
    m, n, nnz = 600, 333, 60000
    rows = rng.integers(0, m, nnz).astype(np.int32)
    rows[:3000] = 5
    rows[3000:5000] = 77
    cols = rng.integers(0, n, nnz).astype(np.int32)
    ps = rng.uniform(0.2, 1.0, (m, 4))
    qs = rng.uniform(0.2, 1.0, (n, 4))
    vals = (np.einsum("ij,ij->i", ps[rows], qs[cols]) + rng.normal(0, 0.05, nnz)).astype(np.float32)
    hold = rng.random(nnz) < 0.1
    tr_r, tr_c, tr_v = (np.ascontiguousarray(x[~hold]) for x in (rows, cols, vals))
    te_r, te_c, te_v = (np.ascontiguousarray(x[hold]) for x in (rows, cols, vals))
    gr, gc, epochs, lr, lam = 3, 5, 60, 0.01, 0.05
    model = mfmod.MatrixFactorization(m, n, k, storage, seed=3, scale=0.1,
                                      options={mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS,
                                               mfmod.MF_OPT_LDS_CHUNK: 24, mfmod.MF_OPT_LDS_WAVES: 8})
    model.load_blocks(tr_r, tr_c, tr_v, gr, gc, 1)
    for _ in range(epochs):
        model.sgd_epoch(lr, lam, mfmod.MF_MODE_HOGWILD)
    a, b, c = model.to_device(te_r, te_c, te_v)
    got = model.rmse(a, b, c)
    model.close()
    arith = _arith(storage)
    perm, bp, _, _ = oracle.partition(tr_r, tr_c, m, n, gr, gc, 1)
    Po, Qo = oracle_init(m, n, k, 3, 0.1, arith)
    for _ in range(epochs):
        oracle.sgd_epoch(Po, Qo, tr_r, tr_c, tr_v, perm, bp, gr, gc, lr, lam, arith)
    want = oracle.rmse(Po, Qo, te_r, te_c, te_v)
    print("long rows k=%d %s: rmse gpu %.6f oracle %.6f" % (k, storage, got, want), flush=True)
    assert abs(got - want) <= 0.005 * want, (got, want)


@pytest.mark.parametrize("ring", [1, 0])
@pytest.mark.parametrize("k", [32, 128, 256])
def test_hogwild_pieces_of_long_rows_in_one_wavefront_follow_the_sequential_order(mfmod, k, ring):
    """With ONE wavefront per workgroup the pieces of a cut row run one after the other in stored
    order, so the Hogwild LDS kernel (pieces of long rows included: rows requested ahead and
    corrected by the wavefront's own changes) must reproduce the oracle's sequential epoch up to
    the 2^-24 grid of its Qt strip.  A row value that missed changes still in flight would be off
    by lr*e*q per missed rating, about 1e-2 here."""
    rng = np.random.default_rng(23)
    m, n, nnz = 300, 200, 30000
    rows = rng.integers(0, m, nnz).astype(np.int32)
    rows[:4000] = 9            # two long rows: ~800 and ~500 ratings in every block of their block row
    rows[4000:6500] = 150
    rows[6500:6600] = 151      # and a row of moderate length right after a long one
    cols = rng.integers(0, n, nnz).astype(np.int32)
    vals = rng.uniform(1.0, 5.0, nnz).astype(np.float32)
    gr, gc, lr, lam = 2, 5, 0.02, 0.05
    model = mfmod.MatrixFactorization(m, n, k, "f32", seed=5, scale=0.3,
                                      options={mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS,
                                               mfmod.MF_OPT_LDS_CHUNK: 24, mfmod.MF_OPT_LDS_WAVES: 1,
                                               mfmod.MF_OPT_RING: ring})
    model.load_blocks(rows, cols, vals, gr, gc, 1)
    model.sgd_epoch(lr, lam, mfmod.MF_MODE_HOGWILD)
    P, Qt = model.get_factors()
    model.close()
    perm, bp, _, _ = oracle.partition(rows, cols, m, n, gr, gc, 1)
    Po, Qo = oracle_init(m, n, k, 5, 0.3, oracle.ARITH_F32)
    oracle.sgd_epoch(Po, Qo, rows, cols, vals, perm, bp, gr, gc, lr, lam, oracle.ARITH_F32)
    dp = float(np.abs(P - Po).max())
    dq = float(np.abs(Qt - Qo).max())
    print("long rows, one wavefront, k=%d ring=%d: max|dP| %.2e max|dQ| %.2e" % (k, ring, dp, dq), flush=True)
    assert dp <= 2e-4 and dq <= 2e-4, (dp, dq)


@pytest.mark.parametrize("storage,k,grid", [("f32", 128, (8, 32)), ("f32", 64, (8, 20)), ("f16", 128, (8, 32)),
                                             ("f32", 256, (8, 63))])
def test_packed_strips_give_the_bits_of_whole_strips(mfmod, storage, k, grid):
    """When the blocks have ratings in a minority of their strips' columns, the Hogwild LDS kernels
    keep only those columns in LDS, packed (a table of touched columns per block, made at load
    time).  With ONE wavefront per workgroup the Hogwild arithmetic is sequential, so the packed
    form -- one launch per epoch and one launch per stratum -- must give the bits of the form that
    keeps whole strips (MF_OPT_PACK_STRIPS = 0), in every column that has a rating.  A column
    without ratings is never copied by the packed form and is put on the 2^-24 grid of the strip
    by the other: there the packed form must return the initial value.
    (Strips of at most 4096 words: what one wavefront's 64 piece bits cover.)"""
    ds = dataset("tiny")
    take = 5600                                  # about half of a block's strip columns have a rating
    rows, cols, vals = ds.rows[:take].copy(), ds.cols[:take].copy(), ds.vals[:take].copy()
    cols[cols >= 990] -= 500                     # columns 990..999 have no ratings at all
    gr, gc = grid
    outs, notes = [], []
    for ring, pack in ((1, 1), (0, 1), (0, 0)):
        model = mfmod.MatrixFactorization(ds.cfg.m, ds.cfg.n, k, storage, seed=3, scale=0.1,
                                          options={mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS,
                                                   mfmod.MF_OPT_LDS_WAVES: 1, mfmod.MF_OPT_RING: ring,
                                                   mfmod.MF_OPT_PACK_STRIPS: pack})
        model.load_blocks(rows, cols, vals, gr, gc, 0)
        if not outs:
            P0, Q0 = model.get_factors()
        plan = model.epoch_plan(mfmod.MF_MODE_HOGWILD)
        assert plan["kernel"] == ("sgd_ring_lds" if ring else "sgd_block_lds"), plan
        notes.append(plan["note"])
        for epoch in range(3):      # the first in natural order of the strata, then two shuffled ones
            order = oracle.stratum_order(11, epoch, gc) if epoch else None
            model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_HOGWILD, stratum_order=order)
        model.sync()
        outs.append(model.get_factors())
        model.close()
    assert "touched columns" in notes[0] and "touched columns" in notes[1] and "touched columns" not in notes[2], notes
    rated = np.zeros(ds.cfg.n, bool)
    rated[cols] = True
    assert not rated[990:].any() and rated[:990].sum() > 900
    for packed in outs[:2]:
        assert np.array_equal(packed[0], outs[2][0])                        # P
        assert np.array_equal(packed[1][rated], outs[2][1][rated])          # Qt where it was ever used
        assert np.array_equal(packed[1][~rated], Q0[~rated])                # and never touched elsewhere
    assert not np.array_equal(outs[0][1][rated], Q0[rated])


@pytest.mark.parametrize("k,grid,take,whole_strip_fits", [(128, (16, 16), 9500, True), (256, (4, 4), 3000, False)])
@pytest.mark.parametrize("ring", [1, 0])
def test_packed_strips_with_sixteen_wavefronts_visit_every_rating_once(mfmod, ring, k, grid, take, whole_strip_fits):
    """The first-order argument of test_hogwild_visits_every_rating_exactly_once for the form that
    keeps only the touched columns of a strip in LDS, with 16 wavefronts per workgroup: at
    lr = 1e-5 and lambda = 0 the order of the ratings matters to second order only, while one
    rating that is missed moves its row by up to 3e-6, and a touched column that went to the wrong
    slot, was not copied in (stale LDS) or not copied back shows at full size.  Second case: strips
    of 250 columns of k = 256, which do not fit the LDS whole (256 KB) -- only the packed form can
    run them there; with packing switched off the L2-atomics kernel takes over."""
    ds = dataset("tiny")
    cfg = ds.cfg
    rows, cols, vals = ds.rows[:take], ds.cols[:take], ds.vals[:take]
    gr, gc = grid
    lr, lam = 1e-5, 0.0
    model = mfmod.MatrixFactorization(cfg.m, cfg.n, k, "f32", seed=1, scale=0.1,
                                      options={mfmod.MF_OPT_RING: ring, mfmod.MF_OPT_LDS_WAVES: 16})
    model.load_blocks(rows, cols, vals, gr, gc, 1)
    plan = model.epoch_plan(mfmod.MF_MODE_HOGWILD)
    assert plan["kernel"] == ("sgd_ring_lds" if ring else "sgd_block_lds") and plan["waves"] == 16, plan
    assert "touched columns" in plan["note"], plan
    model.sgd_epoch(lr, lam, mfmod.MF_MODE_HOGWILD)
    P, Q = model.get_factors()
    mfmod.binding.mf_set_option(model.ctx, mfmod.MF_OPT_PACK_STRIPS, 0)
    model.load_blocks(rows, cols, vals, gr, gc, 1)
    other = model.epoch_plan(mfmod.MF_MODE_HOGWILD)
    assert "touched columns" not in other["note"] and (other["kernel"] == "sgd_chunks") == (not whole_strip_fits), other
    model.close()
    perm, bp, _, _ = oracle.partition(rows, cols, cfg.m, cfg.n, gr, gc, 1)
    P0, Q0 = oracle_init(cfg.m, cfg.n, k, 1, 0.1)
    Po, Qo = P0.copy(), Q0.copy()
    oracle.sgd_epoch_omp(Po, Qo, rows, cols, vals, perm, bp, gr, gc, lr, lam)
    dp, dq = float(np.abs(P - Po).max()), float(np.abs(Q - Qo).max())
    moved = float(np.abs(Po - P0).max())
    print("packed strips, 16 wavefronts, k=%d ring=%d: max|dP| %.2e max|dQ| %.2e, the epoch moves P by up to %.2e"
          % (k, ring, dp, dq, moved), flush=True)
    assert moved > 5e-6 and dp <= 6e-7 and dq <= 1.2e-6, (moved, dp, dq)


def test_epochs_in_one_call_reject_a_count_out_of_range(mfmod):
    ds = dataset("tiny")
    model = _make(mfmod, ds, 32, "f32", 8, 8, 1)
    for count in (0, -3, 4097):
        with pytest.raises(mfmod.MFError) as e:
            model.sgd_epochs(0.01, 0.05, mfmod.MF_MODE_DET, count)
        assert e.value.code == mfmod.binding.MF_EINVAL
    model.sgd_epochs(0.01, 0.05, mfmod.MF_MODE_DET, 1)
    model.sync()
    model.close()


@pytest.mark.parametrize("storage,k,grid,pack", [("f32", 128, (8, 32), 1), ("f32", 32, (16, 16), 1), ("f32", 64, (5, 23), 1),
                                                  ("f16", 128, (8, 32), 2), ("f32", 128, (33, 40), 2), ("f16", 64, (7, 7), 1)])
def test_epochs_in_one_launch_give_the_bits_of_epochs_one_by_one(mfmod, storage, k, grid, pack):
    """mf_sgd_epochs runs its epochs in one launch of the ring kernel: a block row starts the next
    epoch while others are still in the one before, held back only by the strips it needs.  In
    deterministic mode four epochs that way must give the bits of four calls of mf_sgd_epoch (square,
    rectangular and closed grids, whole and packed strips), and of the kernel that launches every
    stratum by itself; in Hogwild mode (lr tiny, no regularisation: an epoch is a sum over the
    ratings to first order) every rating must have been applied four times."""
    ds = dataset("tiny")
    take = 7000
    rows, cols, vals = ds.rows[:take].copy(), ds.cols[:take].copy(), ds.vals[:take].copy()
    gr, gc = grid
    outs = []
    for ring, together in ((1, True), (1, False), (0, True)):
        model = mfmod.MatrixFactorization(ds.cfg.m, ds.cfg.n, k, storage, seed=3, scale=0.1,
                                          options={mfmod.MF_OPT_DET_KERNEL: mfmod.MF_KERNEL_LDS, mfmod.MF_OPT_RING: ring,
                                                   mfmod.MF_OPT_PACK_STRIPS: pack})
        model.load_blocks(rows, cols, vals, gr, gc, 0)
        assert model.epoch_plan(mfmod.MF_MODE_DET)["kernel"] == ("sgd_ring_lds" if ring else "sgd_block_lds")
        model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_DET)          # the counters do not start at zero
        if together:
            model.sgd_epochs(0.01, 0.05, mfmod.MF_MODE_DET, 4)
        else:
            for _ in range(4):
                model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_DET)
        model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_DET)
        model.sync()
        outs.append(model.get_factors())
        model.close()
    for P, Q in outs[1:]:
        assert np.array_equal(P, outs[0][0]) and np.array_equal(Q, outs[0][1])
    if storage == "f32":
        lr = 1e-5
        model = mfmod.MatrixFactorization(ds.cfg.m, ds.cfg.n, k, storage, seed=3, scale=0.1,
                                          options={mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS, mfmod.MF_OPT_RING: 1})
        model.load_blocks(rows, cols, vals, gr, gc, 1)
        assert model.epoch_plan(mfmod.MF_MODE_HOGWILD)["kernel"] == "sgd_ring_lds"
        P0, Q0 = model.get_factors()
        model.sgd_epochs(lr, 0.0, mfmod.MF_MODE_HOGWILD, 4)
        P4, Q4 = model.get_factors()
        model.close()
        perm, bp, _, _ = oracle.partition(rows, cols, ds.cfg.m, ds.cfg.n, gr, gc, 1)
        Po, Qo = P0.astype(np.float64), Q0.astype(np.float64)
        for _ in range(4):
            oracle.sgd_epoch_omp(Po, Qo, rows, cols, vals, perm, bp, gr, gc, lr, 0.0)
        dp, dq = float(np.abs(P4 - Po).max()), float(np.abs(Q4 - Qo).max())
        print("four Hogwild epochs in one launch: max|dP| %.2e max|dQ| %.2e" % (dp, dq), flush=True)
        assert dp <= 2.4e-6 and dq <= 4.8e-6, (dp, dq)


@pytest.mark.parametrize("storage,k,grid", [("f32", 128, (8, 32)), ("f32", 32, (8, 16)), ("f32", 64, (16, 20)),
                                             ("f16", 128, (8, 32)), ("f16", 64, (8, 13)), ("f32", 256, (8, 63))])
def test_deterministic_mode_with_packed_strips_gives_the_same_bits(mfmod, storage, k, grid):
    """The deterministic LDS kernels keep only the touched columns of a strip in LDS too when few
    are touched (they move a strip column by column; MF_OPT_PACK_STRIPS = 2 asks for it wherever it
    is possible).  Packing changes where a column sits in LDS
    and nothing else: one launch per epoch and one launch per stratum with packed strips, the
    same with whole strips (MF_OPT_PACK_STRIPS = 0) and the kernel on Qt in memory must agree bit
    for bit, over three epochs (two of them with shuffled strata), and match the oracle."""
    ds = dataset("tiny")
    take = 5600
    rows, cols, vals = ds.rows[:take].copy(), ds.cols[:take].copy(), ds.vals[:take].copy()
    gr, gc = grid
    outs = []
    for kernel, ring, pack in (("lds", 1, 2), ("lds", 0, 2), ("lds", 1, 0), ("global", 0, 1)):
        which = mfmod.MF_KERNEL_LDS if kernel == "lds" else mfmod.MF_KERNEL_GLOBAL
        model = mfmod.MatrixFactorization(ds.cfg.m, ds.cfg.n, k, storage, seed=3, scale=0.1,
                                          options={mfmod.MF_OPT_DET_KERNEL: which, mfmod.MF_OPT_RING: ring,
                                                   mfmod.MF_OPT_PACK_STRIPS: pack})
        model.load_blocks(rows, cols, vals, gr, gc, 0)
        plan = model.epoch_plan(mfmod.MF_MODE_DET)
        if kernel == "lds":
            assert plan["kernel"] == ("sgd_ring_lds" if ring else "sgd_block_lds"), plan
            assert ("touched columns" in plan["note"]) == bool(pack), plan
        else:
            assert plan["kernel"] == "sgd_chunks", plan
        for epoch in range(3):
            order = oracle.stratum_order(5, epoch, gc) if epoch else None
            model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_DET, stratum_order=order)
        model.sync()
        outs.append(model.get_factors())
        model.close()
    for other in outs[1:]:
        assert np.array_equal(outs[0][0], other[0]) and np.array_equal(outs[0][1], other[1])
    arith = oracle.ARITH_F64 if storage == "f32" else oracle.ARITH_F16
    perm, bp, _, _ = oracle.partition(rows, cols, ds.cfg.m, ds.cfg.n, gr, gc, 0)
    Po, Qo = oracle_init(ds.cfg.m, ds.cfg.n, k, 3, 0.1, arith)
    for epoch in range(3):
        if epoch:
            oracle.sgd_epoch_ordered(Po, Qo, rows, cols, vals, perm, bp, gr, gc, 0.01, 0.05,
                                     oracle.stratum_order(5, epoch, gc), arith)
        else:
            oracle.sgd_epoch(Po, Qo, rows, cols, vals, perm, bp, gr, gc, 0.01, 0.05, arith)
    if storage == "f32":
        assert np.abs(outs[0][0] - Po).max() <= 1e-4 and np.abs(outs[0][1] - Qo).max() <= 1e-4
    else:
        differing = int((outs[0][0] != Po).sum() + (outs[0][1] != Qo).sum())
        assert differing <= max(1, int(1e-5 * (Po.size + Qo.size))), differing


def test_table_of_touched_columns_on_a_grid_of_millions_of_blocks(mfmod):
    """17.2 million blocks, 2.7 million of them with ratings: the kernel that makes the table of
    touched columns takes one workgroup per non-empty block and has to loop over the list (a
    launch dimension holds fewer than 2^32 threads: launched with one workgroup per block it
    left most of the table empty on 25 million blocks, and the packed kernels then skipped columns
    that have ratings).  The packed deterministic kernel must give the bits of the kernel that
    works on Qt in memory."""
    rng = np.random.default_rng(5)
    m, n, nnz, k = 4100, 42_000, 3_000_000, 32      # strips of 10 columns, one or two of them touched by a block
    rows = rng.integers(0, m, nnz).astype(np.int32)
    cols = rng.integers(0, n, nnz).astype(np.int32)
    vals = rng.uniform(1.0, 5.0, nnz).astype(np.float32)
    outs = []
    for which in (mfmod.MF_KERNEL_LDS, mfmod.MF_KERNEL_GLOBAL):
        model = mfmod.MatrixFactorization(m, n, k, "f32", seed=2, scale=0.1, options={mfmod.MF_OPT_DET_KERNEL: which})
        model.load_blocks(rows, cols, vals, 4100, 4200, 0)
        plan = model.epoch_plan(mfmod.MF_MODE_DET)
        if which == mfmod.MF_KERNEL_LDS:
            assert plan["kernel"] in ("sgd_ring_lds", "sgd_block_lds") and "touched columns" in plan["note"], plan
        model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_DET)
        model.sync()
        outs.append(model.get_factors())
        model.close()
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_lds_kernel_is_refused_when_the_strip_does_not_fit(mfmod):
    ds = dataset("tiny")
    model = _make(mfmod, ds, 256, "f32", 2, 2, 0, options={mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS})
    with pytest.raises(mfmod.MFError) as e:        # 500 columns * 256 * 4 B = 500 KiB > LDS
        model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_HOGWILD)
    assert e.value.code == mfmod.binding.MF_EINVAL
    model.close()
    # AUTO falls back to the kernel with atomics in L2 and still trains
    model = _make(mfmod, ds, 256, "f32", 2, 2, 0)
    before = model.rmse()
    model.sgd_epoch(0.01, 0.05, mfmod.MF_MODE_HOGWILD)
    assert model.rmse() < before
    model.close()


def test_tiny_config_hogwild_without_die_affinity_still_trains(mfmod):
    """Diagnostic mode MF_OPT_XCD_AFFINITY = 0: the chunks of one block run on all dies, whose
    private L2 caches do not see each other's updates inside a launch, so updates are lost and
    the 0.5 % band is not promised; the run must still be a valid, converging training."""
    ds = dataset("tiny")
    Po, Qo, _ = oracle_train(ds, 8, 8, 1, ds.cfg.epochs)
    want = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
    P0, Q0 = oracle_init(ds.cfg.m, ds.cfg.n, ds.cfg.k, 1, 0.1)
    start = oracle.rmse(P0, Q0, ds.test_rows, ds.test_cols, ds.test_vals)
    got = _train_gpu(mfmod, ds, ds.cfg.k, "f32", 8, 8, 1, mfmod.MF_MODE_HOGWILD, ds.cfg.epochs,
                     options={mfmod.MF_OPT_XCD_AFFINITY: 0, mfmod.MF_OPT_HOGWILD_CHUNK: 32,
                              mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_GLOBAL_ATOMICS})
    print("tiny HOGWILD (die affinity off): rmse gpu %.6f oracle %.6f start %.6f" % (got, want, start), flush=True)
    assert got < 0.25 * start and abs(got - want) <= 0.10 * want, (got, want, start)


# ------------------------------------------------------------------------------- error paths (forced from the host)
def test_error_codes(mfmod):
    b = mfmod.binding
    ctx = b.mf_create(0, torch.cuda.current_stream().cuda_stream)
    P = torch.empty((10, 32), device="cuda")
    Q = torch.empty((12, 32), device="cuda")
    with pytest.raises(mfmod.MFError) as e:
        b.mf_sgd_epoch(ctx, 0.1, 0.1, 0)                  # epoch before init/load
    assert e.value.code == b.MF_ESTATE
    with pytest.raises(mfmod.MFError) as e:
        b.mf_init(ctx, 10, 12, 48, 0, P.data_ptr(), Q.data_ptr(), 1, 0.1)   # k not supported
    assert e.value.code == b.MF_EINVAL
    with pytest.raises(mfmod.MFError) as e:
        b.mf_init(ctx, 10, 12, 32, 0, 0, Q.data_ptr(), 1, 0.1)              # null buffer
    assert e.value.code == b.MF_EINVAL
    b.mf_init(ctx, 10, 12, 32, 0, P.data_ptr(), Q.data_ptr(), 1, 0.1)
    rows = np.array([0, 3, 9], np.int32)
    cols = np.array([0, 5, 11], np.int32)
    vals = np.ones(3, np.float32)
    nbytes = b.mf_load_blocks_workspace(ctx, 3, 2, 2)
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) & ~255
    with pytest.raises(mfmod.MFError) as e:
        b.mf_load_blocks(ctx, rows, cols, vals, 2, 2, 0, base, nbytes - 1)  # workspace too small
    assert e.value.code == b.MF_ENOMEM
    with pytest.raises(mfmod.MFError) as e:
        b.mf_load_blocks(ctx, rows, cols, vals, 3, 2, 0, base, nbytes)      # grid_r > grid_c
    assert e.value.code == b.MF_EINVAL
    bad = cols.copy()
    bad[1] = 12
    with pytest.raises(mfmod.MFError) as e:
        b.mf_load_blocks(ctx, rows, bad, vals, 2, 2, 0, base, nbytes)       # column out of range
    assert e.value.code == b.MF_ERANGE
    with pytest.raises(mfmod.MFError) as e:
        b.mf_sgd_epoch(ctx, 0.1, 0.1, 0)                  # still nothing loaded
    assert e.value.code == b.MF_ESTATE
    b.mf_load_blocks(ctx, rows, cols, vals, 2, 2, 0, base, nbytes)
    with pytest.raises(mfmod.MFError) as e:
        b.mf_sgd_epoch(ctx, 0.1, 0.1, 5)                  # unknown mode
    assert e.value.code == b.MF_EINVAL
    b.mf_sgd_epoch(ctx, 0.1, 0.1, 0)
    b.mf_sync(ctx)
    b.mf_destroy(ctx)


def test_workgroups_are_dealt_round_robin_over_the_eight_dies(mfmod):
    # the placement MF_OPT_XCD_AFFINITY relies on: workgroup i of a launch runs on die i mod 8
    ctx = mfmod.binding.mf_create(0, torch.cuda.current_stream().cuda_stream)
    ids = mfmod.binding.mf_debug_xcc_ids(ctx, 4096)
    mfmod.binding.mf_destroy(ctx)
    assert set(ids.tolist()) == set(range(8))
    rel = (ids - ids[0]) % 8
    assert np.array_equal(rel, np.arange(4096) % 8)


# ------------------------------------------------------------------------------- configuration 2 (the benchmark workload)
def test_medium_config_scaled_det_and_hogwild(mfmod):
    ds = dataset("medium", 0.05)
    k = 128
    P, Q, Po, Qo = _det_one_epoch(mfmod, ds, k, "f32", 64, 64, 1)
    assert np.abs(P - Po).max() <= 1e-4 and np.abs(Q - Qo).max() <= 1e-4
    epochs = 5
    for gr, gc, which in [(8, 8, mfmod.MF_HOGWILD_GLOBAL_ATOMICS), (32, 32, mfmod.MF_HOGWILD_LDS)]:
        Po, Qo, _ = oracle_train(ds, gr, gc, 1, epochs)
        want = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
        got = _train_gpu(mfmod, ds, k, "f32", gr, gc, 1, mfmod.MF_MODE_HOGWILD, epochs,
                         options={mfmod.MF_OPT_HOGWILD_KERNEL: which})
        print("medium@0.05 HOGWILD kernel %d: rmse gpu %.6f oracle %.6f" % (which, got, want), flush=True)
        assert abs(got - want) <= 0.005 * want, (got, want)


def test_medium_config_full_size(mfmod):
    """Configuration 2 at its full size, in the launch configuration the benchmark times
    (HOGWILD, 256 x 256 grid, LDS kernel with the library's choice of wavefronts per workgroup, one launch per epoch,
    partitioned on the device) plus the deterministic mode on a fine grid."""
    ds = dataset("medium")
    k = ds.cfg.k
    print("medium: max row/col degree", ds.max_row_degree, ds.max_col_degree, flush=True)
    P, Q, Po, Qo = _det_one_epoch(mfmod, ds, k, "f32", 256, 256, 1)
    dP, dQ = np.abs(P - Po).max(), np.abs(Q - Qo).max()
    print("medium DET one epoch: max|dP| %.3g max|dQ| %.3g" % (dP, dQ), flush=True)
    assert dP <= 1e-4 and dQ <= 1e-4
    epochs = ds.cfg.epochs
    Po, Qo, _ = oracle_train(ds, 256, 256, 1, epochs)
    want = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
    model = mfmod.MatrixFactorization(ds.cfg.m, ds.cfg.n, k, "f32", seed=1, scale=0.1,
                                      options={mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS})
    dev = model.P.device
    model.load_blocks_device(*(torch.from_numpy(x).to(dev) for x in (ds.rows, ds.cols, ds.vals)), 256, 256, 1)
    tr, tc, tv = model.to_device(ds.test_rows, ds.test_cols, ds.test_vals)
    for _ in range(epochs):
        model.sgd_epoch(ds.cfg.lr, ds.cfg.lam, mfmod.MF_MODE_HOGWILD)
    got = model.rmse(tr, tc, tv)
    model.close()
    print("medium HOGWILD %d epochs: rmse gpu %.6f oracle %.6f" % (epochs, got, want), flush=True)
    assert abs(got - want) <= 0.005 * want, (got, want)
    got_det = _train_gpu(mfmod, ds, k, "f32", 8, 8, 1, mfmod.MF_MODE_DET, 1)
    Po, Qo, _ = oracle_train(ds, 8, 8, 1, 1)
    want_det = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
    assert abs(got_det - want_det) <= 1e-3, (got_det, want_det)


# ------------------------------------------------------------------------------- configurations 3, 4, 5 at reduced size, oracle run inside the test
OTHER = {
    # name: (scale for the default run, DET grid, HOGWILD grid, epochs for the default run)
    # The HOGWILD grids use the split that bounds a strip's width as well as its ratings, fine
    # enough for the widest column strip to fit the LDS (the LDS kernel is forced, so a strip that
    # does not fit is an error and not a silent change of kernel).
    "large": (0.02, (64, 64), (32, 32), 8),
    "xlarge": (0.01, (128, 128), (128, 512), 8),
    "stress": (0.005, (128, 128), (128, 512), 6),
}
# Initial factors are uniform in [0, this): 0.1 (the tiny configuration names it) except for the
# configuration whose ratings run from 0 to 100, where k * (scale / 2)^2 is the mean rating; from
# 0.1 the first epoch of Algorithm 1 on that input makes steps so large that no fp32 state stays
# within 1e-4 of the fp64 oracle (the oracle's own fp32 arithmetic does not), and at full size it
# diverges.
INIT_SCALE = {"large": 0.1, "xlarge": 1.25, "stress": 0.1}


def _config_case(mfmod, name, scale, det_grid, hog_grid, epochs, hog_split=2, storage=None):
    ds = dataset(name, scale)
    if storage is not None:
        import dataclasses
        ds.cfg = dataclasses.replace(ds.cfg, storage=storage)
    cfg = ds.cfg
    init = INIT_SCALE[name]
    print("%s: m=%d n=%d nnz=%d %s, max row/col degree %d/%d" % (cfg.name, cfg.m, cfg.n, ds.rows.size, cfg.storage,
                                                                  ds.max_row_degree, ds.max_col_degree), flush=True)
    P, Q, Po, Qo = _det_one_epoch(mfmod, ds, cfg.k, cfg.storage, det_grid[0], det_grid[1], 1, scale=init)
    dP, dQ = np.abs(P - Po).max(), np.abs(Q - Qo).max()
    print("%s DET one epoch: max|dP| %.3g max|dQ| %.3g (largest |P| %.3g |Q| %.3g)" % (
        cfg.name, dP, dQ, np.abs(Po).max(), np.abs(Qo).max()), flush=True)
    if cfg.storage == "f32":
        assert dP <= 1e-4 and dQ <= 1e-4, (dP, dQ)          # the stated bar, absolute
    else:
        for X, Xo in ((P, Po), (Q, Qo)):
            print("%s binary16: fraction of differing elements %.3g" % (cfg.name, np.mean(X != Xo)), flush=True)
            assert np.mean(X != Xo) <= 1e-5, float(np.mean(X != Xo))
    arith = _arith(cfg.storage)
    Po, Qo, _ = oracle_train(ds, hog_grid[0], hog_grid[1], hog_split, epochs, scale=init, arith=arith)
    want = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
    got = _train_gpu(mfmod, ds, cfg.k, cfg.storage, hog_grid[0], hog_grid[1], hog_split, mfmod.MF_MODE_HOGWILD,
                     epochs, options={mfmod.MF_OPT_HOGWILD_KERNEL: mfmod.MF_HOGWILD_LDS}, scale=init)
    print("%s HOGWILD %d epochs: rmse gpu %.6f oracle %.6f" % (cfg.name, epochs, got, want), flush=True)
    assert abs(got - want) <= 0.005 * want, (got, want)
    got_det = _train_gpu(mfmod, ds, cfg.k, cfg.storage, det_grid[0], det_grid[1], 1, mfmod.MF_MODE_DET, epochs, scale=init)
    Po, Qo, _ = oracle_train(ds, det_grid[0], det_grid[1], 1, epochs, scale=init, arith=arith)
    want_det = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
    print("%s DET %d epochs: rmse gpu %.6f oracle %.6f" % (cfg.name, epochs, got_det, want_det), flush=True)
    assert abs(got_det - want_det) <= 1e-3, (got_det, want_det)


@pytest.mark.parametrize("name", ["large", "xlarge", "stress"])
def test_other_configs_scaled(mfmod, name):
    scale, det_grid, hog_grid, epochs = OTHER[name]
    _config_case(mfmod, name, scale, det_grid, hog_grid, epochs)


# ------------------------------------------------------------------------------- binary16 storage against the DEFINITION
# The element-wise binary16 comparisons above are against the oracle's F16 arithmetic, whose fp32
# operation sequence is the kernel's.  These two tie the binary16 path to Algorithm 1 itself, i.e.
# to the oracle's F64 arithmetic: one step at a time (where the only freedom is the rounding), and
# over the epochs of the configuration that names binary16 storage.
def test_binary16_single_steps_round_the_fp64_definition(mfmod):
    """n independent ratings (rating i sits alone in row i and column i), one deterministic epoch on
    binary16 storage: every element of the result must be the binary16 neighbour of the exact
    (fp64) step of Algorithm 1 -- the nearest one, or, where the exact value lies within fp32
    rounding of a tie between two binary16 values, either of the two."""
    n, k = 4096, 128
    rng = np.random.Generator(np.random.Philox(77))
    rows = np.arange(n, dtype=np.int32)
    cols = rng.permutation(n).astype(np.int32)
    vals = rng.uniform(1.0, 5.0, n).astype(np.float32)
    P0 = rng.uniform(0.0, 0.5, (n, k)).astype(np.float16).astype(np.float64)
    Q0 = rng.uniform(0.0, 0.5, (n, k)).astype(np.float16).astype(np.float64)
    lr, lam = 0.01, 0.05
    for kernel in ("global", "lds"):
        model = mfmod.MatrixFactorization(n, n, k, "f16", seed=1, scale=-1.0, options=_det_options(mfmod, kernel))
        model.set_factors(P0, Q0)
        model.load_blocks(rows, cols, vals, 64, 64, 1)
        model.sgd_epoch(lr, lam, mfmod.MF_MODE_DET)
        P, Q = model.get_factors()
        model.close()
        Po, Qo = P0.copy(), Q0.copy()
        perm, bp, _, _ = oracle.partition(rows, cols, n, n, 64, 64, 1)
        oracle.sgd_epoch(Po, Qo, rows, cols, vals, perm, bp, 64, 64, lr, lam, oracle.ARITH_F64)
        for X, Xo in ((P, Po), (Q, Qo)):
            nearest = Xo.astype(np.float16).astype(np.float64)
            off = X != nearest
            ulp = np.spacing(np.abs(nearest).astype(np.float16)).astype(np.float64)
            # always within half a binary16 spacing of the exact value, up to the fp32 rounding of the
            # step's operands (all of magnitude below 1: two roundings of 2^-24 each) ...
            assert (np.abs(X - Xo) <= 0.5 * ulp + 2.0 ** -23).all()
            # ... and off the nearest value only at near-ties, which are rare
            print("binary16 single steps (%s): %d of %d elements are not the nearest binary16 value of the fp64 step"
                  % (kernel, int(off.sum()), off.size), flush=True)
            assert off.mean() <= 1e-3


def test_binary16_config_final_rmse_against_the_fp64_definition(mfmod):
    """Configuration 5 (binary16 storage) at the tested scale, all its epochs: the held-out RMSE
    of the deterministic GPU run against the oracle's F64 arithmetic (Algorithm 1 in double,
    nothing rounded to binary16), and against its F16 arithmetic for reference."""
    scale, det_grid, _, _ = OTHER["stress"]
    ds = dataset("stress", scale)
    cfg = ds.cfg
    epochs = cfg.epochs
    got = _train_gpu(mfmod, ds, cfg.k, "f16", det_grid[0], det_grid[1], 1, mfmod.MF_MODE_DET, epochs)
    P64, Q64, _ = oracle_train(ds, det_grid[0], det_grid[1], 1, epochs, arith=oracle.ARITH_F64)
    want64 = oracle.rmse(P64, Q64, ds.test_rows, ds.test_cols, ds.test_vals)
    P16, Q16, _ = oracle_train(ds, det_grid[0], det_grid[1], 1, epochs, arith=oracle.ARITH_F16)
    want16 = oracle.rmse(P16, Q16, ds.test_rows, ds.test_cols, ds.test_vals)
    print("stress@%g DET binary16, %d epochs: rmse gpu %.6f, oracle F64 %.6f, oracle F16 %.6f"
          % (scale, epochs, got, want64, want16), flush=True)
    assert abs(got - want16) <= 1e-3
    assert abs(got - want64) <= 1e-3


def test_binary16_hogwild_on_the_l2_atomics_kernel(mfmod):
    """The Hogwild fallback for grids whose strips do not fit the LDS adds binary16-rounded
    changes with packed atomics in the L2; configuration 5 at the tested scale, on a grid that
    forces it, has to stay inside the 0.5 % band as well."""
    scale, _, _, epochs = OTHER["stress"]
    ds = dataset("stress", scale)
    cfg = ds.cfg
    Po, Qo, _ = oracle_train(ds, 8, 8, 1, epochs, arith=oracle.ARITH_F16)
    want = oracle.rmse(Po, Qo, ds.test_rows, ds.test_cols, ds.test_vals)
    model = _make(mfmod, ds, cfg.k, "f16", 8, 8, 1)
    plan = model.epoch_plan(mfmod.MF_MODE_HOGWILD)
    assert plan["kernel"] == "sgd_chunks", plan          # MF_HOGWILD_AUTO says which kernel it took, and why
    assert "exceeds" in plan["note"]
    tr, tc, tv = model.to_device(ds.test_rows, ds.test_cols, ds.test_vals)
    for _ in range(epochs):
        model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_HOGWILD)
    got = model.rmse(tr, tc, tv)
    model.close()
    print("stress@%g HOGWILD on the L2-atomics kernel, %d epochs: rmse gpu %.6f oracle %.6f" % (scale, epochs, got, want),
          flush=True)
    assert abs(got - want) <= 0.005 * want


@pytest.mark.parametrize("name", ["large", "xlarge"])
def test_binary16_storage_on_the_fp32_configs(mfmod, name):
    """Half-precision storage is an option for every configuration, not only the one that names it."""
    scale, det_grid, hog_grid, epochs = OTHER[name]
    _config_case(mfmod, name, scale, det_grid, hog_grid, epochs, storage="f16")


# ------------------------------------------------------------------------------- configs 3, 4 and 5 at full size
# The CPU oracle needs minutes to an hour on these, so its results are stored by
# tests/golden/make_full_size_expected.py (which calls only the oracle and the input generators):
# the held-out RMSE after every epoch and, after the first epoch, whole rows of P and Qt at 48 + 48
# sampled indices plus the element sum of every group of 64 consecutive rows of both factors (so
# that every row is covered).  Grid, split rule and initial scale are the ones bench.py times.
STORED = ("large", "xlarge", "stress")


def _read_stored(name):
    path = os.path.join(os.path.dirname(__file__), "golden", f"full_{name}.txt")
    if not os.path.exists(path):
        return None
    out = {"P": {}, "Q": {}}
    with open(path) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            if key[0] in "PQ" and key[1:].isdigit():
                out[key[0]][int(key[1:])] = np.array([float.fromhex(v) for v in vals])
            else:
                out[key] = vals
    sums = os.path.join(os.path.dirname(__file__), "golden", f"full_{name}_groupsums.npy")
    out["groupsums"] = np.load(sums) if os.path.exists(sums) else None
    return out


def _group_sums(X, group):
    """Element sum of every `group` consecutive rows of a device matrix, in double, on the device."""
    row = X.double().sum(dim=1)
    pad = (-row.numel()) % group
    if pad:
        row = torch.cat([row, torch.zeros(pad, dtype=row.dtype, device=row.device)])
    return row.view(-1, group).sum(dim=1).cpu().numpy()


@pytest.mark.parametrize("name", STORED)
def test_full_size_against_the_stored_oracle_results(mfmod, name):
    import time
    import workloads
    g = _read_stored(name)
    if g is None:
        pytest.skip("no stored oracle results for this configuration")
    if int(g["recipe"][0]) != workloads.RECIPE:
        pytest.fail("the stored oracle results were made from another recipe of the input generator")
    t0 = time.perf_counter()
    ds = workloads.load(name, keep=False)
    cfg = ds.cfg
    gr, gc = int(g["grid"][0]), int(g["grid"][1])
    split, scale, group = int(g["split"][0]), float(g["init_scale"][0]), int(g["group"][0])
    want_rmse = [float(x) for x in g["rmse"]]
    assert int(g["nnz_train"][0]) == ds.rows.size
    dev = torch.device("cuda:0")
    coo = [torch.from_numpy(x).to(dev) for x in (ds.rows, ds.cols, ds.vals)]
    test = [torch.from_numpy(x).to(dev) for x in (ds.test_rows, ds.test_cols, ds.test_vals)]
    del ds
    print(f"{name}: data generated and on the device after {time.perf_counter() - t0:.1f} s", flush=True)

    # deterministic mode: sampled rows and group sums after one epoch, RMSE after one and after all stored epochs
    model = mfmod.MatrixFactorization(cfg.m, cfg.n, cfg.k, cfg.storage, seed=1, scale=scale)
    model.load_blocks_device(coo[0], coo[1], coo[2], gr, gc, split)
    print(f"{name} " + model.epoch_plan(mfmod.MF_MODE_DET)["note"], flush=True)
    model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_DET)
    for tag, X in (("P", model.P), ("Q", model.Qt)):
        ids = sorted(g[tag])
        got = X[torch.tensor(ids, device=dev)].float().cpu().numpy().astype(np.float64)
        want = np.stack([g[tag][i] for i in ids])
        if cfg.storage == "f16":
            differing = int((got != want).sum())
            print(f"{name} DET epoch 1, {tag}: {differing} of {want.size} sampled elements differ", flush=True)
            assert differing <= max(1, int(1e-5 * want.size))
        else:
            err = np.abs(got - want)
            rel = err / np.maximum(1.0, np.abs(want))
            print(f"{name} DET epoch 1, {tag}: max error {err.max():.3g} absolute, {rel.max():.3g} relative to "
                  f"max(1, |x|), on {len(ids)} sampled rows (largest |x| {np.abs(want).max():.3g})", flush=True)
            assert err.max() <= 1e-4          # the absolute bar, also where factors reach 8 (ratings 0..100)
    if g["groupsums"] is not None:
        got = np.concatenate([_group_sums(model.P, group), _group_sums(model.Qt, group)])
        diff = np.abs(got - g["groupsums"])
        if cfg.storage == "f16":
            # equal elements give equal sums up to the rounding of the two summation orders
            off = int((diff > 1e-7).sum())
            print(f"{name} DET epoch 1: {off} of {diff.size} groups of {group} rows differ in their sum", flush=True)
            assert off <= max(1, int(1e-5 * diff.size * group * cfg.k))
        else:
            # every element within the bar and errors of random sign: sqrt(elements) times the bar
            bound = 1e-4 * np.sqrt(group * cfg.k)
            print(f"{name} DET epoch 1: largest difference of a {group}-row group sum {diff.max():.3g} "
                  f"(bound {bound:.3g}, {diff.size} groups = every row of P and Qt)", flush=True)
            assert diff.max() <= bound
    got = model.rmse(*test)
    print(f"{name} DET epoch 1: rmse gpu {got:.6f} oracle {want_rmse[0]:.6f}", flush=True)
    assert abs(got - want_rmse[0]) <= 1e-3
    # further deterministic epochs, as many as a minute allows (the grid was made for the Hogwild
    # mode: the deterministic one runs on its fallback kernel here); the oracle's held-out RMSE is
    # stored after every epoch
    t0 = time.perf_counter()
    done = 1
    while done < len(want_rmse):
        model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_DET)
        model.sync()
        done += 1
        spent = time.perf_counter() - t0
        if spent + spent / (done - 1) > 60.0:
            break
    got = model.rmse(*test)
    print(f"{name} DET {done} of {len(want_rmse)} epochs: rmse gpu {got:.6f} oracle {want_rmse[done - 1]:.6f} "
          f"({time.perf_counter() - t0:.1f} s)", flush=True)
    assert abs(got - want_rmse[done - 1]) <= 1e-3
    model.close()

    # Hogwild mode as bench.py runs it (kernel and wavefronts per workgroup: the library's choice)
    model = mfmod.MatrixFactorization(cfg.m, cfg.n, cfg.k, cfg.storage, seed=1, scale=scale)
    model.load_blocks_device(coo[0], coo[1], coo[2], gr, gc, split)
    plan = model.epoch_plan(mfmod.MF_MODE_HOGWILD)
    print(f"{name} " + plan["note"], flush=True)
    assert plan["kernel"] == "sgd_ring_lds"
    model.sync()
    t0 = time.perf_counter()
    for e in range(len(want_rmse)):
        model.sgd_epoch(cfg.lr, cfg.lam, mfmod.MF_MODE_HOGWILD)
    model.sync()
    dt = time.perf_counter() - t0
    got = model.rmse(*test)
    print(f"{name} HOGWILD {len(want_rmse)} epochs: rmse gpu {got:.6f} oracle {want_rmse[-1]:.6f}; "
          f"{cfg.nnz_train * len(want_rmse) / dt / 1e9:.3f} G updates/s", flush=True)
    assert abs(got - want_rmse[-1]) <= 5e-3 * want_rmse[-1]
    model.close()
