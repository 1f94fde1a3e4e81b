"""The entry point that allocates nothing (mf_rmse_noalloc) against mf_rmse, through the C ABI.

Two calls in a row on one context, the second over a smaller input: the static scratch array still
holds the first call's partial sums then, and the result must not depend on them.  Bar: the RMSE
kernel's (relative 1e-9 against the fp64 oracle for mf_rmse); the two entry points run the same
kernels in the same order, so they are compared much more tightly here.
"""
import numpy as np
import pytest

from tests.util import dataset

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("storage", ["f32", "f16"])
def test_rmse_noalloc_matches_mf_rmse_on_two_calls_in_a_row(storage):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import oracle
    import paper_2006_15980_amd as mf

    B = mf.binding
    B.lib()
    ds = dataset("tiny")
    cfg = ds.cfg
    model = mf.MatrixFactorization(cfg.m, cfg.n, cfg.k, storage, seed=7, scale=0.4)
    model.load_blocks(ds.rows, ds.cols, ds.vals, 8, 8, mf.MF_SPLIT_NNZ_BALANCED)
    model.sgd_epoch(cfg.lr, cfg.lam, mf.MF_MODE_DET)
    tr, tc, tv = model.to_device(ds.test_rows, ds.test_cols, ds.test_vals)
    out = torch.full((2,), -1.0, dtype=torch.float64, device=model.P.device)
    small = 1234                                   # second call: fewer entries, and a ragged tail
    want_full = model.rmse(tr, tc, tv)
    want_small = model.rmse(tr[:small].contiguous(), tc[:small].contiguous(), tv[:small].contiguous())
    B.mf_rmse_noalloc(model.ctx, tr.data_ptr(), tc.data_ptr(), tv.data_ptr(), tr.numel(), out.data_ptr())
    B.mf_rmse_noalloc(model.ctx, tr.data_ptr(), tc.data_ptr(), tv.data_ptr(), small, out.data_ptr() + 8)
    model.sync()
    got_full, got_small = (float(x) for x in out.cpu())
    assert abs(got_full - want_full) <= 1e-12 * want_full, (got_full, want_full)
    assert abs(got_small - want_small) <= 1e-12 * want_small, (got_small, want_small)
    assert got_small != got_full
    # and the oracle, to the RMSE kernel's own bar
    P, Q = model.get_factors()
    ref = oracle.rmse(P, Q, ds.test_rows[:small], ds.test_cols[:small], ds.test_vals[:small])
    assert abs(got_small - ref) <= 1e-9 * ref, (got_small, ref)
    # sizes beyond the stated maximum and missing arrays are refused without touching the device
    with pytest.raises(mf.MFError) as err:
        B.mf_rmse_noalloc(model.ctx, tr.data_ptr(), tc.data_ptr(), tv.data_ptr(), (1 << 32) + 1, out.data_ptr())
    assert err.value.code == B.MF_EINVAL and "MAX_COUNT" in str(err.value)
    with pytest.raises(mf.MFError):
        B.mf_rmse_noalloc(model.ctx, None, tc.data_ptr(), tv.data_ptr(), 10, out.data_ptr())
    model.close()
