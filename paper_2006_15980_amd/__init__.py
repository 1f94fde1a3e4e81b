"""MI355X-native SGD matrix factorization (hot path of arxiv 2006.15980's method).

``binding`` mirrors the C ABI of include/mf_sgd.h one to one.  ``MatrixFactorization`` is a
small convenience holder that keeps the torch tensors (device memory) alive next to the
library context; every step of the method runs inside libmf_sgd.so.
"""
from __future__ import annotations

import numpy as np

from . import binding
from .binding import *  # noqa: F401,F403
from .binding import (MF_F16, MF_F32, MF_KERNEL_AUTO, MF_KERNEL_GLOBAL, MF_KERNEL_LDS, MF_OPT_DET_KERNEL, MF_OPT_RING, MF_OPT_RING_SPIN_LIMIT, MF_OPT_LDS_PREFETCH, MF_OPT_ROW_ORDER_SEED, MF_OPT_PACK_STRIPS, MF_HOGWILD_AUTO, MF_HOGWILD_GLOBAL_ATOMICS, MF_HOGWILD_LDS, MF_MODE_DET,
                      MF_MODE_HOGWILD, MF_OPT_HOGWILD_CHUNK, MF_OPT_HOGWILD_KERNEL, MF_OPT_LDS_CHUNK,
                      MF_OPT_LDS_WAVES, MF_OPT_PROFILE, MF_OPT_XCD_AFFINITY, MF_PLAN_HOGWILD_LDS, MF_PLAN_LDS_CUT_ROWS,
                      MF_SPLIT_EQUAL_WIDTH, MF_SPLIT_NNZ_BALANCED, MF_SPLIT_NNZ_WIDTH_BALANCED, MFError)


class MatrixFactorization:
    """Owns the device buffers (torch tensors) and a library context on the current stream."""

    def __init__(self, m: int, n: int, k: int, storage: str = "f32", device: int = 0, seed: int = 1,
                 scale: float = 0.1, options: dict | None = None):
        import torch

        if not torch.cuda.is_available():
            raise RuntimeError("no HIP device: the library has no CPU path")
        self.torch = torch
        self.m, self.n, self.k = m, n, k
        self.dtype = {"f32": MF_F32, "f16": MF_F16}[storage]
        tdt = torch.float32 if self.dtype == MF_F32 else torch.float16
        self.dev = torch.device("cuda", device)
        with torch.cuda.device(self.dev):
            self.stream = torch.cuda.current_stream().cuda_stream
        self.ctx = binding.mf_create(device, self.stream)
        for key, val in (options or {}).items():
            binding.mf_set_option(self.ctx, key, val)
        self.P = torch.empty((m, k), dtype=tdt, device=self.dev)
        self.Qt = torch.empty((n, k), dtype=tdt, device=self.dev)
        binding.mf_init(self.ctx, m, n, k, self.dtype, self.P.data_ptr(), self.Qt.data_ptr(), seed, scale)
        self.workspace = None
        self.nnz = 0
        self.grid = (0, 0)

    def set_factors(self, P: np.ndarray, Qt: np.ndarray):
        t = self.torch
        self.P.copy_(t.from_numpy(np.ascontiguousarray(P)).to(self.P.dtype))
        self.Qt.copy_(t.from_numpy(np.ascontiguousarray(Qt)).to(self.Qt.dtype))

    def get_factors(self):
        return self.P.float().cpu().numpy().astype(np.float64), self.Qt.float().cpu().numpy().astype(np.float64)

    def load_blocks(self, rows, cols, vals, grid_r: int, grid_c: int, split: int = MF_SPLIT_NNZ_BALANCED):
        t = self.torch
        nbytes = binding.mf_load_blocks_workspace(self.ctx, rows.size, grid_r, grid_c)
        binding.mf_sync(self.ctx)
        self.workspace = t.empty(nbytes + 256, dtype=t.uint8, device=self.dev)
        base = (self.workspace.data_ptr() + 255) & ~255
        binding.mf_load_blocks(self.ctx, rows, cols, vals, grid_r, grid_c, split, base, nbytes)
        self.nnz = rows.size
        self.grid = (grid_r, grid_c)

    def load_blocks_streamed(self, rows, cols, vals, grid_r: int, grid_c: int, split: int = MF_SPLIT_NNZ_BALANCED):
        """The ratings stay in pinned host memory and are streamed to the device every epoch."""
        t = self.torch
        nbytes = binding.mf_load_blocks_streamed_workspace(self.ctx, rows.size, grid_r, grid_c)
        binding.mf_sync(self.ctx)
        self.workspace = t.empty(nbytes + 256, dtype=t.uint8, device=self.dev)
        base = (self.workspace.data_ptr() + 255) & ~255
        binding.mf_load_blocks_streamed(self.ctx, rows, cols, vals, grid_r, grid_c, split, base, nbytes)
        self.nnz = rows.size
        self.grid = (grid_r, grid_c)

    def load_blocks_device(self, rows, cols, vals, grid_r: int, grid_c: int, split: int = MF_SPLIT_NNZ_BALANCED):
        """rows, cols (int32) and vals (float32): torch tensors on this model's device."""
        t = self.torch
        for x, dt in ((rows, t.int32), (cols, t.int32), (vals, t.float32)):
            if x.dtype != dt or x.device != self.P.device or not x.is_contiguous() or x.numel() != rows.numel():
                raise ValueError("need contiguous int32 / int32 / float32 tensors of one length on the model's device")
        nbytes = binding.mf_load_blocks_workspace(self.ctx, rows.numel(), grid_r, grid_c)
        binding.mf_sync(self.ctx)
        self.workspace = t.empty(nbytes + 256, dtype=t.uint8, device=self.dev)
        base = (self.workspace.data_ptr() + 255) & ~255
        binding.mf_load_blocks_device(self.ctx, rows.data_ptr(), cols.data_ptr(), vals.data_ptr(), rows.numel(),
                                      grid_r, grid_c, split, base, nbytes)
        self.nnz = rows.numel()
        self.grid = (grid_r, grid_c)

    def partition(self):
        return binding.mf_get_partition(self.ctx, self.nnz, *self.grid)

    def sgd_epoch(self, lr: float, lam: float, mode: int, stratum_order=None):
        if stratum_order is None:
            binding.mf_sgd_epoch(self.ctx, lr, lam, mode)
        else:
            if len(stratum_order) != self.grid[1]:
                raise ValueError("stratum_order needs grid_c entries")
            binding.mf_sgd_epoch_ordered(self.ctx, lr, lam, mode, np.ascontiguousarray(stratum_order, np.int32))

    def sgd_epochs(self, lr: float, lam: float, mode: int, n_epochs: int):
        """n_epochs epochs in natural order; one launch where an epoch is one launch (mf_sgd_epochs)."""
        binding.mf_sgd_epochs(self.ctx, lr, lam, mode, n_epochs)

    def epoch_plan(self, mode: int) -> dict:
        """What sgd_epoch(mode) launches on the loaded grid (mf_epoch_plan)."""
        kernel, launches, waves, note = binding.mf_epoch_plan(self.ctx, mode)
        return {"kernel": binding.KERNEL_NAMES[kernel], "launches": launches, "waves": waves, "note": note}

    def rmse(self, rows=None, cols=None, vals=None) -> float:
        if rows is None:
            return binding.mf_rmse(self.ctx, None, None, None, 0)
        return binding.mf_rmse(self.ctx, rows.data_ptr(), cols.data_ptr(), vals.data_ptr(), rows.numel())

    def to_device(self, rows, cols, vals):
        t = self.torch
        return (t.from_numpy(rows).to(self.dev), t.from_numpy(cols).to(self.dev), t.from_numpy(vals).to(self.dev))

    def sync(self):
        binding.mf_sync(self.ctx)

    def close(self):
        if self.ctx:
            binding.mf_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
