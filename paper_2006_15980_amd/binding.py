"""ctypes binding of libmf_sgd.so: argument marshalling only.

Every function has the name and the argument order of its C declaration in
include/mf_sgd.h; all arithmetic of the method runs in the library's HIP kernels.
Device buffers are passed as integer addresses (torch ``tensor.data_ptr()``), host
arrays as C-contiguous numpy arrays.  A negative return code raises ``MFError``.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

MF_OK, MF_EINVAL, MF_ESTATE, MF_ENOMEM, MF_EDEVICE, MF_ERANGE = 0, -1, -2, -3, -4, -5
MF_F32, MF_F16 = 0, 1
MF_MODE_DET, MF_MODE_HOGWILD = 0, 1
MF_SPLIT_EQUAL_WIDTH, MF_SPLIT_NNZ_BALANCED, MF_SPLIT_NNZ_WIDTH_BALANCED = 0, 1, 2
MF_OPT_HOGWILD_CHUNK, MF_OPT_XCD_AFFINITY, MF_OPT_PROFILE = 1, 2, 3
MF_OPT_HOGWILD_KERNEL, MF_OPT_LDS_CHUNK, MF_OPT_LDS_WAVES = 4, 5, 6
MF_OPT_DET_KERNEL = 7
MF_OPT_RING, MF_OPT_RING_SPIN_LIMIT, MF_OPT_LDS_PREFETCH, MF_OPT_ROW_ORDER_SEED = 8, 9, 10, 11
MF_OPT_PACK_STRIPS = 12
MF_KERNEL_AUTO, MF_KERNEL_GLOBAL, MF_KERNEL_LDS = 0, 1, 2
MF_HOGWILD_AUTO, MF_HOGWILD_GLOBAL_ATOMICS, MF_HOGWILD_LDS = 0, 1, 2
MF_PLAN_HOGWILD_LDS = 2
MF_PLAN_LDS_CUT_ROWS = 3
MF_KERNEL_ID_CHUNKS, MF_KERNEL_ID_BLOCK_LDS, MF_KERNEL_ID_RING_LDS = 1, 2, 3
KERNEL_NAMES = {MF_KERNEL_ID_CHUNKS: "sgd_chunks", MF_KERNEL_ID_BLOCK_LDS: "sgd_block_lds",
                MF_KERNEL_ID_RING_LDS: "sgd_ring_lds"}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmf_sgd.so")

EXPORTS = ["mf_create", "mf_destroy", "mf_last_error", "mf_set_option", "mf_init",
           "mf_load_blocks_workspace", "mf_load_blocks", "mf_load_blocks_device",
           "mf_load_blocks_streamed_workspace", "mf_load_blocks_streamed", "mf_get_partition", "mf_sgd_epoch",
           "mf_sgd_epoch_ordered", "mf_sgd_epochs", "mf_stratum_order", "mf_epoch_plan",
           "mf_rmse", "mf_rmse_noalloc", "mf_sync", "mf_profile_read", "mf_debug_xcc_ids", "mf_plan_host", "mf_suggest_grid"]


class MFError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libmf_sgd error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Load the HIP library; there is no fallback if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        l = C.CDLL(LIB_PATH)
        vp, i32, i64, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float
        l.mf_create.argtypes = [C.POINTER(vp), C.c_int, vp]
        l.mf_destroy.argtypes = [vp]
        l.mf_last_error.argtypes = [vp]
        l.mf_last_error.restype = C.c_char_p
        l.mf_set_option.argtypes = [vp, i32, i64]
        l.mf_init.argtypes = [vp, i64, i64, i32, i32, vp, vp, u64, f32]
        l.mf_load_blocks_workspace.argtypes = [vp, i64, i32, i32, C.POINTER(C.c_size_t)]
        l.mf_load_blocks.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, vp, C.c_size_t]
        l.mf_load_blocks_device.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, vp, C.c_size_t]
        l.mf_load_blocks_streamed_workspace.argtypes = [vp, i64, i32, i32, C.POINTER(C.c_size_t)]
        l.mf_load_blocks_streamed.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, vp, C.c_size_t]
        l.mf_get_partition.argtypes = [vp, vp, vp, vp, vp]
        l.mf_sgd_epoch.argtypes = [vp, f32, f32, i32]
        l.mf_sgd_epoch_ordered.argtypes = [vp, f32, f32, i32, vp]
        l.mf_sgd_epochs.argtypes = [vp, f32, f32, i32, i32]
        l.mf_epoch_plan.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i64), C.POINTER(i32)]
        l.mf_stratum_order.argtypes = [C.c_uint64, C.c_uint64, i32, vp]
        l.mf_rmse.argtypes = [vp, vp, vp, vp, i64, C.POINTER(C.c_double)]
        l.mf_rmse_noalloc.argtypes = [vp, vp, vp, vp, i64, vp]
        l.mf_sync.argtypes = [vp]
        l.mf_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
        l.mf_debug_xcc_ids.argtypes = [vp, i32, vp]
        l.mf_suggest_grid.argtypes = [i64, i64, i64, i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        l.mf_plan_host.argtypes = [vp, vp, i64, i64, i64, i32, i32, i32, i32, i32, i32,
                                   vp, vp, vp, vp, vp, vp, i64, vp, C.POINTER(i64)]
        for name in EXPORTS:
            if name != "mf_last_error":
                getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


def _host(a: Optional[np.ndarray], dtype) -> Optional[int]:
    if a is None:
        return None
    if not (isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous):
        raise TypeError(f"expected a C-contiguous numpy array of {np.dtype(dtype)}")
    return a.ctypes.data


def _check(ctx, rc: int):
    if rc != MF_OK:
        msg = lib().mf_last_error(ctx).decode() if ctx else "no context"
        raise MFError(rc, msg)


def mf_create(device: int = 0, hip_stream: int = 0) -> int:
    out = C.c_void_p()
    rc = lib().mf_create(C.byref(out), device, C.c_void_p(hip_stream))
    if rc != MF_OK:
        raise MFError(rc, "mf_create failed (no usable HIP device?)")
    return out.value


def mf_destroy(ctx: int) -> None:
    _check(None, lib().mf_destroy(ctx))


def mf_last_error(ctx: int) -> str:
    return lib().mf_last_error(ctx).decode()


def mf_set_option(ctx: int, option: int, value: int) -> None:
    _check(ctx, lib().mf_set_option(ctx, option, value))


def mf_init(ctx: int, m: int, n: int, k: int, dtype: int, dP: int, dQt: int, seed: int, scale: float) -> None:
    _check(ctx, lib().mf_init(ctx, m, n, k, dtype, dP, dQt, seed, scale))


def mf_load_blocks_workspace(ctx: int, nnz: int, grid_r: int, grid_c: int) -> int:
    out = C.c_size_t()
    _check(ctx, lib().mf_load_blocks_workspace(ctx, nnz, grid_r, grid_c, C.byref(out)))
    return out.value


def mf_load_blocks(ctx: int, rows: np.ndarray, cols: np.ndarray, vals: np.ndarray, grid_r: int, grid_c: int,
                   split: int, d_workspace: int, workspace_bytes: int) -> None:
    nnz = rows.size
    if cols.size != nnz or vals.size != nnz:
        raise ValueError("rows, cols and vals must have the same length")
    _check(ctx, lib().mf_load_blocks(ctx, _host(rows, np.int32), _host(cols, np.int32), _host(vals, np.float32),
                                     nnz, grid_r, grid_c, split, d_workspace, workspace_bytes))


def mf_load_blocks_streamed_workspace(ctx: int, nnz: int, grid_r: int, grid_c: int) -> int:
    out = C.c_size_t()
    _check(ctx, lib().mf_load_blocks_streamed_workspace(ctx, nnz, grid_r, grid_c, C.byref(out)))
    return out.value


def mf_load_blocks_streamed(ctx: int, rows: np.ndarray, cols: np.ndarray, vals: np.ndarray, grid_r: int, grid_c: int,
                            split: int, d_workspace: int, workspace_bytes: int) -> None:
    nnz = rows.size
    if cols.size != nnz or vals.size != nnz:
        raise ValueError("rows, cols and vals must have the same length")
    _check(ctx, lib().mf_load_blocks_streamed(ctx, _host(rows, np.int32), _host(cols, np.int32),
                                              _host(vals, np.float32), nnz, grid_r, grid_c, split, d_workspace,
                                              workspace_bytes))


def mf_load_blocks_device(ctx: int, d_rows: int, d_cols: int, d_vals: int, nnz: int, grid_r: int, grid_c: int,
                          split: int, d_workspace: int, workspace_bytes: int) -> None:
    """d_rows, d_cols, d_vals: device addresses of int32 / int32 / float32 arrays of nnz entries."""
    _check(ctx, lib().mf_load_blocks_device(ctx, d_rows, d_cols, d_vals, nnz, grid_r, grid_c, split, d_workspace,
                                            workspace_bytes))


def mf_get_partition(ctx: int, nnz: int, grid_r: int, grid_c: int):
    perm = np.empty(nnz, np.int64)
    bp = np.empty(grid_r * grid_c + 1, np.int64)
    rb = np.empty(grid_r + 1, np.int32)
    cb = np.empty(grid_c + 1, np.int32)
    _check(ctx, lib().mf_get_partition(ctx, perm.ctypes.data, bp.ctypes.data, rb.ctypes.data, cb.ctypes.data))
    return perm, bp, rb, cb


def mf_sgd_epoch(ctx: int, lr: float, lam: float, mode: int) -> None:
    _check(ctx, lib().mf_sgd_epoch(ctx, lr, lam, mode))


def mf_sgd_epochs(ctx: int, lr: float, lam: float, mode: int, n_epochs: int) -> None:
    _check(ctx, lib().mf_sgd_epochs(ctx, lr, lam, mode, n_epochs))


def mf_sgd_epoch_ordered(ctx: int, lr: float, lam: float, mode: int, stratum_order: Optional[np.ndarray]) -> None:
    order = None if stratum_order is None else _host(stratum_order, np.int32)
    _check(ctx, lib().mf_sgd_epoch_ordered(ctx, lr, lam, mode, order))


def mf_epoch_plan(ctx: int, mode: int):
    """-> (kernel id, launches per epoch, wavefronts per workgroup, the library's description)"""
    kernel, launches, waves = C.c_int32(), C.c_int64(), C.c_int32()
    _check(ctx, lib().mf_epoch_plan(ctx, mode, C.byref(kernel), C.byref(launches), C.byref(waves)))
    return kernel.value, launches.value, waves.value, lib().mf_last_error(ctx).decode()


def mf_stratum_order(seed: int, epoch: int, grid_c: int) -> np.ndarray:
    out = np.empty(grid_c, np.int32)
    rc = lib().mf_stratum_order(seed, epoch, grid_c, out.ctypes.data)
    if rc != MF_OK:
        raise MFError(rc, "mf_stratum_order failed")
    return out


def mf_rmse(ctx: int, d_rows: Optional[int], d_cols: Optional[int], d_vals: Optional[int], count: int) -> float:
    out = C.c_double()
    _check(ctx, lib().mf_rmse(ctx, d_rows, d_cols, d_vals, count, C.byref(out)))
    return out.value


def mf_rmse_noalloc(ctx: int, d_rows: int, d_cols: int, d_vals: int, count: int, d_rmse_out: int) -> None:
    """Enqueue only: the result lands in the device double at d_rmse_out."""
    _check(ctx, lib().mf_rmse_noalloc(ctx, d_rows, d_cols, d_vals, count, d_rmse_out))


def mf_sync(ctx: int) -> None:
    _check(ctx, lib().mf_sync(ctx))


def mf_profile_read(ctx: int):
    ms = C.c_double()
    cnt = C.c_int64()
    _check(ctx, lib().mf_profile_read(ctx, C.byref(ms), C.byref(cnt)))
    return ms.value, cnt.value


def mf_debug_xcc_ids(ctx: int, n_groups: int) -> np.ndarray:
    out = np.empty(n_groups, np.int32)
    _check(ctx, lib().mf_debug_xcc_ids(ctx, n_groups, out.ctypes.data))
    return out


def mf_suggest_grid(m: int, n: int, nnz: int, k: int, mode: int):
    """-> (grid_r, grid_c, split)"""
    gr, gc, sp = C.c_int32(), C.c_int32(), C.c_int32()
    rc = lib().mf_suggest_grid(m, n, nnz, k, mode, C.byref(gr), C.byref(gc), C.byref(sp))
    if rc != MF_OK:
        raise MFError(rc, "mf_suggest_grid failed")
    return gr.value, gc.value, sp.value


def mf_plan_host(rows: np.ndarray, cols: np.ndarray, m: int, n: int, grid_r: int, grid_c: int, split: int,
                 mode: int, chunk: int = 128, xcd_affinity: int = 1):
    """-> dict(perm, block_ptr, row_bounds, col_bounds, entry_begin, entry_len, stratum_entry)."""
    nnz = rows.size
    perm = np.empty(nnz, np.int64)
    bp = np.empty(grid_r * grid_c + 1, np.int64)
    rb = np.empty(grid_r + 1, np.int32)
    cb = np.empty(grid_c + 1, np.int32)
    se = np.empty(grid_c + 1, np.int64)
    n_entries = C.c_int64()
    rc = lib().mf_plan_host(_host(rows, np.int32), _host(cols, np.int32), nnz, m, n, grid_r, grid_c, split, mode,
                            chunk, xcd_affinity, perm.ctypes.data, bp.ctypes.data, rb.ctypes.data, cb.ctypes.data,
                            None, None, 0, se.ctypes.data, C.byref(n_entries))
    if rc != MF_OK:
        raise MFError(rc, "mf_plan_host failed")
    eb = np.empty(n_entries.value, np.int64)
    el = np.empty(n_entries.value, np.int32)
    rc = lib().mf_plan_host(_host(rows, np.int32), _host(cols, np.int32), nnz, m, n, grid_r, grid_c, split, mode,
                            chunk, xcd_affinity, None, None, None, None, eb.ctypes.data, el.ctypes.data,
                            n_entries.value, None, None)
    if rc != MF_OK:
        raise MFError(rc, "mf_plan_host failed")
    return dict(perm=perm, block_ptr=bp, row_bounds=rb, col_bounds=cb, entry_begin=eb, entry_len=el,
                stratum_entry=se)
