"""ctypes binding of libsgap.so: argument marshalling only.

Function names mirror the C ABI in include/sgap.h.  Tensors are torch CUDA
tensors (used purely as device memory); every computation happens in the HIP
kernels of the library.  There is no fallback: if the shared library is not
built, or a tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsgap.so")

SGAP_OK = 0
SGAP_ERR_INVALID_ARG = 1
SGAP_ERR_UNSUPPORTED = 2
SGAP_ERR_HIP = 3

SGAP_REDUCE_PARALLEL = 0
SGAP_REDUCE_SERIAL = 1
SGAP_SCHED_ROW_SPLIT = 0
SGAP_SCHED_NNZ_BALANCED = 1

STRATEGIES = {"parallel": SGAP_REDUCE_PARALLEL, "serial": SGAP_REDUCE_SERIAL}
SCHEDULES = {"row_split": SGAP_SCHED_ROW_SPLIT, "nnz_balanced": SGAP_SCHED_NNZ_BALANCED}
STRATEGY_NAMES = {v: k for k, v in STRATEGIES.items()}
SCHEDULE_NAMES = {v: k for k, v in SCHEDULES.items()}
GROUP_SIZES = (1, 2, 4, 8, 16, 32, 64)

# every symbol include/sgap.h and include/sgap_debug.h declare: name -> (restype, argtypes)
_i64, _int, _p = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
EXPORTS = {
    "sgap_set_schedule": (_int, [_int]),
    "sgap_get_schedule": (_int, []),
    "sgap_spmm_csr": (_int, [_i64, _i64, _i64, _p, _p, _p, _p, _p, _int, _int, _p]),
    "sgap_spmm_csr_ex": (_int, [_i64, _i64, _i64, _p, _p, _p, _p, _p, _int, _int, _int, _i64, _p]),
    "sgap_spmm_csr_gr": (_int, [_i64, _i64, _i64, _p, _p, _p, _p, _p, _int, _int, _i64, _p]),
    "sgap_config_init": (_int, [_p]),
    "sgap_spmm_csr_workspace_size": (_i64, [_i64, _i64, _i64, _p]),
    "sgap_spmm_csr_cfg": (_int, [_i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _i64, _p, _i64, _p]),
    "sgap_spmm_csr_cfg_static": (_int, [_i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _i64, _p]),
    "sgap_autotune_csr": (_int, [_i64, _i64, _i64, _p, _p, _p, _p, _p, _i64, _int, _p, _p, _p]),
    "sgap_autotune_csr_cfg": (_int, [_i64, _i64, _i64, _p, _p, _p, _p, _p, _i64, _int, _p, _i64, _p, _int, _p, _p, _p]),
    "sgap_sddmm_csr": (_int, [_i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _int, _int, _i64, _p]),
    "sgap_sddmm_csr_windows": (_int, [_i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _int, _int, _i64, _int, _int, _int, _p,
                                      _i64, _p]),
    "sgap_sddmm_csr_workspace_size": (_i64, [_i64, _i64, _int, _int]),
    "sgap_validate_csr": (_int, [_i64, _i64, _p, _p, _i64, _p, _p]),
    "sgap_reorder_rows_workspace_size": (_i64, [_i64]),
    "sgap_reorder_rows_csr": (_int, [_i64, _i64, _p, _p, _p, _int, _p, _p, _p, _p, _p, _i64, _p]),
    "sgap_ttm_csf": (_int, [_i64, _i64, _i64, _p, _p, _p, _p, _p, _int, _int, _int, _i64, _p]),
    "sgap_mttkrp_csf": (_int, [_i64, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _p, _p, _int, _int, _p]),
    "sgap_mttkrp_csf_ex": (_int, [_i64, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _p, _p, _int, _int, _int, _i64, _p]),
    "sgap_status_string": (ctypes.c_char_p, [_int]),
    "sgap_last_error": (ctypes.c_char_p, []),
    "sgap_version": (_int, []),
    "sgap_set_tuning": (_int, [_int, _int]),
    "sgap_profile_enable": (_int, [_int]),
    "sgap_profile_collect": (_int, [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_int)]),
    "sgap_debug_group_reduce": (_int, [_p, _p, _int, _int, _p]),
    "sgap_debug_group_partial_reduce": (_int, [_p, _p, _int, _int, _int, _p]),
    "sgap_debug_group_seg_reduce": (_int, [_p, _p, _p, _int, _int, _p]),
    "sgap_debug_tile_deal": (_i64, [_i64, _int, _int, _p, _i64]),
    "sgap_debug_plan_nnz_serial": (_int, [_int, _int, _int, _i64, _int, _int, _p, _p, _p]),
    "sgap_copy_f32": (_int, [_p, _p, _i64, _p]),
    "sgap_stream_f32": (_int, [_p, _p, _i64, _int, _p]),
}

_lib = None


class SgapError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"sgap status {status} ({what})")
        self.status = status


def load():
    """Load libsgap.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2209_02882_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(status: int):
    if status != SGAP_OK:
        lib = load()
        what = lib.sgap_status_string(status).decode()
        detail = lib.sgap_last_error().decode()
        raise SgapError(status, f"{what}: {detail}" if detail else what)


def _dev_ptr(t, dtype, name):
    import torch

    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor (device memory)")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr() if t.numel() else None


def _stream_ptr(stream):
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def sgap_version() -> int:
    return load().sgap_version()


def sgap_set_schedule(schedule: int) -> None:
    _check(load().sgap_set_schedule(int(schedule)))


def sgap_get_schedule() -> int:
    return load().sgap_get_schedule()


def _spmm_args(M, K, N, rowptr, colidx, vals, B, C):
    import torch

    if rowptr.numel() != M + 1:
        raise ValueError("rowptr must have M+1 entries")
    if colidx.numel() != vals.numel():
        raise ValueError("colidx and vals must have the same length")
    if B.numel() != K * N or C.numel() != M * N:
        raise ValueError("B must hold K*N and C must hold M*N elements")
    return (
        _dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
        _dev_ptr(vals, torch.float32, "vals"), _dev_ptr(B, torch.float32, "B"),
        _dev_ptr(C, torch.float32, "C"))


def sgap_spmm_csr(M, K, N, rowptr, colidx, vals, B, C, group_size, strategy, stream=None) -> None:
    """C = A_csr * B with the process-wide schedule (see include/sgap.h)."""
    ptrs = _spmm_args(M, K, N, rowptr, colidx, vals, B, C)
    _check(load().sgap_spmm_csr(M, K, N, *ptrs, int(group_size), int(strategy), _stream_ptr(stream)))


def sgap_spmm_csr_ex(M, K, N, rowptr, colidx, vals, B, C, group_size, strategy, schedule,
                     nnz_hint=None, stream=None) -> None:
    """C = A_csr * B with an explicit schedule.  nnz_hint defaults to the
    length of colidx, which the host knows without touching the device."""
    ptrs = _spmm_args(M, K, N, rowptr, colidx, vals, B, C)
    if nnz_hint is None:
        nnz_hint = colidx.numel()
    _check(load().sgap_spmm_csr_ex(M, K, N, *ptrs, int(group_size), int(strategy), int(schedule),
                                   int(nnz_hint), _stream_ptr(stream)))


SGAP_TUNE_TILE_COLS = 0
SGAP_TUNE_XCD_REMAP = 1
SGAP_TUNE_ROWS_PER_GROUP = 2
SGAP_TUNE_PERSISTENT = 3
SGAP_TUNE_NNZ_TILE = 4
SGAP_TUNE_SDDMM_ROW_CACHE = 5


class Config(ctypes.Structure):
    """Mirror of sgap_config: the point of the design space and the tiling knobs of one call."""
    _fields_ = [(name, ctypes.c_int) for name in (
        "schedule", "strategy", "group_size", "reduce_size", "block_size", "tile_cols", "rows_per_group",
        "xcd_remap", "persistent", "nnz_tile", "wave_rows", "long_row_min", "window_kb", "max_long_rows")]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


def make_config(group_size, strategy, schedule, **knobs) -> Config:
    """sgap_config with the library's defaults (sgap_config_init) and the named fields set; strategy and
    schedule by name or number."""
    c = Config()
    _check(load().sgap_config_init(ctypes.byref(c)))
    c.group_size = int(group_size)
    c.strategy = STRATEGIES.get(strategy, strategy)
    c.schedule = SCHEDULES.get(schedule, schedule)
    for k, v in knobs.items():
        if k not in dict(Config._fields_):
            raise KeyError(k)
        setattr(c, k, int(v))
    return c


def sgap_spmm_csr_workspace_size(M, K, N, config: Config) -> int:
    size = load().sgap_spmm_csr_workspace_size(M, K, N, ctypes.byref(config))
    if size < 0:
        raise SgapError(SGAP_ERR_INVALID_ARG, load().sgap_last_error().decode())
    return size


def _workspace_args(workspace):
    import torch

    if workspace is None:
        return None, 0
    if not isinstance(workspace, torch.Tensor) or not workspace.is_cuda or workspace.dtype != torch.uint8:
        raise TypeError("workspace must be a CUDA uint8 tensor")
    return (workspace.data_ptr() if workspace.numel() else None), workspace.numel()


def sgap_spmm_csr_cfg(M, K, N, rowptr, colidx, vals, B, C, config: Config, nnz_hint=None, workspace=None,
                      stream=None) -> None:
    """C = A_csr * B at the point and with the tiling `config` names; `workspace` is a CUDA uint8 tensor of
    at least sgap_spmm_csr_workspace_size bytes when the configuration sets long rows apart."""
    ptrs = _spmm_args(M, K, N, rowptr, colidx, vals, B, C)
    if nnz_hint is None:
        nnz_hint = colidx.numel()
    ws, ws_bytes = _workspace_args(workspace)
    _check(load().sgap_spmm_csr_cfg(M, K, N, *ptrs, ctypes.byref(config), int(nnz_hint), ws, ws_bytes,
                                    _stream_ptr(stream)))


def sgap_set_tuning(knob: int, value: int) -> None:
    _check(load().sgap_set_tuning(int(knob), int(value)))


def sgap_profile_enable(on: bool) -> None:
    _check(load().sgap_profile_enable(1 if on else 0))


def sgap_profile_collect():
    """(total milliseconds, number of timed main-kernel launches) since the last collect."""
    total = ctypes.c_double(0.0)
    count = ctypes.c_int(0)
    _check(load().sgap_profile_collect(ctypes.byref(total), ctypes.byref(count)))
    return total.value, count.value


def sgap_spmm_csr_gr(M, K, N, rowptr, colidx, vals, B, C, group_size, reduce_size, nnz_hint=None,
                     stream=None) -> None:
    """Row-split C = A_csr * B with group_size lanes per row reducing in
    sub-groups of reduce_size lanes (see include/sgap.h)."""
    ptrs = _spmm_args(M, K, N, rowptr, colidx, vals, B, C)
    if nnz_hint is None:
        nnz_hint = colidx.numel()
    _check(load().sgap_spmm_csr_gr(M, K, N, *ptrs, int(group_size), int(reduce_size), int(nnz_hint),
                                   _stream_ptr(stream)))


def sgap_sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T, out_vals, group_size, strategy, nnz_hint=None,
                   stream=None) -> None:
    """out_vals[p] = vals[p] * <X1[row(p), :], X2T[colidx[p], :]> (see include/sgap.h)."""
    import torch

    if rowptr.numel() != M + 1:
        raise ValueError("rowptr must have M+1 entries")
    if colidx.numel() != vals.numel() or out_vals.numel() != vals.numel():
        raise ValueError("colidx, vals and out_vals must have the same length")
    if X1.numel() != M * J or X2T.numel() != K * J:
        raise ValueError("X1 must hold M*J and X2T must hold K*J elements")
    if nnz_hint is None:
        nnz_hint = colidx.numel()
    _check(load().sgap_sddmm_csr(
        M, K, J, _dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
        _dev_ptr(vals, torch.float32, "vals"), _dev_ptr(X1, torch.float32, "X1"),
        _dev_ptr(X2T, torch.float32, "X2T"), _dev_ptr(out_vals, torch.float32, "out_vals"),
        int(group_size), int(strategy), int(nnz_hint), _stream_ptr(stream)))


def sgap_sddmm_csr_workspace_size(K, J, window_kb=0, max_long_rows=0) -> int:
    size = load().sgap_sddmm_csr_workspace_size(K, J, int(window_kb), int(max_long_rows))
    if size < 0:
        raise SgapError(SGAP_ERR_INVALID_ARG, load().sgap_last_error().decode())
    return size


def sgap_sddmm_csr_windows(M, K, J, rowptr, colidx, vals, X1, X2T, out_vals, group_size, strategy, long_row_min,
                           window_kb=0, max_long_rows=0, workspace=None, nnz_hint=None, stream=None) -> None:
    """sgap_sddmm_csr with the stored entries of rows of at least long_row_min entries taken by column
    windows of X2T (see include/sgap.h)."""
    import torch

    if rowptr.numel() != M + 1:
        raise ValueError("rowptr must have M+1 entries")
    if colidx.numel() != vals.numel() or out_vals.numel() != vals.numel():
        raise ValueError("colidx, vals and out_vals must have the same length")
    if X1.numel() != M * J or X2T.numel() != K * J:
        raise ValueError("X1 must hold M*J and X2T must hold K*J elements")
    if nnz_hint is None:
        nnz_hint = colidx.numel()
    ws, ws_bytes = _workspace_args(workspace)
    _check(load().sgap_sddmm_csr_windows(
        M, K, J, _dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
        _dev_ptr(vals, torch.float32, "vals"), _dev_ptr(X1, torch.float32, "X1"),
        _dev_ptr(X2T, torch.float32, "X2T"), _dev_ptr(out_vals, torch.float32, "out_vals"),
        int(group_size), int(strategy), int(nnz_hint), int(long_row_min), int(window_kb), int(max_long_rows),
        ws, ws_bytes, _stream_ptr(stream)))


def sgap_ttm_csf(F, K, L, eptr, eidx, vals, X1, Yf, group_size, strategy, schedule, nnz_hint=None,
                 stream=None) -> None:
    """Yf[f, :] = sum over the entries p of fiber f of vals[p] * X1[eidx[p], :] (see include/sgap.h)."""
    ptrs = _spmm_args(F, K, L, eptr, eidx, vals, X1, Yf)
    if nnz_hint is None:
        nnz_hint = eidx.numel()
    _check(load().sgap_ttm_csf(F, K, L, *ptrs, int(group_size), int(strategy), int(schedule), int(nnz_hint),
                               _stream_ptr(stream)))


def sgap_mttkrp_csf(I, K, L, J, fptr, fidx, eptr, eidx, vals, X1, X2, Y, group_size, strategy, stream=None) -> None:
    """Y[i, j] = sum over the stored (i, k, l) of A[i,k,l] * X1[k, j] * X2[l, j] (see include/sgap.h)."""
    import torch

    if fptr.numel() != I + 1:
        raise ValueError("fptr must have I+1 entries")
    if eptr.numel() != fidx.numel() + 1:
        raise ValueError("eptr must have one entry more than fidx")
    if eidx.numel() != vals.numel():
        raise ValueError("eidx and vals must have the same length")
    if X1.numel() != K * J or X2.numel() != L * J or Y.numel() != I * J:
        raise ValueError("X1 must hold K*J, X2 L*J and Y I*J elements")
    _check(load().sgap_mttkrp_csf(
        I, K, L, J, _dev_ptr(fptr, torch.int32, "fptr"), _dev_ptr(fidx, torch.int32, "fidx"),
        _dev_ptr(eptr, torch.int32, "eptr"), _dev_ptr(eidx, torch.int32, "eidx"),
        _dev_ptr(vals, torch.float32, "vals"), _dev_ptr(X1, torch.float32, "X1"), _dev_ptr(X2, torch.float32, "X2"),
        _dev_ptr(Y, torch.float32, "Y"), int(group_size), int(strategy), _stream_ptr(stream)))


def sgap_mttkrp_csf_ex(I, K, L, J, fptr, fidx, eptr, eidx, vals, X1, X2, Y, group_size, strategy, schedule,
                       nnz_hint=None, stream=None) -> None:
    """sgap_mttkrp_csf with a choice of schedule: slices (row-split) or stored entries (nnz-balanced) as the
    unit of work.  nnz_hint defaults to the length of vals."""
    import torch

    if fptr.numel() != I + 1:
        raise ValueError("fptr must have I+1 entries")
    if eptr.numel() != fidx.numel() + 1:
        raise ValueError("eptr must have one entry more than fidx")
    if eidx.numel() != vals.numel():
        raise ValueError("eidx and vals must have the same length")
    if X1.numel() != K * J or X2.numel() != L * J or Y.numel() != I * J:
        raise ValueError("X1 must hold K*J, X2 L*J and Y I*J elements")
    if nnz_hint is None:
        nnz_hint = vals.numel()
    _check(load().sgap_mttkrp_csf_ex(
        I, K, L, J, _dev_ptr(fptr, torch.int32, "fptr"), _dev_ptr(fidx, torch.int32, "fidx"),
        _dev_ptr(eptr, torch.int32, "eptr"), _dev_ptr(eidx, torch.int32, "eidx"),
        _dev_ptr(vals, torch.float32, "vals"), _dev_ptr(X1, torch.float32, "X1"), _dev_ptr(X2, torch.float32, "X2"),
        _dev_ptr(Y, torch.float32, "Y"), int(group_size), int(strategy), int(schedule), int(nnz_hint),
        _stream_ptr(stream)))


def sgap_validate_csr(M, K, rowptr, colidx, stream=None):
    """Counts of (rowptr defects, columns out of range, unsorted or repeated
    columns, empty rows) of a CSR matrix in device memory; the last two are -1
    when rowptr is damaged.  Waits for the stream (see include/sgap.h)."""
    import torch

    if rowptr.numel() != M + 1:
        raise ValueError("rowptr must have M+1 entries")
    report = (ctypes.c_int64 * 4)()
    _check(load().sgap_validate_csr(M, K, _dev_ptr(rowptr, torch.int32, "rowptr"),
                                    _dev_ptr(colidx, torch.int32, "colidx"), colidx.numel(), report,
                                    _stream_ptr(stream)))
    return tuple(report)


ROW_ORDERS = {"first_column": 0, "length": 1}


def sgap_reorder_rows_workspace_size(M):
    size = load().sgap_reorder_rows_workspace_size(M)
    if size < 0:
        raise SgapError(SGAP_ERR_INVALID_ARG, load().sgap_last_error().decode())
    return size


def sgap_reorder_rows_csr(M, K, rowptr, colidx, vals, order, perm, rowptr_out, colidx_out, vals_out, workspace,
                          stream=None):
    """Enqueue the row reordering of a CSR matrix in device memory (see include/sgap.h); `order` is a name of
    ROW_ORDERS or its number.  All arrays are the caller's tensors; nothing is allocated here."""
    import torch

    if rowptr.numel() != M + 1 or rowptr_out.numel() != M + 1:
        raise ValueError("rowptr and rowptr_out must have M+1 entries")
    if perm.numel() != M:
        raise ValueError("perm must have M entries")
    if colidx_out.numel() != colidx.numel() or vals_out.numel() != vals.numel() or vals.numel() != colidx.numel():
        raise ValueError("colidx, vals and their outputs must have nnz entries each")
    ws_ptr, ws_bytes = _workspace_args(workspace)
    _check(load().sgap_reorder_rows_csr(M, K, _dev_ptr(rowptr, torch.int32, "rowptr"),
                                        _dev_ptr(colidx, torch.int32, "colidx"), _dev_ptr(vals, torch.float32, "vals"),
                                        ROW_ORDERS.get(order, order), _dev_ptr(perm, torch.int32, "perm"),
                                        _dev_ptr(rowptr_out, torch.int32, "rowptr_out"),
                                        _dev_ptr(colidx_out, torch.int32, "colidx_out"),
                                        _dev_ptr(vals_out, torch.float32, "vals_out"), ws_ptr, ws_bytes,
                                        _stream_ptr(stream)))


class PointTime(ctypes.Structure):
    """Mirror of sgap_point_time."""
    _fields_ = [("group_size", ctypes.c_int), ("strategy", ctypes.c_int), ("schedule", ctypes.c_int),
                ("ms", ctypes.c_float)]


SGAP_NUM_POINTS = 28


def sgap_autotune_csr(M, K, N, rowptr, colidx, vals, B, C, nnz_hint=None, reps=3, stream=None):
    """Time every design-space point on these operands (blocking).  Returns
    (best, table): PointTime of the fastest point and the list of all 28."""
    ptrs = _spmm_args(M, K, N, rowptr, colidx, vals, B, C)
    if nnz_hint is None:
        nnz_hint = colidx.numel()
    table = (PointTime * SGAP_NUM_POINTS)()
    best = PointTime()
    _check(load().sgap_autotune_csr(M, K, N, *ptrs, int(nnz_hint), int(reps),
                                    ctypes.cast(table, ctypes.c_void_p), ctypes.cast(ctypes.pointer(best), ctypes.c_void_p),
                                    _stream_ptr(stream)))
    return best, list(table)


def sgap_spmm_csr_cfg_static(M, K, N, rowptr, colidx, vals, B, C, config: Config, nnz_hint=None, stream=None) -> None:
    """sgap_spmm_csr_cfg with the working memory in the library's built-in array (no allocation anywhere)."""
    ptrs = _spmm_args(M, K, N, rowptr, colidx, vals, B, C)
    if nnz_hint is None:
        nnz_hint = colidx.numel()
    _check(load().sgap_spmm_csr_cfg_static(M, K, N, *ptrs, ctypes.byref(config), int(nnz_hint), _stream_ptr(stream)))


class TunedPoint(ctypes.Structure):
    """Mirror of sgap_tuned_point."""
    _fields_ = [("config", Config), ("ms", ctypes.c_float)]


SGAP_MAX_TUNED_POINTS = 96


def sgap_autotune_csr_cfg(M, K, N, rowptr, colidx, vals, B, C, nnz_hint=None, reps=3, workspace=None, stream=None):
    """Rate the whole configuration space on these operands (blocking).  Returns (best, table): the
    fastest TunedPoint and the list of all rated ones."""
    ptrs = _spmm_args(M, K, N, rowptr, colidx, vals, B, C)
    if nnz_hint is None:
        nnz_hint = colidx.numel()
    ws, ws_bytes = _workspace_args(workspace)
    table = (TunedPoint * SGAP_MAX_TUNED_POINTS)()
    best = TunedPoint()
    count = ctypes.c_int(0)
    _check(load().sgap_autotune_csr_cfg(M, K, N, *ptrs, int(nnz_hint), int(reps), ws, ws_bytes,
                                        ctypes.cast(table, ctypes.c_void_p), SGAP_MAX_TUNED_POINTS,
                                        ctypes.cast(ctypes.pointer(count), ctypes.c_void_p),
                                        ctypes.cast(ctypes.pointer(best), ctypes.c_void_p), _stream_ptr(stream)))
    return best, list(table)[:min(count.value, SGAP_MAX_TUNED_POINTS)]


def sgap_debug_group_partial_reduce(inp, out, group_size, reduce_size, lanes_per_row, stream=None) -> None:
    import torch

    _check(load().sgap_debug_group_partial_reduce(
        _dev_ptr(inp, torch.float32, "in"), _dev_ptr(out, torch.float32, "out"),
        int(group_size), int(reduce_size), int(lanes_per_row), _stream_ptr(stream)))


def sgap_debug_group_reduce(inp, out, group_size, lanes_per_row, stream=None) -> None:
    import torch

    _check(load().sgap_debug_group_reduce(
        _dev_ptr(inp, torch.float32, "in"), _dev_ptr(out, torch.float32, "out"),
        int(group_size), int(lanes_per_row), _stream_ptr(stream)))


def sgap_debug_group_seg_reduce(inp, span, out, group_size, lanes_per_row, stream=None) -> None:
    import torch

    _check(load().sgap_debug_group_seg_reduce(
        _dev_ptr(inp, torch.float32, "in"), _dev_ptr(span, torch.int32, "span"),
        _dev_ptr(out, torch.float32, "out"), int(group_size), int(lanes_per_row), _stream_ptr(stream)))


def sgap_copy_f32(src, dst, n=None, stream=None) -> None:
    import torch

    if n is None:
        n = src.numel()
    if n > src.numel() or n > dst.numel():
        raise ValueError("copy length exceeds a buffer")
    _check(load().sgap_copy_f32(_dev_ptr(src, torch.float32, "src"), _dev_ptr(dst, torch.float32, "dst"),
                                int(n), _stream_ptr(stream)))


def sgap_stream_f32(src, dst, n, mode, stream=None) -> None:
    """mode 0: copy src -> dst; 1: read src only (dst: a one-float sink); 2: write dst only (see include/sgap_debug.h)."""
    import torch

    _check(load().sgap_stream_f32(_dev_ptr(src, torch.float32, "src") if src is not None else None,
                                  _dev_ptr(dst, torch.float32, "dst"), int(n), int(mode), _stream_ptr(stream)))
