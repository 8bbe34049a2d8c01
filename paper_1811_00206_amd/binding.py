"""Python names for the C-ABI calls of ``libbs.so`` (see ``include/bs.h``).

Argument marshalling only: each function checks tensor device / dtype /
contiguity, passes raw device pointers and torch's current HIP stream to the
library, and raises :class:`BsError` on a non-zero status.  There is no Python
or CPU implementation behind these names; if the library is missing the first
call fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbs.so")

BS_F32, BS_F16 = 0, 1

EXPORTS = (
    "bs_init", "bs_nnz", "bs_vals_bytes", "bs_idx_bytes", "bs_status_str", "bs_prune_pack", "bs_spmv",
    "bs_spmv_ex", "bs_spmv_plan", "bs_spmm_workspace_bytes", "bs_spmm_plan", "bs_spmm", "bs_spmm_static", "bs_spmm_static_limit", "bs_dense_gemv", "bs_dense_gemm",
    "bs_lstm_step", "bs_lstm_sequence", "bs_reprune",
    "bs_idx_bytes_wide", "bs_prune_pack_wide", "bs_spmv_wide", "bs_spmm_workspace_bytes_wide", "bs_spmm_wide",
)


class BsError(RuntimeError):
    def __init__(self, status: int, call: str):
        self.status = status
        super().__init__(f"{call}: {bs_status_str(status)} (status {status})")


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load ``libbs.so`` (built by ``python -m paper_1811_00206_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_1811_00206_amd.build`; "
            "there is no fallback implementation")
    lib = ctypes.CDLL(_LIB_PATH)
    i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    lib.bs_nnz.argtypes = [i64, i64, i32, i32]
    lib.bs_nnz.restype = sz
    lib.bs_vals_bytes.argtypes = [i64, i64, i32, i32, i32]
    lib.bs_vals_bytes.restype = sz
    lib.bs_idx_bytes.argtypes = [i64, i64, i32, i32]
    lib.bs_idx_bytes.restype = sz
    lib.bs_status_str.argtypes = [i32]
    lib.bs_status_str.restype = ctypes.c_char_p
    lib.bs_prune_pack.argtypes = [vp, i32, i64, i64, i32, i32, vp, vp, vp]
    lib.bs_spmv.argtypes = [vp, vp, i32, i64, i64, i32, i32, vp, vp, vp]
    lib.bs_spmv_ex.argtypes = [vp, vp, i32, i64, i64, i32, i32, vp, vp, i32, i32, vp, vp, vp]
    lib.bs_spmv_plan.argtypes = [i32, i64, i64, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_int64), i32]
    lib.bs_spmv_plan.restype = i32
    lib.bs_spmm_workspace_bytes.argtypes = [i32, i64, i64, i32, i32, i64]
    lib.bs_spmm_workspace_bytes.restype = sz
    lib.bs_spmm_plan.argtypes = [i32, i64, i64, i32, i32, i64, ctypes.POINTER(ctypes.c_int64), i32]
    lib.bs_spmm_plan.restype = i32
    lib.bs_spmm.argtypes = [vp, vp, i32, i64, i64, i32, i32, vp, i64, i64, vp, i64, vp, sz, vp]
    lib.bs_spmm_static.argtypes = [vp, vp, i32, i64, i64, i32, i32, vp, i64, i64, vp, i64, vp]
    lib.bs_spmm_static_limit.argtypes = []
    lib.bs_spmm_static_limit.restype = sz
    lib.bs_dense_gemv.argtypes = [vp, i32, i64, i64, vp, vp, vp]
    lib.bs_dense_gemm.argtypes = [vp, i32, i64, i64, vp, i64, i64, vp, i64, vp]
    lib.bs_reprune.argtypes = [vp, vp, i32, i64, i64, i32, i32, i32, vp, vp, vp]
    lib.bs_lstm_step.argtypes = [vp, vp, i32, i64, i64, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.bs_lstm_sequence.argtypes = [vp, vp, i32, i64, i64, i32, i32, vp, i64, vp, vp, vp, vp, vp]
    lib.bs_idx_bytes_wide.argtypes = [i64, i64, i32, i32]
    lib.bs_idx_bytes_wide.restype = sz
    lib.bs_prune_pack_wide.argtypes = [vp, i32, i64, i64, i32, i32, vp, vp, vp]
    lib.bs_spmv_wide.argtypes = [vp, vp, i32, i64, i64, i32, i32, vp, vp, vp]
    lib.bs_spmm_workspace_bytes_wide.argtypes = [i32, i64, i64, i32, i32, i64]
    lib.bs_spmm_workspace_bytes_wide.restype = sz
    lib.bs_spmm_wide.argtypes = [vp, vp, i32, i64, i64, i32, i32, vp, i64, i64, vp, i64, vp, sz, vp]
    for name in ("bs_prune_pack_wide", "bs_spmv_wide", "bs_spmm_wide"):
        getattr(lib, name).restype = i32
    lib.bs_init.argtypes = []
    for name in ("bs_init", "bs_prune_pack", "bs_spmv", "bs_spmv_ex", "bs_spmm", "bs_spmm_static", "bs_dense_gemv",
                 "bs_dense_gemm", "bs_lstm_step", "bs_lstm_sequence", "bs_reprune"):
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


# ------------------------------------------------------------------ helpers

def _dtype_code(t: torch.Tensor, what: str) -> int:
    if t.dtype == torch.float32:
        return BS_F32
    if t.dtype == torch.float16:
        return BS_F16
    raise TypeError(f"{what} must be float32 or float16, got {t.dtype}")


def _dev(t: torch.Tensor, what: str, dtype=None) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what} must be a tensor on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{what} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t


def _rows(t: torch.Tensor, what: str) -> int:
    """A 2-D fp32 GPU tensor whose rows are contiguous (a column slice of a wider
    row-major tensor is fine): returns its leading dimension in elements."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what} must be a tensor on the GPU")
    if t.dtype != torch.float32 or t.dim() != 2:
        raise TypeError(f"{what} must be a 2-D float32 tensor")
    if t.shape[1] > 1 and t.stride(1) != 1:
        raise ValueError(f"{what}: elements of a row must be adjacent")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], 1)
    if ld < t.shape[1]:
        raise ValueError(f"{what}: rows overlap")
    return ld


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _check(status: int, call: str):
    if status != 0:
        raise BsError(status, call)


def bs_init():
    """Prepare every kernel on the current device (optional; needed only before a capture
    whose first-ever library calls would happen inside it)."""
    _check(load_library().bs_init(), "bs_init")


# ------------------------------------------------------------ host-only calls

def bs_nnz(M: int, K: int, bank: int, k: int) -> int:
    return load_library().bs_nnz(M, K, bank, k)


def bs_vals_bytes(M: int, K: int, bank: int, k: int, dtype: int) -> int:
    return load_library().bs_vals_bytes(M, K, bank, k, dtype)


def bs_idx_bytes(M: int, K: int, bank: int, k: int) -> int:
    return load_library().bs_idx_bytes(M, K, bank, k)


def bs_status_str(status: int) -> str:
    return load_library().bs_status_str(status).decode()


def bs_spmm_workspace_bytes(dtype: int, M: int, K: int, bank: int, k: int, N: int) -> int:
    return load_library().bs_spmm_workspace_bytes(dtype, M, K, bank, k, N)


SPMV_PLAN_FIELDS = ("slab_kernel", "ch", "lpr", "u", "threads", "rows_per_wg", "workgroups", "lds_bytes",
                    "table", "bank_mode")


def bs_spmv_plan(dtype: int, M: int, K: int, bank: int, k: int, lanes_per_row: int = 0,
                 rows_per_wg: int = 0) -> dict:
    """The launch bs_spmv / bs_spmv_ex would make (host only).  Raises on an unsupported shape."""
    out = (ctypes.c_int64 * len(SPMV_PLAN_FIELDS))()
    _check(load_library().bs_spmv_plan(dtype, M, K, bank, k, lanes_per_row, rows_per_wg, out,
                                       len(SPMV_PLAN_FIELDS)), "bs_spmv_plan")
    return dict(zip(SPMV_PLAN_FIELDS, (int(v) for v in out)))


SPMM_PLAN_FIELDS = ("rows_kernel", "ch", "nl", "nt", "n_tiles", "sb", "n_slabs", "lpr", "u", "threads",
                    "rows_per_wg", "row_groups", "n_passes", "lds_bytes", "workgroups", "table_off")


def bs_spmm_plan(dtype: int, M: int, K: int, bank: int, k: int, N: int) -> dict:
    """The launch bs_spmm would make (host only).  Raises on an unsupported shape."""
    out = (ctypes.c_int64 * len(SPMM_PLAN_FIELDS))()
    _check(load_library().bs_spmm_plan(dtype, M, K, bank, k, N, out, len(SPMM_PLAN_FIELDS)), "bs_spmm_plan")
    return dict(zip(SPMM_PLAN_FIELDS, (int(v) for v in out)))


# --------------------------------------------------------------- GPU calls

def bs_prune_pack(W: torch.Tensor, bank: int, k: int, out=None):
    """W [M, K] on the GPU (fp32/fp16) -> (vals [M, K/bank, k], idx uint8 same shape);
    `out` = (vals, idx) to write into existing tensors."""
    _dev(W, "W")
    code = _dtype_code(W, "W")
    if W.dim() != 2:
        raise ValueError("W must be 2-D")
    M, K = W.shape
    if bank < 1 or K % bank or k < 1 or k > bank:
        raise BsError(2, "bs_prune_pack")
    nb = K // bank
    if out is None:
        vals = torch.empty((M, nb, k), dtype=W.dtype, device=W.device)
        idx = torch.empty((M, nb, k), dtype=torch.uint8, device=W.device)
    else:
        vals, idx = out
        _dev(vals, "vals", W.dtype)
        _dev(idx, "idx", torch.uint8)
        if tuple(vals.shape) != (M, nb, k) or tuple(idx.shape) != (M, nb, k):
            raise ValueError(f"out must be two [{M}, {nb}, {k}] tensors")
    _check(load_library().bs_prune_pack(_ptr(W), code, M, K, bank, k, _ptr(vals), _ptr(idx),
                                        _stream()), "bs_prune_pack")
    return vals, idx


def _packed(vals, idx, bank):
    _dev(vals, "vals")
    _dev(idx, "idx", torch.uint8)
    if vals.dim() != 3 or idx.shape != vals.shape:
        raise ValueError("vals and idx must both be [M, K/bank, k]")
    M, nb, k = vals.shape
    return _dtype_code(vals, "vals"), M, nb * bank, k


def bs_spmv(vals, idx, bank: int, x, out=None, lanes_per_row: int = 0, rows_per_wg: int = 0,
            start_event: int = 0, stop_event: int = 0):
    """y [M] = W_sparse . x, x [K] fp32 on the GPU.  start_event / stop_event are
    optional raw hipEvent_t handles that receive the kernel's own time stamps."""
    code, M, K, k = _packed(vals, idx, bank)
    _dev(x, "x", torch.float32)
    if x.numel() != K:
        raise ValueError(f"x must have {K} elements")
    y = torch.empty(M, dtype=torch.float32, device=vals.device) if out is None else _dev(
        out, "out", torch.float32)
    if y.numel() != M:
        raise ValueError(f"out must have {M} elements")
    lib = load_library()
    if lanes_per_row or rows_per_wg or start_event or stop_event:
        st = lib.bs_spmv_ex(_ptr(vals), _ptr(idx), code, M, K, bank, k, _ptr(x), _ptr(y),
                            lanes_per_row, rows_per_wg, ctypes.c_void_p(start_event),
                            ctypes.c_void_p(stop_event), _stream())
    else:
        st = lib.bs_spmv(_ptr(vals), _ptr(idx), code, M, K, bank, k, _ptr(x), _ptr(y), _stream())
    _check(st, "bs_spmv")
    return y


class PreparedSpmv:
    """bs_spmv_ex with its arguments marshalled once, for launch loops where the
    Python-side checks of :func:`bs_spmv` would dominate a microsecond kernel.
    Each call is exactly one C-ABI call on torch's current stream (read at every
    call, so the same object works inside and outside a graph capture); the tensors
    are kept alive by this object."""

    def __init__(self, vals, idx, bank: int, x, out, lanes_per_row: int = 0, rows_per_wg: int = 0):
        code, M, K, k = _packed(vals, idx, bank)
        _dev(x, "x", torch.float32)
        _dev(out, "out", torch.float32)
        if x.numel() != K or out.numel() != M:
            raise ValueError("x must have K elements and out M elements")
        self._keep = (vals, idx, x, out)
        self._fn = load_library().bs_spmv_ex
        self._head = (_ptr(vals), _ptr(idx), code, M, K, bank, k, _ptr(x), _ptr(out),
                      lanes_per_row, rows_per_wg)

    def __call__(self, start_event: int = 0, stop_event: int = 0):
        st = self._fn(*self._head, start_event, stop_event, _stream())
        if st:
            raise BsError(st, "bs_spmv_ex")


def bs_spmv_ex(vals, idx, bank, x, lanes_per_row, rows_per_wg, out=None, start_event=0,
               stop_event=0):
    return bs_spmv(vals, idx, bank, x, out=out, lanes_per_row=lanes_per_row,
                   rows_per_wg=rows_per_wg, start_event=start_event, stop_event=stop_event)


def new_spmm_workspace(nbytes: int, device) -> torch.Tensor:
    """A workspace for bs_spmm / bs_spmm_wide (uninitialised device memory)."""
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def bs_spmm(vals, idx, bank: int, X, out=None, workspace=None):
    """Y [M, N] = W_sparse . X, X [K, N] fp32 on the GPU, rows contiguous (X and `out`
    may be column slices of wider row-major tensors: their row strides are passed as
    leading dimensions).  `workspace` is an optional uint8 tensor of at least
    bs_spmm_workspace_bytes(...) bytes; without it one is taken from torch's allocator
    for this call."""
    code, M, K, k = _packed(vals, idx, bank)
    ldx = _rows(X, "X")
    if X.shape[0] != K:
        raise ValueError(f"X must be [{K}, N]")
    N = X.shape[1]
    Y = torch.empty((M, N), dtype=torch.float32, device=vals.device) if out is None else out
    ldy = _rows(Y, "out")
    if tuple(Y.shape) != (M, N):
        raise ValueError(f"out must be [{M}, {N}]")
    lib = load_library()
    need = lib.bs_spmm_workspace_bytes(code, M, K, bank, k, N)
    if need and workspace is None:
        workspace = new_spmm_workspace(need, vals.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.bs_spmm(_ptr(vals), _ptr(idx), code, M, K, bank, k, _ptr(X), N, ldx, _ptr(Y), ldy,
                       _ptr(workspace), ws_bytes, _stream()), "bs_spmm")
    return Y


def bs_spmm_static_limit() -> int:
    return load_library().bs_spmm_static_limit()


def bs_spmm_static(vals, idx, bank: int, X, out):
    """bs_spmm without a workspace and without any allocation: the slab partial sums go to
    the library's static device array, and `out` must be given (this wrapper allocates
    nothing either).  Calls that overlap on one GPU race on that array."""
    code, M, K, k = _packed(vals, idx, bank)
    ldx = _rows(X, "X")
    if X.shape[0] != K:
        raise ValueError(f"X must be [{K}, N]")
    N = X.shape[1]
    ldy = _rows(out, "out")
    if tuple(out.shape) != (M, N):
        raise ValueError(f"out must be [{M}, {N}]")
    _check(load_library().bs_spmm_static(_ptr(vals), _ptr(idx), code, M, K, bank, k, _ptr(X), N, ldx,
                                         _ptr(out), ldy, _stream()), "bs_spmm_static")
    return out


def bs_dense_gemv(W, x, out=None):
    """y = W . x with the hand-written dense baseline kernel."""
    _dev(W, "W")
    code = _dtype_code(W, "W")
    M, K = W.shape
    _dev(x, "x", torch.float32)
    if x.numel() != K:
        raise ValueError(f"x must have {K} elements")
    y = torch.empty(M, dtype=torch.float32, device=W.device) if out is None else _dev(
        out, "out", torch.float32)
    _check(load_library().bs_dense_gemv(_ptr(W), code, M, K, _ptr(x), _ptr(y), _stream()),
           "bs_dense_gemv")
    return y


def bs_dense_gemm(W, X, out=None):
    """Y = W . X with the hand-written dense baseline kernel."""
    _dev(W, "W")
    code = _dtype_code(W, "W")
    M, K = W.shape
    _dev(X, "X", torch.float32)
    if X.dim() != 2 or X.shape[0] != K:
        raise ValueError(f"X must be [{K}, N]")
    N = X.shape[1]
    Y = torch.empty((M, N), dtype=torch.float32, device=W.device) if out is None else _dev(
        out, "out", torch.float32)
    _check(load_library().bs_dense_gemm(_ptr(W), code, M, K, _ptr(X), N, N, _ptr(Y), N, _stream()),
           "bs_dense_gemm")
    return Y


# ---- balance ranges over 256: 16-bit offsets (torch has no uint16 arithmetic, but tensors of
# that dtype can be allocated, copied and compared, which is all that is needed here)

def bs_idx_bytes_wide(M: int, K: int, bank: int, k: int) -> int:
    return load_library().bs_idx_bytes_wide(M, K, bank, k)


def bs_spmm_workspace_bytes_wide(dtype: int, M: int, K: int, bank: int, k: int, N: int) -> int:
    return load_library().bs_spmm_workspace_bytes_wide(dtype, M, K, bank, k, N)


def bs_prune_pack_wide(W: torch.Tensor, bank: int, k: int, out=None):
    """W [M, K] on the GPU (fp32/fp16) -> (vals [M, K/bank, k], idx uint16 same shape)."""
    _dev(W, "W")
    code = _dtype_code(W, "W")
    if W.dim() != 2:
        raise ValueError("W must be 2-D")
    M, K = W.shape
    if bank < 1 or K % bank or k < 1 or k > bank:
        raise BsError(2, "bs_prune_pack_wide")
    nb = K // bank
    if out is None:
        vals = torch.empty((M, nb, k), dtype=W.dtype, device=W.device)
        idx = torch.empty((M, nb, k), dtype=torch.uint16, device=W.device)
    else:
        vals, idx = out
        _dev(vals, "vals", W.dtype)
        _dev(idx, "idx", torch.uint16)
        if tuple(vals.shape) != (M, nb, k) or tuple(idx.shape) != (M, nb, k):
            raise ValueError(f"out must be two [{M}, {nb}, {k}] tensors")
    _check(load_library().bs_prune_pack_wide(_ptr(W), code, M, K, bank, k, _ptr(vals), _ptr(idx),
                                             _stream()), "bs_prune_pack_wide")
    return vals, idx


def _packed_wide(vals, idx, bank):
    _dev(vals, "vals")
    _dev(idx, "idx", torch.uint16)
    if vals.dim() != 3 or idx.shape != vals.shape:
        raise ValueError("vals and idx must both be [M, K/bank, k]")
    M, nb, k = vals.shape
    return _dtype_code(vals, "vals"), M, nb * bank, k


def bs_spmv_wide(vals, idx, bank: int, x, out=None):
    """y [M] = W_sparse . x for a packed matrix with uint16 offsets."""
    code, M, K, k = _packed_wide(vals, idx, bank)
    _dev(x, "x", torch.float32)
    if x.numel() != K:
        raise ValueError(f"x must have {K} elements")
    y = torch.empty(M, dtype=torch.float32, device=vals.device) if out is None else _dev(
        out, "out", torch.float32)
    if y.numel() != M:
        raise ValueError(f"out must have {M} elements")
    _check(load_library().bs_spmv_wide(_ptr(vals), _ptr(idx), code, M, K, bank, k, _ptr(x), _ptr(y),
                                       _stream()), "bs_spmv_wide")
    return y


def bs_spmm_wide(vals, idx, bank: int, X, out=None, workspace=None):
    """Y [M, N] = W_sparse . X for a packed matrix with uint16 offsets (see bs_spmm)."""
    code, M, K, k = _packed_wide(vals, idx, bank)
    ldx = _rows(X, "X")
    if X.shape[0] != K:
        raise ValueError(f"X must be [{K}, N]")
    N = X.shape[1]
    Y = torch.empty((M, N), dtype=torch.float32, device=vals.device) if out is None else out
    ldy = _rows(Y, "out")
    if tuple(Y.shape) != (M, N):
        raise ValueError(f"out must be [{M}, {N}]")
    lib = load_library()
    need = lib.bs_spmm_workspace_bytes_wide(code, M, K, bank, k, N)
    if need and workspace is None:
        workspace = new_spmm_workspace(need, vals.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.bs_spmm_wide(_ptr(vals), _ptr(idx), code, M, K, bank, k, _ptr(X), N, ldx, _ptr(Y), ldy,
                            _ptr(workspace), ws_bytes, _stream()), "bs_spmm_wide")
    return Y


def _lstm_shape(vals, idx, bank):
    code, M, K, k = _packed(vals, idx, bank)
    if M % 4:
        raise ValueError("the gate matrix must have 4H rows")
    H = M // 4
    I = K - H
    if I < 1:
        raise ValueError("the gate matrix must have I + H columns with I >= 1")
    return code, H, I, k


def bs_lstm_step(vals, idx, bank: int, x, h, bias, c, c_out=None, h_out=None):
    """One LSTM step on the packed 4H x (I+H) gate matrix: returns (c_out, h_out)."""
    code, H, I, k = _lstm_shape(vals, idx, bank)
    for t, name, n in ((x, "x", I), (h, "h", H), (bias, "bias", 4 * H), (c, "c", H)):
        _dev(t, name, torch.float32)
        if t.numel() != n:
            raise ValueError(f"{name} must have {n} elements")
    c_out = torch.empty(H, dtype=torch.float32, device=vals.device) if c_out is None else _dev(
        c_out, "c_out", torch.float32)
    h_out = torch.empty(H, dtype=torch.float32, device=vals.device) if h_out is None else _dev(
        h_out, "h_out", torch.float32)
    _check(load_library().bs_lstm_step(_ptr(vals), _ptr(idx), code, H, I, bank, k, _ptr(x), _ptr(h),
                                       _ptr(bias), _ptr(c), _ptr(c_out), _ptr(h_out), _stream()),
           "bs_lstm_step")
    return c_out, h_out


def bs_lstm_sequence(vals, idx, bank: int, X, h0, bias, c, H_all=None):
    """T steps; X is [T, I]; `c` is updated in place.  Returns H_all [T, H]."""
    code, H, I, k = _lstm_shape(vals, idx, bank)
    _dev(X, "X", torch.float32)
    if X.dim() != 2 or X.shape[1] != I:
        raise ValueError(f"X must be [T, {I}]")
    T = X.shape[0]
    for t, name, n in ((h0, "h0", H), (bias, "bias", 4 * H), (c, "c", H)):
        _dev(t, name, torch.float32)
        if t.numel() != n:
            raise ValueError(f"{name} must have {n} elements")
    H_all = torch.empty((T, H), dtype=torch.float32, device=vals.device) if H_all is None else _dev(
        H_all, "H_all", torch.float32)
    _check(load_library().bs_lstm_sequence(_ptr(vals), _ptr(idx), code, H, I, bank, k, _ptr(X), T,
                                           _ptr(h0), _ptr(bias), _ptr(c), _ptr(H_all), _stream()),
           "bs_lstm_sequence")
    return H_all


def bs_reprune(vals, idx, bank: int, k2: int, out=None):
    """Packed [M, K/bank, k] -> packed [M, K/bank, k2], k2 <= k: (vals2, idx2);
    `out` = (vals2, idx2) to write into existing tensors."""
    code, M, K, k = _packed(vals, idx, bank)
    if k2 < 1 or k2 > k:
        raise BsError(2, "bs_reprune")
    nb = K // bank
    if out is None:
        vals2 = torch.empty((M, nb, k2), dtype=vals.dtype, device=vals.device)
        idx2 = torch.empty((M, nb, k2), dtype=torch.uint8, device=vals.device)
    else:
        vals2, idx2 = out
        _dev(vals2, "vals2", vals.dtype)
        _dev(idx2, "idx2", torch.uint8)
        if tuple(vals2.shape) != (M, nb, k2) or tuple(idx2.shape) != (M, nb, k2):
            raise ValueError(f"out must be two [{M}, {nb}, {k2}] tensors")
    _check(load_library().bs_reprune(_ptr(vals), _ptr(idx), code, M, K, bank, k, k2, _ptr(vals2),
                                     _ptr(idx2), _stream()), "bs_reprune")
    return vals2, idx2
