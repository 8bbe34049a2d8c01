"""ctypes front end of the CPU oracle (``bs_ref.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, the smoke check and the
bench's ``cpu_baseline`` leg, never by the product package.  It takes and
returns numpy arrays on the host and holds no arithmetic of its own: every
number comes out of ``bs_ref.c`` (the plain definition of Sec. 3.1 / Sec. 3.2 /
Algorithm 1 / Fig. 3 / eq. (1) of arXiv 1811.00206).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bs_ref.c")
_LIB = os.path.join(_HERE, "libbs_ref.so")

OK, ERR_NULL, ERR_SHAPE, ERR_NONFINITE = 0, 1, 2, 6


class OracleError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"oracle {where} failed with status {status}")
        self.status = status


def build(force: bool = False) -> str:
    """Compile ``bs_ref.c`` with gcc (no fast-math) into ``libbs_ref.so``."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared",
             "-o", tmp, _SRC, "-lm", "-lpthread"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        # the _w entry points take the width of a stored offset (1 or 2 bytes)
        lib.bs_ref_prune_pack_w.argtypes = [vp, i32, i64, i64, i32, i32, vp, vp, i32]
        lib.bs_ref_unpack_w.argtypes = [vp, i32, vp, i32, i64, i64, i32, i32, vp]
        lib.bs_ref_spmm_f64_w.argtypes = [vp, i32, vp, i32, i64, i64, i32, i32, vp, i64, i64, vp, i64]
        lib.bs_ref_spmm_w.argtypes = [vp, i32, vp, i32, i64, i64, i32, i32, vp, i64, i64, vp, i64, i32]
        lib.bs_ref_spmv.argtypes = [vp, i32, vp, i64, i64, i32, i32, vp, vp, i32]
        lib.bs_ref_dense_gemm_f64.argtypes = [vp, i32, i64, i64, vp, i64, i64, vp, i64]
        lib.bs_ref_reprune.argtypes = [vp, i32, vp, i64, i32, i32, vp, vp]
        lib.bs_ref_lstm_step.argtypes = [vp, i32, vp, i64, i64, i32, i32, vp, vp, vp, vp, vp, vp]
        lib.bs_ref_rel_l2.argtypes = [vp, vp, i64]
        lib.bs_ref_rel_l2.restype = ctypes.c_double
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _storage(a: np.ndarray, what: str):
    """(is_f16, contiguous array) for an fp32 or fp16 array."""
    if a.dtype == np.float32:
        return 0, np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return 1, np.ascontiguousarray(a)
    raise TypeError(f"{what} must be float32 or float16, got {a.dtype}")


def host_threads() -> int:
    """Cores in this process's affinity mask."""
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def _offsets(idx: np.ndarray):
    """(bytes per stored offset, contiguous array) for a uint8 or uint16 offset array."""
    if idx.dtype == np.uint8 or idx.dtype == np.uint16:
        return idx.dtype.itemsize, np.ascontiguousarray(idx)
    raise TypeError(f"idx must be uint8 or uint16, got {idx.dtype}")


def prune_pack(W: np.ndarray, bank: int, k: int, wide: bool = False):
    """W (M x K, fp32 or fp16) -> vals [M, K/bank, k] (same dtype, bit copies),
    idx [M, K/bank, k], ascending offsets inside each bank: uint8 (bank <= 256), or
    with wide=True uint16 (bank <= 65536)."""
    is16, W = _storage(W, "W")
    if W.ndim != 2:
        raise ValueError("W must be 2-D")
    M, K = W.shape
    if bank < 1 or K % bank or k < 1 or k > bank or bank > (65536 if wide else 256):
        raise OracleError(ERR_SHAPE, "prune_pack")
    nb = K // bank
    vals = np.empty((M, nb, k), dtype=W.dtype)
    idx = np.empty((M, nb, k), dtype=np.uint16 if wide else np.uint8)
    st = _load().bs_ref_prune_pack_w(_p(W), is16, M, K, bank, k, _p(vals), _p(idx), idx.dtype.itemsize)
    if st:
        raise OracleError(st, "prune_pack")
    return vals, idx


def unpack(vals: np.ndarray, idx: np.ndarray, bank: int) -> np.ndarray:
    """Packed form -> the pruned dense matrix (zeros elsewhere)."""
    is16, vals = _storage(vals, "vals")
    ib, idx = _offsets(idx)
    M, nb, k = vals.shape
    K = nb * bank
    Wp = np.empty((M, K), dtype=vals.dtype)
    st = _load().bs_ref_unpack_w(_p(vals), is16, _p(idx), ib, M, K, bank, k, _p(Wp))
    if st:
        raise OracleError(st, "unpack")
    return Wp


def _x2d(X: np.ndarray, K: int):
    X = np.ascontiguousarray(X, dtype=np.float32)
    vec = X.ndim == 1
    X2 = X.reshape(K, -1)
    return vec, X2


def spmm_f64(vals, idx, bank: int, X) -> np.ndarray:
    """Un-rounded double sums of the sparse product (for exactness pins)."""
    is16, vals = _storage(vals, "vals")
    ib, idx = _offsets(idx)
    M, nb, k = vals.shape
    K = nb * bank
    vec, X2 = _x2d(X, K)
    N = X2.shape[1]
    Yd = np.empty((M, N), dtype=np.float64)
    st = _load().bs_ref_spmm_f64_w(_p(vals), is16, _p(idx), ib, M, K, bank, k, _p(X2), N, N, _p(Yd), N)
    if st:
        raise OracleError(st, "spmm_f64")
    return Yd[:, 0] if vec else Yd


def spmm(vals, idx, bank: int, X, threads: int = 1) -> np.ndarray:
    """Y = fp32(W_sparse . X); X is [K, N] (or [K] for the matrix-vector case)."""
    is16, vals = _storage(vals, "vals")
    ib, idx = _offsets(idx)
    M, nb, k = vals.shape
    K = nb * bank
    vec, X2 = _x2d(X, K)
    N = X2.shape[1]
    Y = np.empty((M, N), dtype=np.float32)
    st = _load().bs_ref_spmm_w(_p(vals), is16, _p(idx), ib, M, K, bank, k, _p(X2), N, N, _p(Y), N,
                               int(threads))
    if st:
        raise OracleError(st, "spmm")
    return Y[:, 0] if vec else Y


def spmv(vals, idx, bank: int, x, threads: int = 1) -> np.ndarray:
    """y = fp32(W_sparse . x)."""
    is16, vals = _storage(vals, "vals")
    ib, idx = _offsets(idx)
    M, nb, k = vals.shape
    K = nb * bank
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(K)
    y = np.empty(M, dtype=np.float32)
    if ib == 1:
        st = _load().bs_ref_spmv(_p(vals), is16, _p(idx), M, K, bank, k, _p(x), _p(y), int(threads))
    else:   # the N = 1 case of the product with 16-bit offsets
        st = _load().bs_ref_spmm_w(_p(vals), is16, _p(idx), ib, M, K, bank, k, _p(x), 1, 1, _p(y), 1,
                                   int(threads))
    if st:
        raise OracleError(st, "spmv")
    return y


def reprune(vals, idx, k2: int):
    """Keep the k2 largest magnitudes of the k stored per bank: (vals2, idx2) [M, nb, k2]."""
    is16, vals = _storage(vals, "vals")
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    M, nb, k = vals.shape
    vals2 = np.empty((M, nb, k2), dtype=vals.dtype)
    idx2 = np.empty((M, nb, k2), dtype=np.uint8)
    st = _load().bs_ref_reprune(_p(vals), is16, _p(idx), M * nb, k, int(k2), _p(vals2), _p(idx2))
    if st:
        raise OracleError(st, "reprune")
    return vals2, idx2


def lstm_step(vals, idx, bank: int, x, h, bias, c):
    """One LSTM step on the packed 4H x (I+H) gate matrix (gate blocks i, f, g, o):
    returns (c_out, h_out) as fp32."""
    is16, vals = _storage(vals, "vals")
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    M, nb, k = vals.shape
    H = M // 4
    K = nb * bank
    I = K - H
    if M != 4 * H or I < 1:
        raise ValueError("gate matrix must be 4H x (I + H)")
    f32 = lambda a, n: np.ascontiguousarray(a, dtype=np.float32).reshape(n)
    x, h, bias, c = f32(x, I), f32(h, H), f32(bias, 4 * H), f32(c, H)
    c_out = np.empty(H, dtype=np.float32)
    h_out = np.empty(H, dtype=np.float32)
    st = _load().bs_ref_lstm_step(_p(vals), is16, _p(idx), H, I, bank, k, _p(x), _p(h), _p(bias),
                                  _p(c), _p(c_out), _p(h_out))
    if st:
        raise OracleError(st, "lstm_step")
    return c_out, h_out


def lstm_sequence(vals, idx, bank: int, X, h0, bias, c0):
    """T steps, X is [T, I]; the state is carried in fp32 between steps.  Returns
    (H_all [T, H], c_T)."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    h = np.asarray(h0, dtype=np.float32)
    c = np.asarray(c0, dtype=np.float32)
    out = np.empty((X.shape[0], h.size), dtype=np.float32)
    for t in range(X.shape[0]):
        c, h = lstm_step(vals, idx, bank, X[t], h, bias, c)
        out[t] = h
    return out, c


def dense_gemm_f64(Wd: np.ndarray, X) -> np.ndarray:
    """Double-precision dense product over all K columns in ascending order."""
    is16, Wd = _storage(Wd, "Wd")
    M, K = Wd.shape
    vec, X2 = _x2d(X, K)
    N = X2.shape[1]
    Yd = np.empty((M, N), dtype=np.float64)
    st = _load().bs_ref_dense_gemm_f64(_p(Wd), is16, M, K, _p(X2), N, N, _p(Yd), N)
    if st:
        raise OracleError(st, "dense_gemm_f64")
    return Yd[:, 0] if vec else Yd


def rel_l2(a, b) -> float:
    """||a - b||_2 / ||b||_2 in double, b the reference."""
    a = np.ascontiguousarray(a, dtype=np.float32).ravel()
    b = np.ascontiguousarray(b, dtype=np.float32).ravel()
    if a.size != b.size:
        raise ValueError("size mismatch")
    return float(_load().bs_ref_rel_l2(_p(a), _p(b), a.size))
