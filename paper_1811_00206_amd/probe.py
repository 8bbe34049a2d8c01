"""Python names for the measurement helpers of ``libbs_probe.so`` (``probe/bs_probe.h``).

Not part of the method and not part of ``libbs.so``: an empty kernel, a read-only
kernel, a kernel of LDS gathers and a grid-barrier loop, which ``bench.py`` times
beside the products to show the machine's floor.  Marshalling only.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbs_probe.so")

EXPORTS = ("bs_probe_timestamp", "bs_probe_wall_clock_khz", "bs_probe_empty", "bs_probe_stream_read", "bs_probe_lds_gather", "bs_probe_grid_barrier")

_lib = None


class ProbeError(RuntimeError):
    def __init__(self, status: int, call: str):
        self.status = status
        super().__init__(f"{call}: status {status}")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_1811_00206_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    i32, u32, vp, sz = ctypes.c_int, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_size_t
    lib.bs_probe_timestamp.argtypes = [vp, vp]
    lib.bs_probe_wall_clock_khz.argtypes = []
    lib.bs_probe_empty.argtypes = [i32, i32, vp]
    lib.bs_probe_stream_read.argtypes = [vp, sz, i32, i32, i32, vp, sz, vp]
    lib.bs_probe_lds_gather.argtypes = [i32, i32, i32, i32, vp, vp]
    lib.bs_probe_grid_barrier.argtypes = [i32, i32, i32, i32, i32, u32, vp, vp, vp]
    for name in EXPORTS:
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _check(status: int, call: str):
    if status != 0:
        raise ProbeError(status, call)


def _dev(t, what):
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{what} must be a contiguous tensor on the GPU")
    return t


def probe_timestamp(slots: torch.Tensor, i: int):
    """Store the GPU's wall clock into slots[i] (an int64 tensor on the GPU) on the current stream."""
    _dev(slots, "slots")
    if slots.dtype != torch.int64 or not 0 <= i < slots.numel():
        raise ValueError("slots must be an int64 tensor and i inside it")
    _check(load_library().bs_probe_timestamp(ctypes.c_void_p(slots.data_ptr() + 8 * i), _stream()),
           "bs_probe_timestamp")


def wall_clock_khz() -> int:
    return load_library().bs_probe_wall_clock_khz()


def probe_empty(grid: int = 256, threads: int = 256):
    """Launch an empty kernel on the current stream."""
    _check(load_library().bs_probe_empty(grid, threads, _stream()), "bs_probe_empty")


def probe_stream_read(src: torch.Tensor, pieces_per_lane: int = 0, sink: torch.Tensor = None,
                      store_mode: int = 0, store_every: int = 32):
    """A kernel that only reads all of `src` (bytes a multiple of 16); with store_mode 1..3 one
    lane in `store_every` also stores a word to `sink` (plain / non-temporal / agent-scope
    atomic store)."""
    _dev(src, "src")
    nbytes = src.numel() * src.element_size()
    sink_bytes = 0 if sink is None else sink.numel() * sink.element_size()
    _check(load_library().bs_probe_stream_read(_ptr(src), nbytes, pieces_per_lane, store_mode, store_every,
                                               _ptr(sink), sink_bytes, _stream()), "bs_probe_stream_read")


def probe_lds_gather(threads: int = 768, pattern: int = 1, group_lanes: int = 8, reads: int = 16000):
    """256 workgroups that only issue LDS reads (`reads` per lane); pattern 0 = adjacent 16-byte
    pieces, 1 = groups of `group_lanes` lanes on random rows, 2 = a random word per lane,
    3 = a random 256-byte row per lane, word = lane number (no LDS bank shared)."""
    _check(load_library().bs_probe_lds_gather(threads, pattern, group_lanes, reads, None, _stream()),
           "bs_probe_lds_gather")


def probe_grid_barrier(wgs: int, threads: int, steps: int, vec_floats: int, mode: int,
                       sync: torch.Tensor, hbuf: torch.Tensor, spin_limit: int = 1 << 16):
    """`steps` rounds of read-vector / write-slice / grid-wide barrier with bounded waits.
    `sync`: two zeroed int32 on the GPU ([0] arrivals, [1] abort flag); `hbuf`: 2*vec_floats fp32."""
    _dev(sync, "sync")
    _dev(hbuf, "hbuf")
    if sync.numel() * sync.element_size() < 8 or hbuf.numel() * hbuf.element_size() < 8 * vec_floats:
        raise ValueError("sync needs 8 bytes, hbuf 2*vec_floats floats")
    _check(load_library().bs_probe_grid_barrier(wgs, threads, steps, vec_floats, mode, spin_limit,
                                                _ptr(sync), _ptr(hbuf), _stream()),
           "bs_probe_grid_barrier")
