"""Host-side checks of libbs.so that need no GPU: it loads, exports every
symbol the header declares, sizes are right, and bad arguments are refused
before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1811_00206_amd", "libbs.so")
HEADER = os.path.join(ROOT, "include", "bs.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bs_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = declared_functions()
    assert {"bs_prune_pack", "bs_spmv", "bs_spmm"} <= set(names)
    lib = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_covers_header():
    from paper_1811_00206_amd import binding
    assert sorted(binding.EXPORTS) == declared_functions()
    lib = binding.load_library()
    for n in binding.EXPORTS:
        assert getattr(lib, n) is not None
        assert hasattr(binding, n)


def test_sizes():
    from paper_1811_00206_amd import binding as b
    assert b.bs_nnz(6000, 3000, 100, 10) == 1_800_000
    assert b.bs_vals_bytes(6000, 3000, 100, 10, b.BS_F32) == 7_200_000
    assert b.bs_vals_bytes(4096, 25088, 64, 6, b.BS_F16) == 19_267_584
    assert b.bs_idx_bytes(4096, 25088, 64, 6) == 9_633_792
    assert b.bs_nnz(6000, 3000, 101, 10) == 0      # K % bank
    assert b.bs_nnz(6000, 3000, 100, 101) == 0     # k > bank
    assert b.bs_nnz(10, 1024, 512, 4) == 0         # bank > 256
    assert b.bs_vals_bytes(1, 4, 4, 1, 7) == 0     # unknown dtype
    assert b.bs_status_str(0) == "ok"
    assert "shape" in b.bs_status_str(2)


def test_workspace_query_is_pure_host():
    from paper_1811_00206_amd import binding as b
    assert b.bs_spmm_workspace_bytes(b.BS_F32, 256, 256, 64, 16, 8) == 0      # one slab
    ws = b.bs_spmm_workspace_bytes(b.BS_F32, 6000, 3000, 100, 10, 128)
    assert ws > 0 and ws % (6000 * 128 * 4) == 0
    assert b.bs_spmm_workspace_bytes(b.BS_F32, 6000, 3000, 101, 10, 8) == 0   # bad shape


def test_bad_arguments_are_refused_before_launch():
    from paper_1811_00206_amd import binding as b
    lib = b.load_library()
    p = ctypes.c_void_p(4096)      # never dereferenced: validation fails first
    odd = ctypes.c_void_p(4100)
    null = ctypes.c_void_p(0)
    assert lib.bs_spmv(null, p, 0, 4, 8, 4, 2, p, p, null) == 1
    assert lib.bs_spmv(p, p, 0, 4, 10, 4, 2, p, p, null) == 2            # K % bank
    assert lib.bs_spmv(p, p, 0, 4, 8, 4, 5, p, p, null) == 2             # k > bank
    assert lib.bs_spmv(p, p, 0, 0, 8, 4, 2, p, p, null) == 2             # M < 1
    assert lib.bs_spmv(p, p, 9, 4, 8, 4, 2, p, p, null) == 3             # dtype
    assert lib.bs_spmv(p, p, 0, 4, 1024, 512, 2, p, p, null) == 3        # bank > 256
    assert lib.bs_spmv(p, odd, 0, 4, 8, 4, 2, p, p, null) == 4           # alignment
    assert lib.bs_prune_pack(null, 0, 4, 8, 4, 2, p, p, null) == 1
    assert lib.bs_prune_pack(p, 0, 4, 8, 3, 2, p, p, null) == 2
    assert lib.bs_spmm(p, p, 0, 4, 8, 4, 2, p, 4, 3, p, 4, null, 0, null) == 2   # ldx < N
    assert lib.bs_spmv_ex(p, p, 0, 4, 8, 4, 2, p, p, 3, 0, null, null, null) == 3    # lanes not a power of two
    assert lib.bs_spmv_ex(p, p, 0, 4, 8, 4, 2, p, p, 16, 3, null, null, null) == 3   # 48 lanes per workgroup
    assert lib.bs_dense_gemv(p, 0, 0, 8, p, p, null) == 2
    assert lib.bs_dense_gemm(p, 0, 4, 8, p, 4, 2, p, 4, null) == 2
