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
    out = (ctypes.c_int64 * 16)()
    assert lib.bs_spmm_plan(0, 4, 8, 4, 2, 4, None, 16) == 1             # no output array
    assert lib.bs_spmm_plan(0, 4, 10, 4, 2, 4, out, 16) == 2             # K % bank
    assert lib.bs_spmm_plan(0, 4, 8, 4, 2, 0, out, 16) == 2              # N < 1
    assert lib.bs_spmm_plan(5, 4, 8, 4, 2, 4, out, 16) == 3              # dtype
    # LSTM step and pruning round: shape rules of their own
    assert lib.bs_lstm_step(p, p, 0, 6, 8, 2, 1, p, p, p, p, p, p, null) == 3       # H % 4
    assert lib.bs_lstm_step(p, p, 0, 8, 8, 2, 1, p, p, p, p, p, p, null) == 3       # h_out == h_in
    assert lib.bs_reprune(p, p, 0, 4, 8, 4, 2, 3, p, p, null) == 2                  # k2 > k
    # the no-allocation product validates like bs_spmm, and refuses a product over its static
    # scratch before it touches the GPU
    assert lib.bs_spmm_static(p, p, 0, 4, 8, 4, 2, p, 4, 3, p, 4, null) == 2         # ldx < N
    assert lib.bs_spmm_static(p, null, 0, 4, 8, 4, 2, p, 4, 4, p, 4, null) == 1
    assert b.bs_spmm_workspace_bytes(b.BS_F32, 6000, 3000, 100, 10, 2048) > b.bs_spmm_static_limit()
    assert lib.bs_spmm_static(p, p, 0, 6000, 3000, 100, 10, p, 2048, 2048, p, 2048, null) == 8
    assert "scratch" in b.bs_status_str(8)
    assert b.bs_spmm_static_limit() == 16 << 20


def test_first_use_inside_a_capture_has_its_own_status():
    from paper_1811_00206_amd import binding as b
    assert "bs_init" in b.bs_status_str(7)


def test_probe_library_is_separate():
    """The measurement helpers are not in the product library."""
    from paper_1811_00206_amd import probe
    lib = ctypes.CDLL(LIB)
    plib = probe.load_library()
    for n in probe.EXPORTS:
        assert not hasattr(lib, n), n
        assert getattr(plib, n) is not None
    null = ctypes.c_void_p(0)
    assert plib.bs_probe_empty(0, 256, null) == 2
    assert plib.bs_probe_stream_read(null, 64, 0, 0, 0, null, 0, null) == 1
    assert plib.bs_probe_stream_read(ctypes.c_void_p(4096), 24, 0, 0, 0, null, 0, null) == 2
    assert plib.bs_probe_stream_read(ctypes.c_void_p(4096), 4096, 1, 1, 32, ctypes.c_void_p(8192), 16, null) == 2
    assert plib.bs_probe_stream_read(ctypes.c_void_p(4096), 4096, 1, 1, 0, ctypes.c_void_p(8192), 4096, null) == 2
    assert plib.bs_probe_lds_gather(768, 1, 3, 64, null, null) == 2
    assert plib.bs_probe_grid_barrier(257, 256, 10, 1500, 0, 100, ctypes.c_void_p(4096),
                                      ctypes.c_void_p(4096), null) == 2


def _plan_invariants(b, dtype, M, K, bank, k, N):
    """What the SpMM kernels assume about their launch, checked on the host for one shape."""
    vsize = 2 if dtype == b.BS_F16 else 4
    p = b.bs_spmm_plan(dtype, M, K, bank, k, N)
    nb = K // bank
    where = f"{(dtype, M, K, bank, k, N)} -> {p}"
    # tile geometry
    assert p["nl"] in (1, 2, 4, 8, 16) and p["nt"] == 4 * p["nl"], where
    assert p["n_tiles"] * p["nt"] >= N > (p["n_tiles"] - 1) * p["nt"], where
    assert 1 <= p["sb"] <= nb and p["n_slabs"] == -(-nb // p["sb"]), where
    # chunks: whole 16-byte (or narrower) chunks in every slab's run, including the last slab's
    assert p["ch"] in (1, 2, 4, 8) and p["ch"] * vsize <= 16, where
    assert (nb * k) % p["ch"] == 0, where
    last = nb - (p["n_slabs"] - 1) * p["sb"]
    for banks in {p["sb"], last}:
        assert (banks * k) % p["ch"] == 0, where
    if p["n_slabs"] > 1:
        assert (p["sb"] * k * vsize) % (p["ch"] * vsize) == 0, where   # slab starts stay chunk-aligned
    # LDS: tile, then the position table
    tile = p["sb"] * bank * p["nl"] * 16
    assert p["table_off"] * 4 == tile, where
    assert p["lds_bytes"] == tile + p["sb"] * k * 4 <= 160 * 1024, where
    # lanes
    assert p["threads"] % 64 == 0 and 64 <= p["threads"] <= 1024, where
    if p["rows_kernel"]:
        assert p["nl"] >= 4 and p["lpr"] == 1 and p["u"] == 4, where
    else:
        assert p["lpr"] in (4, 8, 16, 32, 64) and p["u"] in (2, 4) and p["nl"] * p["lpr"] <= 64, where
    rows_per_pass = p["threads"] // (p["nl"] * p["lpr"])
    assert rows_per_pass >= 1, where
    # rows: every row in exactly one group, every row of a group in one pass
    assert p["row_groups"] * p["rows_per_wg"] >= M > (p["row_groups"] - 1) * p["rows_per_wg"], where
    assert p["n_passes"] * rows_per_pass >= p["rows_per_wg"] > (p["n_passes"] - 1) * rows_per_pass, where
    # grid: a multiple of the 8 XCDs that covers every (tile, slab, row group)
    total = p["n_tiles"] * p["n_slabs"] * p["row_groups"]
    assert p["workgroups"] % 8 == 0 and total <= p["workgroups"] < total + 8, where
    # workspace: partial sums of every slab, or none
    ws = b.bs_spmm_workspace_bytes(dtype, M, K, bank, k, N)
    assert ws == (p["n_slabs"] * M * N * 4 if p["n_slabs"] > 1 else 0), where
    return p


def test_spmm_plan_invariants_on_the_paper_shapes():
    from paper_1811_00206_amd import binding as b
    seen = set()
    for dtype, M, K, bank, k, Ns in [
            (b.BS_F32, 256, 256, 64, 16, (1, 8)),
            (b.BS_F32, 6000, 3000, 100, 10, (1, 8, 32, 128)),
            (b.BS_F32, 4096, 4096, 64, 32, (1, 8)),
            (b.BS_F16, 4096, 25088, 64, 6, (1, 16)),
            (b.BS_F32, 16384, 8192, 256, 128, (1, 8)),
            (b.BS_F32, 16384, 8192, 256, 8, (8,)),
            (b.BS_F32, 512, 4608, 64, 16, (196, 784)),
            (b.BS_F32, 128, 576, 64, 16, (12544,))]:
        for N in Ns:
            seen.add(_plan_invariants(b, dtype, M, K, bank, k, N)["rows_kernel"])
    assert seen == {0, 1}       # both kernels are in use on these shapes


def test_spmm_plan_invariants_random_shapes():
    import random
    from paper_1811_00206_amd import binding as b
    rng = random.Random(1811_00206)
    done = 0
    for _ in range(4000):
        bank = rng.choice([1, 2, 3, 4, 5, 8, 16, 25, 32, 50, 64, 100, 128, 200, 255, 256])
        nb = rng.choice([1, 2, 3, 7, 30, 32, 64, 100, 392, 1000])
        k = rng.randint(1, bank)
        M = rng.choice([1, 2, 63, 64, 65, 500, 1000, 4096, 6000, 16384, 100000])
        N = rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 17, 31, 32, 33, 64, 100, 128, 196, 784, 1000, 12544])
        dtype = rng.choice([b.BS_F32, b.BS_F16])
        try:
            _plan_invariants(b, dtype, M, bank * nb, bank, k, N)
            done += 1
        except b.BsError as e:                       # a documented refusal, never a bad plan
            assert "unsupported" in str(e), (dtype, M, bank * nb, bank, k, N, str(e))
    assert done > 3000


def test_spmv_plan_invariants_on_the_paper_shapes_and_random_ones():
    """What spmv_kernel assumes about its launch, checked on the host: whole wavefronts, a row's
    lanes inside one wavefront, every row in exactly one workgroup, LDS within a compute unit's."""
    import random
    from paper_1811_00206_amd import binding as b
    rng = random.Random(181100206)
    shapes = [(b.BS_F32, 256, 256, 64, 16), (b.BS_F32, 6000, 3000, 100, 10), (b.BS_F32, 4096, 4096, 64, 32),
              (b.BS_F32, 4096, 4096, 64, 2), (b.BS_F16, 4096, 25088, 64, 6), (b.BS_F32, 16384, 8192, 256, 128),
              (b.BS_F32, 6000, 3000, 25, 10), (b.BS_F32, 4096, 2048, 64, 8), (b.BS_F32, 1, 4, 4, 4)]
    for _ in range(3000):
        bank = rng.choice([1, 2, 3, 4, 5, 8, 16, 25, 32, 50, 64, 100, 128, 200, 255, 256])
        nb = rng.choice([1, 2, 3, 7, 30, 32, 64, 100, 160, 392, 1000])
        if bank * nb > 40960:
            continue
        shapes.append((rng.choice([b.BS_F32, b.BS_F16]), rng.choice([1, 2, 63, 64, 65, 500, 4096, 6000, 16384, 100000]),
                       bank * nb, bank, rng.randint(1, bank)))
    for dtype, M, K, bank, k in shapes:
        p = b.bs_spmv_plan(dtype, M, K, bank, k)
        where = f"{(dtype, M, K, bank, k)} -> {p}"
        assert p["slab_kernel"] == 0, where
        vsize = 2 if dtype == b.BS_F16 else 4
        row_len = K // bank * k
        assert p["ch"] in (1, 2, 4, 8) and p["ch"] * vsize <= 16 and row_len % p["ch"] == 0, where
        assert p["lpr"] in (1, 2, 4, 8, 16, 32, 64) and 2 <= p["u"] <= 8, where
        assert p["threads"] == p["lpr"] * p["rows_per_wg"] and p["threads"] % 64 == 0 and 64 <= p["threads"] <= 1024, where
        assert (p["workgroups"] - 1) * p["rows_per_wg"] < M <= p["workgroups"] * p["rows_per_wg"], where
        x_bytes = (K + 3) // 4 * 16
        assert p["lds_bytes"] == x_bytes + (row_len * 4 if p["table"] else 0) <= 160 * 1024, where
        assert p["bank_mode"] == (0 if k % p["ch"] == 0 else 1 if k >= p["ch"] else 2), where
    # x beyond one compute unit's LDS: the slab kernel, and no launch-shape overrides there
    assert b.bs_spmv_plan(b.BS_F32, 70, 65536, 256, 16)["slab_kernel"] == 1
    with pytest.raises(b.BsError):
        b.bs_spmv_plan(b.BS_F32, 70, 65536, 256, 16, 64, 4)
    with pytest.raises(b.BsError):
        b.bs_spmv_plan(b.BS_F32, 64, 256, 64, 16, 3, 0)        # lanes per row not a power of two
