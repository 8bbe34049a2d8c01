"""GPU parity: the HIP path, called through the C-ABI binding, against the CPU
oracle on the same seeded inputs.  vals/idx must match bit for bit; products
must stay within 1e-5 relative L2 (fp32 storage) or 1e-2 (fp16 storage)."""
import numpy as np
import pytest
import torch

from oracle import bs_ref
from paper_1811_00206_amd import binding as bs
from paper_1811_00206_amd import probe
from paper_1811_00206_amd import workloads

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "f16": 1e-2}
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def say(*a):
    print(*a, flush=True)


def check_pack(W, bank, k):
    v_ref, i_ref = bs_ref.prune_pack(W, bank, k)
    v, i = bs.bs_prune_pack(dev(W), bank, k)
    v, i = host(v), host(i)
    assert i.shape == i_ref.shape and v.dtype == v_ref.dtype
    assert i.tobytes() == i_ref.tobytes(), "idx differs"
    assert v.tobytes() == v_ref.tobytes(), "vals differ"
    return v_ref, i_ref


SMALL_SHAPES = [(7, 64, 16, 4), (5, 300, 100, 10), (3, 256, 64, 1), (4, 96, 32, 31),
                (2, 512, 256, 13), (9, 30, 3, 2), (1, 128, 128, 5), (6, 40, 1, 1),
                (33, 520, 130, 7), (17, 768, 192, 192), (1, 4, 4, 4), (257, 200, 100, 99),
                (1000, 64, 64, 64), (3, 2048, 256, 255)]


# ------------------------------------------------------------ prune + pack

@pytest.mark.parametrize("M,K,bank,k", SMALL_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_prune_pack_small(M, K, bank, k, dtype):
    say("prune_pack small", M, K, bank, k, dtype)
    W = workloads.draw_weights(M, K, 1.0, dtype, 31)
    check_pack(W, bank, k)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("levels", [1, 2, 3, 5])
def test_prune_pack_ties(dtype, levels):
    say("prune_pack ties", dtype, levels)
    W = workloads.tie_heavy_weights(64, 1024, levels, dtype, 32)
    for bank, k in [(64, 16), (32, 5), (256, 100), (4, 2), (128, 127), (1, 1), (64, 64)]:
        check_pack(W, bank, k)


def test_prune_pack_special_values():
    # signed zeros, subnormals, largest finite; all-zero banks
    W = np.zeros((4, 128), dtype=np.float32)
    W[0, ::3] = -0.0
    W[1, :] = np.float32(1e-45)
    W[1, 5] = -np.float32(1e-45) * 3
    W[2, :] = np.finfo(np.float32).max
    W[2, ::2] *= -1
    W[3, :] = np.linspace(-1, 1, 128, dtype=np.float32)
    for bank, k in [(128, 7), (64, 32), (32, 1)]:
        check_pack(W, bank, k)
    Wh = W.astype(np.float16)
    Wh[2, :] = np.float16(65504)
    Wh[1, :] = np.array([0x0001], dtype=np.uint16).view(np.float16)[0]
    for bank, k in [(128, 7), (64, 32), (32, 1)]:
        check_pack(Wh, bank, k)


@pytest.mark.parametrize("M,K,bank,k", SMALL_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_reprune_small(M, K, bank, k, dtype):
    """Every k2 from 1 to k: bit-exact against the oracle's re-prune (which is pinned to
    the one-shot prune of the dense matrix)."""
    say("reprune", M, K, bank, k, dtype)
    W = workloads.draw_weights(M, K, 1.0, dtype, 61)
    v, i = bs_ref.prune_pack(W, bank, k)
    vals, idx = dev(v), dev(i)
    for k2 in sorted({1, 2, 3, max(1, k // 2), max(1, k - 1), k} & set(range(1, k + 1))):
        v2, i2 = bs.bs_reprune(vals, idx, bank, k2)
        v_ref, i_ref = bs_ref.reprune(v, i, k2)
        assert host(v2).tobytes() == v_ref.tobytes(), (k2,)
        assert host(i2).tobytes() == i_ref.tobytes(), (k2,)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_reprune_ties(dtype):
    W = workloads.tie_heavy_weights(33, 512, 3, dtype, 62)
    for bank, k, k2 in [(64, 24, 8), (128, 40, 13), (32, 32, 5), (256, 100, 31)]:
        v, i = bs_ref.prune_pack(W, bank, k)
        v2, i2 = bs.bs_reprune(dev(v), dev(i), bank, k2)
        v_ref, i_ref = bs_ref.reprune(v, i, k2)
        assert host(v2).tobytes() == v_ref.tobytes() and host(i2).tobytes() == i_ref.tobytes()


@pytest.mark.parametrize("name,k2", [("lstm1500", 5), ("sweep_k32", 8), ("fc6_b1", 3)])
def test_reprune_full_size(name, k2):
    """At full size the re-pruned matrix must be what pruning W to k2 directly gives
    (checked on the GPU's own one-shot result, itself checked against the oracle in
    test_full_size_pack_and_spmv) and what the oracle gives on a sample of rows."""
    say("reprune full", name, k2)
    wl, W, _ = workloads.make(name)
    Wd = dev(W)
    vals, idx = bs.bs_prune_pack(Wd, wl.bank, wl.k)
    v2, i2 = bs.bs_reprune(vals, idx, wl.bank, k2)
    v1, i1 = bs.bs_prune_pack(Wd, wl.bank, k2)
    assert torch.equal(v2.view(torch.uint8), v1.view(torch.uint8)) and torch.equal(i2, i1)
    rows = np.arange(0, wl.M, 97)
    v_ref, i_ref = bs_ref.reprune(*bs_ref.prune_pack(np.ascontiguousarray(W[rows]), wl.bank, wl.k), k2)
    rsel = torch.from_numpy(rows).to(v2.device)
    assert host(v2[rsel]).tobytes() == v_ref.tobytes() and host(i2[rsel]).tobytes() == i_ref.tobytes()


FULL = ["tiny", "lstm1500", "sweep_k32", "sweep_k16", "sweep_k8", "sweep_k4", "sweep_k2",
        "fc6_b1", "lstm1500_b25_k5", "lstm1500_b50_k15", "lstm1500_b100_k40",
        # the rest of Table 4's axes and Sec. 4.3's second model as a plain product
        "lstm1500_b25_k10", "lstm1500_b50_k20", "lstm1500_b50_k10", "lstm1500_b100_k30",
        "lstm1500_b100_k20", "bilstm1024"]


def assert_close(y, y_ref, tol, what=""):
    """Relative L2 and element by element (a single wrong row hides in an L2 norm)."""
    err = bs_ref.rel_l2(y, y_ref)
    worst = float(np.abs(y.astype(np.float64) - y_ref).max())
    scale = float(np.abs(y_ref).max()) + 1e-30
    say(f"  {what} relL2 {err:.3g}, max |err| / max |ref| {worst / scale:.3g}")
    assert err <= tol, (what, err)
    assert worst <= tol * scale, (what, worst, scale)


@pytest.mark.parametrize("name", FULL)
def test_full_size_pack_and_spmv(name):
    """The five configurations at full size: pack bit-exact, product in tolerance,
    in the launch shape the bench times (the default one)."""
    say("full", name)
    wl, W, x = workloads.make(name)
    v_ref, i_ref = check_pack(W, wl.bank, wl.k)
    y_ref = bs_ref.spmv(v_ref, i_ref, wl.bank, x, threads=bs_ref.host_threads())
    vals, idx = dev(v_ref), dev(i_ref)
    y = bs.bs_spmv(vals, idx, wl.bank, dev(x))
    assert_close(host(y), y_ref, TOL[wl.dtype], "spmv " + name)
    # bit-reproducible from call to call
    y2 = bs.bs_spmv(vals, idx, wl.bank, dev(x))
    assert host(y).tobytes() == host(y2).tobytes()


# ------------------------------------------------------------------- SpMV

@pytest.mark.parametrize("M,K,bank,k", SMALL_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_spmv_small(M, K, bank, k, dtype):
    say("spmv small", M, K, bank, k, dtype)
    W = workloads.draw_weights(M, K, 0.05, dtype, 33)
    x = workloads.draw_activations(K, 1, 33)
    v, i = bs_ref.prune_pack(W, bank, k)
    y_ref = bs_ref.spmv(v, i, bank, x)
    y = host(bs.bs_spmv(dev(v), dev(i), bank, dev(x)))
    assert bs_ref.rel_l2(y, y_ref) <= TOL[dtype]
    # element by element as well (a single wrong row hides in an L2 norm)
    scale = np.abs(y_ref).max() + 1e-30
    assert np.abs(y - y_ref).max() <= (1e-5 if dtype == "f32" else 1e-2) * scale


@pytest.mark.parametrize("lanes", [1, 2, 4, 8, 16, 32, 64])
def test_spmv_every_launch_shape(lanes):
    say("spmv launch shapes", lanes)
    for name, rows in [("tiny", None), ("lstm1500", 1000)]:
        wl, W, x = workloads.make(name, rows=rows)
        v, i = bs_ref.prune_pack(W, wl.bank, wl.k)
        y_ref = bs_ref.spmv(v, i, wl.bank, x)
        vd, idd, xd = dev(v), dev(i), dev(x)
        for threads in (64, 256, 1024):
            y = host(bs.bs_spmv_ex(vd, idd, wl.bank, xd, lanes, threads // lanes))
            assert bs_ref.rel_l2(y, y_ref) <= 1e-5, (name, lanes, threads)


def test_spmv_largest_x_that_fits_lds_and_beyond():
    K = 40960                      # 160 KB of fp32: the whole LDS of a compute unit
    say("spmv K", K)
    W = workloads.draw_weights(48, K, 1.0, "f32", 34)
    x = workloads.draw_activations(K, 1, 34)
    v, i = bs_ref.prune_pack(W, 256, 3)
    y = host(bs.bs_spmv(dev(v), dev(i), 256, dev(x)))
    assert bs_ref.rel_l2(y, bs_ref.spmv(v, i, 256, x)) <= 1e-5
    # one bank more: x no longer fits, the product walks x in slabs
    K2 = K + 256
    say("spmv K", K2)
    W2 = workloads.draw_weights(48, K2, 1.0, "f32", 35)
    x2 = workloads.draw_activations(K2, 1, 35)
    v2, i2 = bs_ref.prune_pack(W2, 256, 3)
    y2 = host(bs.bs_spmv(dev(v2), dev(i2), 256, dev(x2)))
    assert bs_ref.rel_l2(y2, bs_ref.spmv(v2, i2, 256, x2)) <= 1e-5
    # ... but neither launch-shape overrides nor the fused LSTM step exist there
    with pytest.raises(bs.BsError) as e:
        bs.bs_spmv_ex(dev(v2), dev(i2), 256, dev(x2), 64, 4)
    assert e.value.status == 3


@pytest.mark.parametrize("M,K,bank,k,dtype,mode", [
    (16, 36864, 64, 8, "f32", 0),         # a chunk never leaves its bank
    (16, 38400, 100, 10, "f32", 1),       # a chunk touches at most two banks
    (8, 40960, 128, 24, "f16", 0),
    (12, 40000, 100, 3, "f32", 2),        # several banks per chunk
    (5, 40960, 64, 3, "f16", 2),
    (9, 39936, 96, 9, "f16", 1),
])
def test_spmv_without_bank_table(M, K, bank, k, dtype, mode):
    """x fills LDS so far that the per-entry bank table no longer fits: banks are then found by
    arithmetic, in one of three ways depending on k and the chunk width."""
    say("spmv without table", M, K, bank, k, dtype)
    plan = bs.bs_spmv_plan(bs.BS_F16 if dtype == "f16" else bs.BS_F32, M, K, bank, k)
    assert plan["slab_kernel"] == 0 and plan["table"] == 0 and plan["bank_mode"] == mode, plan
    W = workloads.draw_weights(M, K, 1.0, dtype, 38)
    x = workloads.draw_activations(K, 1, 38)
    v, i = bs_ref.prune_pack(W, bank, k)
    y = host(bs.bs_spmv(dev(v), dev(i), bank, dev(x)))
    y_ref = bs_ref.spmv(v, i, bank, x)
    Wp = bs_ref.unpack(v, i, bank).astype(np.float64)
    scale = (np.abs(Wp) @ np.abs(x.astype(np.float64))).max() + 1e-300
    assert np.abs(y - y_ref).max() <= TOL[dtype] * scale
    assert bs_ref.rel_l2(y, y_ref) <= 10 * TOL[dtype]      # a dozen outputs: cancellation in the norm


@pytest.mark.gpu
@pytest.mark.parametrize("M,K,bank,k,dtype", [
    (70, 65536, 256, 16, "f32"),          # 4 slabs of whole banks, 16-byte chunks
    (133, 50000, 100, 7, "f32"),          # chunks of 4 entries cross banks; ragged last slab
    (5, 49152, 64, 3, "f16"),             # 8-entry chunks: slabs of a multiple of 8 banks
    (9, 41003, 131, 5, "f32"),            # odd everything: 1-entry chunks, K % 4 != 0
    (1, 262144, 256, 256, "f16"),         # one dense row of 512 KB of x
    (300, 81920, 2, 1, "f32"),            # 40960 banks of two
    (17, 89030, 2, 1, "f16"),             # slab and table fill LDS to the last 16 bytes
])
def test_spmv_x_larger_than_lds(M, K, bank, k, dtype):
    say("spmv slabs", M, K, bank, k, dtype)
    W = workloads.draw_weights(M, K, 1.0, dtype, 36)
    x = workloads.draw_activations(K, 1, 36)
    v, i = bs_ref.prune_pack(W, bank, k)
    y = host(bs.bs_spmv(dev(v), dev(i), bank, dev(x)))
    Wp = bs_ref.unpack(v, i, bank).astype(np.float64)
    scale = (np.abs(Wp) @ np.abs(x.astype(np.float64))).max() + 1e-300
    assert np.abs(y - bs_ref.spmv(v, i, bank, x)).max() <= 1e-5 * scale
    assert bs_ref.rel_l2(y, bs_ref.spmv(v, i, bank, x)) <= (1e-5 if M > 8 else 1e-4)


# ------------------------------------------------------------------- SpMM

def check_spmm(W, bank, k, X, tol):
    v, i = bs_ref.prune_pack(W, bank, k)
    Y_ref = bs_ref.spmm(v, i, bank, X, threads=bs_ref.host_threads())
    Y = host(bs.bs_spmm(dev(v), dev(i), bank, dev(X)))
    err = bs_ref.rel_l2(Y, Y_ref)
    say("  spmm relL2", err)
    assert err <= tol
    scale = np.abs(Y_ref).max() + 1e-30
    assert np.abs(Y - Y_ref).max() <= tol * scale
    return v, i, Y


@pytest.mark.parametrize("M,K,bank,k", SMALL_SHAPES)
@pytest.mark.parametrize("N", [1, 2, 3, 4, 7, 8, 16, 20, 33, 64, 130])
def test_spmm_small(M, K, bank, k, N):
    say("spmm small", M, K, bank, k, N)
    W = workloads.draw_weights(M, K, 0.05, "f32", 35)
    X = workloads.draw_activations(K, N, 35).reshape(K, N)
    check_spmm(W, bank, k, X, 1e-5)


@pytest.mark.parametrize("name", ["lstm1500_n8", "lstm1500_n32", "lstm1500_n128", "fc6_b16",
                                  "conv5_n196", "conv4_n784", "conv2_n12544", "conv1_n50176"])
def test_spmm_full_size(name):
    say("spmm full", name)
    wl, W, X = workloads.make(name)
    v, i, Y = check_spmm(W, wl.bank, wl.k, X, TOL[wl.dtype])
    Y2 = host(bs.bs_spmm(dev(v), dev(i), wl.bank, dev(X)))
    assert Y.tobytes() == Y2.tobytes()      # slab sums are added in a fixed order


@pytest.mark.parametrize("name", ["bench16k_k128", "bench16k_k64", "bench16k_k32", "bench16k_k16",
                                  "bench16k_k8", "bench16k_k128_n8", "bench16k_k32_n8",
                                  "bench16k_k8_n8"])
def test_benchmark_shape_sampled_rows(name):
    """Sec. 4.1's 16384 x 8192 matrix (32 banks of 256 per row) in the launch shape the
    bench times: the GPU packs and multiplies the whole matrix, the oracle does the
    rows of a spread sample one by one (the quadratic rank count over 134 M elements
    would take minutes); rows are independent, so a row's result does not depend on
    which other rows are present."""
    say("benchmark shape", name)
    wl, W, X = workloads.make(name)
    rows = np.unique(np.concatenate([np.arange(0, wl.M, 257), [1, 63, 64, wl.M - 2, wl.M - 1]]))
    Ws = np.ascontiguousarray(W[rows])
    v_ref, i_ref = bs_ref.prune_pack(Ws, wl.bank, wl.k)
    vals, idx = bs.bs_prune_pack(dev(W), wl.bank, wl.k)
    rsel = torch.from_numpy(rows).to(vals.device)
    assert host(vals[rsel]).tobytes() == v_ref.tobytes()
    assert host(idx[rsel]).tobytes() == i_ref.tobytes()
    if wl.N == 1:
        y_ref = bs_ref.spmv(v_ref, i_ref, wl.bank, X)
        y = host(bs.bs_spmv(vals, idx, wl.bank, dev(X)))[rows]
    else:
        y_ref = bs_ref.spmm(v_ref, i_ref, wl.bank, X)
        y = host(bs.bs_spmm(vals, idx, wl.bank, dev(X)))[rows]
    assert_close(y, y_ref, TOL[wl.dtype], f"{name} on {len(rows)} rows")


def _oracle_pack_rows(args):
    W_rows, bank, k = args
    return bs_ref.prune_pack(W_rows, bank, k)


@pytest.mark.timeout(900)
def test_benchmark_shape_pack_every_row():
    """Sec. 4.1's 16384 x 8192 matrix at 87.5 %: vals/idx of EVERY row against the oracle.  The
    oracle's pruning is row-independent, so the rows are split over worker processes, each
    running the unchanged single-threaded oracle on its share."""
    import concurrent.futures as cf
    import multiprocessing as mp
    name = "bench16k_k32"
    say("benchmark shape, every row", name)
    wl, W, _ = workloads.make(name)
    vals, idx = bs.bs_prune_pack(dev(W), wl.bank, wl.k)
    v_gpu, i_gpu = host(vals), host(idx)
    workers = max(1, min(16, bs_ref.host_threads()))
    bounds = np.linspace(0, wl.M, 4 * workers + 1).astype(int)
    jobs = [(np.ascontiguousarray(W[a:b]), wl.bank, wl.k) for a, b in zip(bounds[:-1], bounds[1:])]
    with cf.ProcessPoolExecutor(workers, mp_context=mp.get_context("spawn")) as ex:
        parts = list(ex.map(_oracle_pack_rows, jobs))
    for (a, b), (v_ref, i_ref) in zip(zip(bounds[:-1], bounds[1:]), parts):
        assert i_gpu[a:b].tobytes() == i_ref.tobytes(), f"idx differs in rows {a}..{b}"
        assert v_gpu[a:b].tobytes() == v_ref.tobytes(), f"vals differ in rows {a}..{b}"


@pytest.mark.parametrize("N,ldx,ldy,col0", [(8, 12, 24, 4), (33, 40, 37, 0), (64, 68, 64, 4),
                                            (5, 7, 9, 0), (130, 136, 132, 0), (16, 21, 16, 4)])
def test_spmm_leading_dimensions(N, ldx, ldy, col0):
    """X and Y as column slices of wider row-major buffers (ldx, ldy > N): the product
    reads only its N columns and writes only its N columns."""
    M, K, bank, k = 70, 600, 100, 10
    W = workloads.draw_weights(M, K, 0.05, "f32", 71)
    v, i = bs_ref.prune_pack(W, bank, k)
    X = workloads.draw_activations(K, N, 71).reshape(K, N)
    Xw = torch.full((K, ldx + col0), float("nan"), device=DEV)      # poison around the slice
    Xs = Xw[:, col0:col0 + N]
    Xs.copy_(dev(X))
    Yw = torch.full((M, ldy), -7.0, device=DEV)
    Ys = Yw[:, :N]
    bs.bs_spmm(dev(v), dev(i), bank, Xs, out=Ys)
    Y = host(Ys.contiguous())
    assert bs_ref.rel_l2(Y, bs_ref.spmm(v, i, bank, X)) <= 1e-5
    assert bool((Yw[:, N:] == -7.0).all())                           # padding untouched
    if ldx > N + 1:   # a slice that does not start on a 16-byte boundary is refused
        with pytest.raises(bs.BsError) as e:
            bs.bs_spmm(dev(v), dev(i), bank, Xw[:, 1:1 + N], out=Ys)
        assert e.value.status == 4


def test_spmm_n1_matches_spmv_and_f16_small():
    wl, W, x = workloads.make("tiny")
    v, i = bs_ref.prune_pack(W, wl.bank, wl.k)
    Y = host(bs.bs_spmm(dev(v), dev(i), wl.bank, dev(x.reshape(-1, 1))))
    assert bs_ref.rel_l2(Y[:, 0], bs_ref.spmv(v, i, wl.bank, x)) <= 1e-5
    Wh = workloads.draw_weights(50, 1024, 0.01, "f16", 36)
    X = workloads.draw_activations(1024, 16, 36)
    check_spmm(Wh, 64, 6, X, 1e-2)


def test_spmm_workspace_contract():
    wl, W, X = workloads.make("lstm1500_n128", rows=64)
    v, i = bs_ref.prune_pack(W, wl.bank, wl.k)
    need = bs.bs_spmm_workspace_bytes(bs.BS_F32, 64, wl.K, wl.bank, wl.k, wl.N)
    assert need > 0
    small = torch.empty(need - 16, dtype=torch.uint8, device=DEV)
    with pytest.raises(bs.BsError) as e:
        bs.bs_spmm(dev(v), dev(i), wl.bank, dev(X), workspace=small)
    assert e.value.status == 6
    ws = bs.new_spmm_workspace(need, DEV)
    ws.fill_(255)                                   # a workspace needs no initialisation
    Y_ref = bs_ref.spmm(v, i, wl.bank, X)
    for _ in range(3):                              # and is reusable as a call leaves it
        Y = host(bs.bs_spmm(dev(v), dev(i), wl.bank, dev(X), workspace=ws))
        assert bs_ref.rel_l2(Y, Y_ref) <= 1e-5
    # ... also by a product of another shape
    wl2, W2, X2 = workloads.make("fc6_b16", rows=96)
    v2, i2 = bs_ref.prune_pack(W2, wl2.bank, wl2.k)
    assert 0 < bs.bs_spmm_workspace_bytes(bs.BS_F16, 96, wl2.K, wl2.bank, wl2.k, wl2.N) <= need
    Y2 = host(bs.bs_spmm(dev(v2), dev(i2), wl2.bank, dev(X2), workspace=ws))
    assert bs_ref.rel_l2(Y2, bs_ref.spmm(v2, i2, wl2.bank, X2)) <= 1e-2
    Y = host(bs.bs_spmm(dev(v), dev(i), wl.bank, dev(X), workspace=ws))
    assert bs_ref.rel_l2(Y, Y_ref) <= 1e-5


# ------------------------------------------------------- dense baselines

# ------------------------------------------------------------------- LSTM step

def check_lstm(W, bank, k, H, I, T, seed, tol):
    v, i = bs_ref.prune_pack(W, bank, k)
    X, h0, c0, bias = workloads.draw_lstm_inputs(H, I, T, seed)
    H_ref, c_ref = bs_ref.lstm_sequence(v, i, bank, X, h0, bias, c0)
    vals, idx = dev(v), dev(i)
    # one step through bs_lstm_step ...
    c1, h1 = bs.bs_lstm_step(vals, idx, bank, dev(X[0]), dev(h0), dev(bias), dev(c0))
    c1_ref, h1_ref = bs_ref.lstm_step(v, i, bank, X[0], h0, bias, c0)
    assert bs_ref.rel_l2(host(c1), c1_ref) <= tol
    assert bs_ref.rel_l2(host(h1), h1_ref) <= tol
    assert np.abs(host(h1) - h1_ref).max() <= tol * 4      # |h| <= 1
    # ... and the whole sequence, cell state updated in place
    c = dev(c0)
    H_all = bs.bs_lstm_sequence(vals, idx, bank, dev(X), dev(h0), dev(bias), c)
    e_h, e_c = bs_ref.rel_l2(host(H_all).ravel(), H_ref.ravel()), bs_ref.rel_l2(host(c), c_ref)
    say("  lstm", W.shape, bank, k, "T", T, "relL2 h", e_h, "c", e_c)
    assert e_h <= tol and e_c <= tol
    assert host(H_all)[0].tobytes() == host(h1).tobytes()      # same kernel, same order
    return e_h


@pytest.mark.parametrize("H,I,bank,k", [(8, 24, 16, 3), (12, 20, 8, 8), (4, 12, 4, 1),
                                        (36, 64, 100, 10), (100, 60, 32, 5), (64, 448, 256, 77)])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_lstm_small(H, I, bank, k, dtype):
    say("lstm small", H, I, bank, k, dtype)
    W = workloads.draw_weights(4 * H, I + H, 0.3, dtype, 41)
    check_lstm(W, bank, k, H, I, 5, 41, TOL[dtype])


@pytest.mark.parametrize("name,H,I", [("lstm1500", 1500, 1500), ("bilstm1024", 1024, 1024)])
def test_lstm_full_size(name, H, I):
    """The recurrent models of Sec. 4.3 at full size, four steps."""
    say("lstm full", name)
    wl, W, _ = workloads.make(name)
    assert wl.M == 4 * H and wl.K == I + H
    check_lstm(W, wl.bank, wl.k, H, I, 4, wl.seed, TOL[wl.dtype])


def test_lstm_refused_arguments():
    H, I, bank, k = 8, 24, 16, 3
    W = workloads.draw_weights(4 * H, I + H, 0.3, "f32", 42)
    v, i = bs_ref.prune_pack(W, bank, k)
    X, h0, c0, bias = workloads.draw_lstm_inputs(H, I, 1, 42)
    vals, idx, x, h, b, c = dev(v), dev(i), dev(X[0]), dev(h0), dev(bias), dev(c0)
    with pytest.raises(bs.BsError):      # hidden state updated in place: refused
        bs.bs_lstm_step(vals, idx, bank, x, h, b, c, h_out=h)
    # sizes that are not multiples of 4 are refused, not mis-computed
    W2 = workloads.draw_weights(4 * 6, 10 + 6, 0.3, "f32", 43)
    v2, i2 = bs_ref.prune_pack(W2, 8, 2)
    X2, h2, c2, b2 = workloads.draw_lstm_inputs(6, 10, 1, 43)
    with pytest.raises(bs.BsError):
        bs.bs_lstm_step(dev(v2), dev(i2), 8, dev(X2[0]), dev(h2), dev(b2), dev(c2))


def close_to_scale(Y, Y_ref, W, X, tol):
    """|error| <= tol * max_r sum_c |w_rc| |x_c|: an fp32 sum can lose that much
    when terms cancel, so tiny outputs are judged against the size of the terms."""
    scale = (np.abs(W.astype(np.float64)) @ np.abs(X.astype(np.float64))).max() + 1e-300
    return np.abs(Y.astype(np.float64) - Y_ref).max() <= tol * scale


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("M,K", [(37, 300), (64, 1024), (130, 77), (1, 8)])
def test_dense_baselines(dtype, M, K):
    say("dense", dtype, M, K)
    W = workloads.draw_weights(M, K, 0.05, dtype, 37)
    x = workloads.draw_activations(K, 1, 37)
    y_ref = bs_ref.dense_gemm_f64(W, x)
    y = host(bs.bs_dense_gemv(dev(W), dev(x)))
    assert close_to_scale(y, y_ref, W, x, 1e-5)
    if M > 8:
        assert bs_ref.rel_l2(y, y_ref.astype(np.float32)) <= 1e-5
    for N in (1, 8, 20, 32, 100):
        X = workloads.draw_activations(K, N, 38).reshape(K, N)
        Y_ref = bs_ref.dense_gemm_f64(W, X)
        Y = host(bs.bs_dense_gemm(dev(W), dev(X)))
        assert close_to_scale(Y, Y_ref, W, X, 1e-5), N
        if M > 8:
            assert bs_ref.rel_l2(Y, Y_ref.astype(np.float32)) <= 1e-5, N


def test_sparse_product_equals_dense_product_of_pruned_matrix_on_gpu():
    """Eq. (2): the pruned layer is W_p . X; both GPU paths agree on it."""
    wl, W, x = workloads.make("lstm1500", rows=512)
    v, i = bs_ref.prune_pack(W, wl.bank, wl.k)
    Wp = bs_ref.unpack(v, i, wl.bank)
    y_s = host(bs.bs_spmv(dev(v), dev(i), wl.bank, dev(x)))
    y_d = host(bs.bs_dense_gemv(dev(Wp), dev(x)))
    assert bs_ref.rel_l2(y_s, y_d) <= 1e-5


# ----------------------------------------------------- errors via the C-ABI

def test_measurement_helpers_run_and_refuse_bad_sizes():
    """The benchmark's helper kernels (a library of their own, not the product's)."""
    buf = torch.ones(1 << 20, dtype=torch.uint8, device=DEV)
    probe.probe_empty(4, 64)
    probe.probe_stream_read(buf)
    for pieces in (1, 2, 4, 8):
        probe.probe_stream_read(buf, pieces)
    probe.probe_stream_read(buf[:4096], sink=torch.zeros(64, dtype=torch.int32, device=DEV))
    sink = torch.zeros((1 << 20) // 128 + 1, dtype=torch.int32, device=DEV)
    for mode in (1, 2, 3):
        probe.probe_stream_read(buf, 1, sink=sink, store_mode=mode, store_every=8)
        probe.probe_stream_read(buf, 1, sink=sink, store_mode=mode, store_every=94)
    torch.cuda.synchronize()
    assert bool((buf == 1).all())
    with pytest.raises(probe.ProbeError):
        probe.probe_stream_read(buf[:24])            # not a multiple of 16 bytes
    with pytest.raises(probe.ProbeError):
        probe.probe_stream_read(buf, 3)
    with pytest.raises(probe.ProbeError):
        probe.probe_empty(0, 256)
    with pytest.raises(probe.ProbeError):
        probe.probe_empty(4, 100)
    probe.probe_lds_gather(256, 0, 16, 64)
    probe.probe_lds_gather(768, 1, 8, 64)
    probe.probe_lds_gather(1024, 1, 2, 8)
    probe.probe_lds_gather(768, 2, 16, 64)
    probe.probe_lds_gather(768, 3, 16, 64)
    torch.cuda.synchronize()
    with pytest.raises(probe.ProbeError):
        probe.probe_lds_gather(768, 1, 3, 64)        # group of lanes not 2, 4, 8 or 16
    with pytest.raises(probe.ProbeError):
        probe.probe_lds_gather(768, 1, 8, 60)        # reads not a multiple of 8
    # the grid-barrier loop ends by itself: all arrivals counted, or (with a wait of one poll,
    # forced here from the host) the abort flag raised and every workgroup gone
    hbuf = torch.zeros(2 * 1500, device=DEV)
    for mode in (0, 1):
        sync = torch.zeros(4, dtype=torch.int32, device=DEV)
        probe.probe_grid_barrier(64, 256, 50, 1500, mode, sync, hbuf)
        torch.cuda.synchronize()
        assert sync[:2].tolist() == [50 * 64, 0]
    sync = torch.zeros(4, dtype=torch.int32, device=DEV)
    probe.probe_grid_barrier(256, 1024, 200, 1500, 0, sync, hbuf, spin_limit=1)
    torch.cuda.synchronize()
    arrivals, aborted = sync[:2].tolist()
    assert aborted in (0, 1) and arrivals <= 200 * 256 and (aborted or arrivals == 200 * 256)


def test_init_is_idempotent():
    bs.bs_init()
    bs.bs_init()


def test_device_side_argument_errors():
    v = torch.zeros((4, 2, 2), dtype=torch.float32, device=DEV)
    i = torch.zeros((4, 2, 2), dtype=torch.uint8, device=DEV)
    x = torch.zeros(8, device=DEV)
    with pytest.raises(ValueError):
        bs.bs_spmv(v, i, 4, torch.zeros(9, device=DEV))
    with pytest.raises(TypeError):
        bs.bs_spmv(v, i, 4, x.cpu())
    base = torch.zeros(64, device=DEV)
    with pytest.raises(bs.BsError) as e:           # x not 16-byte aligned
        bs.bs_spmv(v, i, 4, base[1:9])
    assert e.value.status == 4
    y = bs.bs_spmv(v, i, 4, x)
    assert host(y).tolist() == [0.0] * 4


# ------------------------------------------- the launch configuration bench.py times

@pytest.mark.gpu
def test_graph_replays_match_eager_launches():
    """bench.py times a captured graph of launches over rotating copies of the packed matrix.
    The whole path (prune+pack, SpMV, SpMM with its workspace and reduce kernel, a fused LSTM
    sequence) is captured once and replayed several times, with eager work and
    synchronisations between the replays; every replay must reproduce the eager results
    bit for bit (the kernels have a fixed summation order) and the eager results match the
    oracle."""
    say("graph replays")
    wl, W, x = workloads.make("lstm1500", rows=1200)          # 1200 x 3000: H = 300, I = 2700
    X = workloads.draw_activations(wl.K, 32, wl.seed + 5)
    Hn, T = 300, 5
    Xs, h0, c0, bias = workloads.draw_lstm_inputs(Hn, wl.K - Hn, T, wl.seed)
    v_ref, i_ref = bs_ref.prune_pack(W, wl.bank, wl.k)

    Wd, xd, Xd = dev(W), dev(x), dev(X)
    Xs_d, h0_d, bias_d = dev(Xs), dev(h0), dev(bias)
    copies = 3
    vals = [torch.empty((1200, wl.K // wl.bank, wl.k), dtype=torch.float32, device=DEV) for _ in range(copies)]
    idx = [torch.empty((1200, wl.K // wl.bank, wl.k), dtype=torch.uint8, device=DEV) for _ in range(copies)]
    y = [torch.empty(1200, device=DEV) for _ in range(copies)]
    Y = [torch.empty((1200, 32), device=DEV) for _ in range(copies)]
    need = bs.bs_spmm_workspace_bytes(bs.BS_F32, 1200, wl.K, wl.bank, wl.k, 32)
    ws = bs.new_spmm_workspace(need, DEV)
    c = torch.empty(Hn, device=DEV)
    c0_d = dev(c0)
    H_all = torch.empty((T, Hn), device=DEV)

    def run_all():
        for j in range(copies):
            bs.bs_prune_pack(Wd, wl.bank, wl.k, out=(vals[j], idx[j]))
            bs.bs_spmv(vals[j], idx[j], wl.bank, xd, out=y[j])
            bs.bs_spmm(vals[j], idx[j], wl.bank, Xd, out=Y[j], workspace=ws)
        c.copy_(c0_d)                                         # a copy kernel, no memset node
        bs.bs_lstm_sequence(vals[0], idx[0], wl.bank, Xs_d, h0_d, bias_d, c, H_all=H_all)

    def snapshot():
        torch.cuda.synchronize()
        return ([t.cpu().numpy().tobytes() for t in vals + idx + y + Y] +
                [c.cpu().numpy().tobytes(), H_all.cpu().numpy().tobytes()])

    def scribble():
        for t in vals + y + Y + [c, H_all]:
            t.fill_(7.0)
        for t in idx:
            t.fill_(7)
        ws.fill_(255)
        torch.cuda.synchronize()

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        run_all()                                             # eager, also warms every kernel up
    eager = snapshot()
    assert vals[0].cpu().numpy().tobytes() == v_ref.tobytes()
    assert idx[0].cpu().numpy().tobytes() == i_ref.tobytes()
    assert bs_ref.rel_l2(host(y[1]), bs_ref.spmv(v_ref, i_ref, wl.bank, x)) <= 1e-5
    assert bs_ref.rel_l2(host(Y[2]), bs_ref.spmm(v_ref, i_ref, wl.bank, X)) <= 1e-5
    H_ref, c_ref = bs_ref.lstm_sequence(v_ref, i_ref, wl.bank, Xs, h0, bias, c0)
    assert bs_ref.rel_l2(host(H_all), H_ref) <= 1e-5 and bs_ref.rel_l2(host(c), c_ref) <= 1e-5

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_all()
    for replay in range(4):
        scribble()                                            # eager work between the replays
        g.replay()
        assert snapshot() == eager, f"replay {replay} differs from the eager launches"


def test_first_use_inside_a_capture_is_refused_and_init_prevents_it():
    """The library raises a kernel's LDS limit at its first launch on a device, never while the
    stream is being captured: a first use inside a capture returns BS_ERR_NOT_INITIALISED (7)
    and enqueues nothing; after bs_init() the same capture works.  Run in a fresh process (one,
    on the same GPU), where no kernel has been used yet."""
    import subprocess
    import sys
    code = r'''
import numpy as np, torch
from oracle import bs_ref
from paper_1811_00206_amd import binding as bs, workloads
dev = "cuda:0"
W = workloads.draw_weights(64, 25088, 0.01, "f16", 5)          # x of 100 KB: a kernel that needs the raised limit
x = workloads.draw_activations(25088, 1, 5)
v, i = bs_ref.prune_pack(W, 64, 6)
vd, idd, xd = (torch.from_numpy(np.ascontiguousarray(t)).to(dev) for t in (v, i, x))
y = torch.empty(64, device=dev)
torch.zeros(1, device=dev); torch.cuda.synchronize()
def capture():
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        bs.bs_spmv(vd, idd, 64, xd, out=y)
    return g
try:
    capture()
    print("RESULT first capture unexpectedly worked")
except bs.BsError as e:
    print("RESULT refused with status", e.status)
torch.cuda.synchronize()
bs.bs_init()
g = capture()
y.fill_(0); g.replay(); torch.cuda.synchronize()
err = bs_ref.rel_l2(y.cpu().numpy(), bs_ref.spmv(v, i, 64, x))
print("RESULT after init relL2 ok", err <= 1e-2)
'''
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=240,
                         cwd=str(__import__("pathlib").Path(__file__).resolve().parent.parent))
    say(out.stdout[-600:], out.stderr[-600:])
    lines = [ln for ln in out.stdout.splitlines() if ln.startswith("RESULT")]
    assert out.returncode == 0, out.stderr[-2000:]
    assert lines == ["RESULT refused with status 7", "RESULT after init relL2 ok True"], lines
