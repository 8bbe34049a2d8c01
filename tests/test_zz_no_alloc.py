"""bs_spmm_static, the entry point for callers that cannot allocate: called through the
C ABI, its output must equal bs_spmm's (same kernels, same fixed summation order, so bit
for bit; bs_spmm itself is checked against the oracle) on two calls in a row, the second
with a smaller input, and the call must allocate no device memory."""
import numpy as np
import pytest
import torch

from oracle import bs_ref
from paper_1811_00206_amd import binding as bs
from paper_1811_00206_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _case(M, K, bank, k, N, dtype, seed):
    W = workloads.draw_weights(M, K, 0.05, dtype, seed)
    X = workloads.draw_activations(K, N, seed).reshape(K, N)
    v, i = bs_ref.prune_pack(W, bank, k)
    return v, i, X


def test_static_scratch_matches_workspace_entry_point_twice():
    print("bs_spmm_static: two calls, the second smaller", flush=True)
    # multi-slab shapes (the scratch is in use), then a smaller one that leaves most of the
    # previous call's partial sums in the array, then a one-slab shape (scratch unused)
    cases = [(1200, 3000, 100, 10, 128, "f32"), (600, 3000, 100, 10, 128, "f32"),
             (64, 25088, 64, 6, 16, "f16"), (256, 256, 64, 16, 8, "f32")]
    code = {"f32": bs.BS_F32, "f16": bs.BS_F16}
    prepared = []
    for n, (M, K, bank, k, N, dt) in enumerate(cases):
        v, i, X = _case(M, K, bank, k, N, dt, 90 + n)
        vd, idd, Xd = dev(v), dev(i), dev(X)
        need = bs.bs_spmm_workspace_bytes(code[dt], M, K, bank, k, N)
        assert need <= bs.bs_spmm_static_limit()
        ws = bs.new_spmm_workspace(need, DEV)
        Y_ws = bs.bs_spmm(vd, idd, bank, Xd, workspace=ws)
        Y_ref = bs_ref.spmm(v, i, bank, X)
        tol = 1e-5 if dt == "f32" else 1e-2
        assert bs_ref.rel_l2(Y_ws.cpu().numpy(), Y_ref) <= tol
        out = torch.full((M, N), float("nan"), device=DEV)
        prepared.append((need, vd, idd, bank, Xd, Y_ws, out))
        del ws
    assert prepared[0][0] > 0 and prepared[1][0] > 0 and prepared[1][0] < prepared[0][0]
    import gc
    gc.collect()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for need, vd, idd, bank, Xd, Y_ws, out in prepared:      # back to back on one stream
        bs.bs_spmm_static(vd, idd, bank, Xd, out)
    assert torch.cuda.memory_allocated() <= before           # nothing taken from torch's allocator
    torch.cuda.synchronize()
    for n, (need, vd, idd, bank, Xd, Y_ws, out) in enumerate(prepared):
        assert torch.equal(out, Y_ws), f"case {n}: bs_spmm_static differs from bs_spmm"
    # once more in the other order: every call overwrites what it reads from the array
    for need, vd, idd, bank, Xd, Y_ws, out in reversed(prepared):
        out.fill_(float("nan"))
        bs.bs_spmm_static(vd, idd, bank, Xd, out)
    torch.cuda.synchronize()
    for n, (need, vd, idd, bank, Xd, Y_ws, out) in enumerate(prepared):
        assert torch.equal(out, Y_ws), f"case {n}, second round"


def test_static_scratch_refuses_products_over_its_limit():
    # 3 slabs x 6000 x 2048 x 4 bytes is far beyond 16 MiB: refused before any launch
    M, K, bank, k, N = 6000, 3000, 100, 10, 2048
    need = bs.bs_spmm_workspace_bytes(bs.BS_F32, M, K, bank, k, N)
    assert need > bs.bs_spmm_static_limit()
    v = torch.zeros((M, K // bank, k), device=DEV)
    i = torch.zeros((M, K // bank, k), dtype=torch.uint8, device=DEV)
    X = torch.zeros((K, N), device=DEV)
    out = torch.full((M, N), 3.0, device=DEV)
    with pytest.raises(bs.BsError) as e:
        bs.bs_spmm_static(v, i, bank, X, out)
    assert e.value.status == 8
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())
