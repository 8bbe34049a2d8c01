"""GPU parity on random shapes: every entry point (byte and 16-bit offsets, fp32 and binary16
storage, tie-heavy and Gaussian weights, 1..130 columns) against the CPU oracle.  A fixed seed
and a fixed number of cases; each case is printed before it runs."""
import random

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


def close(y, ref, tol, scale):
    return float(np.abs(y.astype(np.float64) - ref).max()) <= tol * scale


@pytest.mark.timeout(600)
@pytest.mark.parametrize("seed", [11, 12])
def test_random_shapes_against_the_oracle(seed):
    rng = random.Random(seed)
    threads = min(16, bs_ref.host_threads())
    for n in range(120):
        wide = rng.random() < 0.35
        dtype = rng.choice(["f32", "f16"])
        if wide:
            unit = 8 if dtype == "f16" else 4
            bank = rng.choice([260, 264, 320, 384, 512, 520, 640, 768, 784, 1000, 1024, 1536, 2048, 8, 16, 64, 256])
            bank = (bank + unit - 1) // unit * unit
            nb = rng.choice([1, 2, 3, 5, 8, 16, 31])
        else:
            bank = rng.choice([1, 2, 3, 4, 5, 7, 8, 16, 25, 32, 50, 64, 100, 128, 200, 255, 256])
            nb = rng.choice([1, 2, 3, 7, 30, 32, 64, 100, 157])
        K = bank * nb
        if K > 40000:
            continue
        k = min(bank, rng.choice([1, 2, 3, max(1, bank // 10), max(1, bank // 4), max(1, bank // 2),
                                  max(1, bank - 1), bank, rng.randint(1, bank)]))
        M = rng.choice([1, 2, 3, 5, 17, 63, 64, 65, 100, 255, 256, 257, 500, 1000, 2048])
        M = max(1, min(M, 4_000_000 // K))
        N = rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 17, 31, 32, 33, 64, 100, 130])
        ties = rng.random() < 0.3
        what = f"seed {seed} case {n}: wide {wide} {dtype} M {M} K {K} bank {bank} k {k} N {N} ties {ties}"
        print(what, flush=True)
        s = seed * 1000 + n
        W = (workloads.tie_heavy_weights(M, K, rng.choice([1, 2, 3, 5]), dtype, s) if ties
             else workloads.draw_weights(M, K, 0.05, dtype, s))
        v_ref, i_ref = bs_ref.prune_pack(W, bank, k, wide=wide)
        v, i = (bs.bs_prune_pack_wide if wide else bs.bs_prune_pack)(dev(W), bank, k)
        torch.cuda.synchronize()
        i_bits = i.view(torch.int16) if wide else i
        assert v.cpu().numpy().tobytes() == v_ref.tobytes(), what
        assert i_bits.cpu().numpy().tobytes() == i_ref.tobytes(), what
        tol = 1e-5 if dtype == "f32" else 1e-2
        Wp = np.abs(bs_ref.unpack(v_ref, i_ref, bank).astype(np.float64))
        x = workloads.draw_activations(K, 1, s)
        y = (bs.bs_spmv_wide if wide else bs.bs_spmv)(v, i, bank, dev(x))
        torch.cuda.synchronize()
        assert close(y.cpu().numpy(), bs_ref.spmv(v_ref, i_ref, bank, x),
                     tol, (Wp @ np.abs(x.astype(np.float64))).max() + 1e-300), "spmv " + what
        if N > 1 and M * K * N < 200_000_000:
            X = workloads.draw_activations(K, N, s)
            Y = (bs.bs_spmm_wide if wide else bs.bs_spmm)(v, i, bank, dev(X))
            torch.cuda.synchronize()
            assert close(Y.cpu().numpy(), bs_ref.spmm(v_ref, i_ref, bank, X, threads=threads),
                         tol, (Wp @ np.abs(X.astype(np.float64))).max() + 1e-300), "spmm " + what
            if not wide:
                Ys = torch.empty_like(Y)
                bs.bs_spmm_static(v, i, bank, dev(X), Ys)
                torch.cuda.synchronize()
                assert torch.equal(Ys, Y), "spmm_static " + what
        if not wide and k > 1:
            k2 = rng.randint(1, k)
            v2, i2 = bs.bs_reprune(v, i, bank, k2)
            torch.cuda.synchronize()
            v2_ref, i2_ref = bs_ref.reprune(v_ref, i_ref, k2)
            assert v2.cpu().numpy().tobytes() == v2_ref.tobytes(), f"reprune {k2} " + what
            assert i2.cpu().numpy().tobytes() == i2_ref.tobytes(), f"reprune {k2} " + what
        Hn = M // 4
        if not wide and M % 16 == 0 and K > Hn and (K - Hn) % 4 == 0:
            Xs, h0, c0, bias = workloads.draw_lstm_inputs(Hn, K - Hn, 2, s)
            c = dev(c0)
            H_all = bs.bs_lstm_sequence(v, i, bank, dev(Xs), dev(h0), dev(bias), c)
            torch.cuda.synchronize()
            H_ref, _ = bs_ref.lstm_sequence(v_ref, i_ref, bank, Xs, h0, bias, c0)
            assert close(H_all.cpu().numpy(), H_ref, 4 * tol, 1.0), "lstm " + what
