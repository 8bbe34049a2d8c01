"""Seeded synthetic inputs for the Balanced-Sparsity multiply.

This module only draws random numbers; it holds none of the method's
arithmetic (no pruning, no products) and loads no native code, so the tests,
the bench and the CPU checker can all take their inputs from here.

The shapes stand in for the paper's trained models, which are not needed to
time or check the multiply (arXiv 1811.00206): the 6000 x 3000 matrix is the
four stacked gates of an LSTM with hidden size 1500 acting on [x; h]
(Sec. 4.2, "LSTM on PTB"; balance range 100 as in Table 4); 4096 x 25088 is
VGG-16's fc6 (Table 2); 16384 x 8192 with 32 banks per row is the matmul
benchmark of Sec. 4.1 (the paper prints 8196, which 32 does not divide).
Weights are i.i.d. Gaussian, the prior of Sec. 3.3; activations are uniform on
(-1, 1).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_BASE = 181100206


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    K: int
    bank: int
    k: int
    sigma: float
    dtype: str          # "f32" or "f16": storage type of W / vals
    N: int              # columns of X; 1 = matrix-vector
    seed: int

    @property
    def nb(self) -> int:
        return self.K // self.bank

    @property
    def nnz(self) -> int:
        return self.M * self.nb * self.k

    @property
    def sparsity(self) -> float:
        return 1.0 - self.k / self.bank

    @property
    def val_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def idx_bytes(self) -> int:
        """Bytes per stored offset: one, or two for balance ranges over 256."""
        return 1 if self.bank <= 256 else 2

    def spmv_bytes(self) -> int:
        """Algorithmic HBM bytes of one sparse product: every stored value and
        offset once, X once, Y once."""
        return self.nnz * (self.val_bytes + self.idx_bytes) + 4 * self.K * self.N + 4 * self.M * self.N

    def dense_bytes(self) -> int:
        return self.M * self.K * self.val_bytes + 4 * self.K * self.N + 4 * self.M * self.N

    def flops(self) -> int:
        return 2 * self.nnz * self.N


def _mk(i, name, M, K, bank, k, sigma, dtype="f32", N=1):
    return Workload(name, M, K, bank, k, sigma, dtype, N, SEED_BASE + i)


WORKLOADS = {w.name: w for w in [
    _mk(1, "tiny", 256, 256, 64, 16, 1.0),
    _mk(2, "lstm1500", 6000, 3000, 100, 10, 0.05),
    _mk(3, "sweep_k32", 4096, 4096, 64, 32, 1.0),
    _mk(3, "sweep_k16", 4096, 4096, 64, 16, 1.0),
    _mk(3, "sweep_k8", 4096, 4096, 64, 8, 1.0),
    _mk(3, "sweep_k4", 4096, 4096, 64, 4, 1.0),
    _mk(3, "sweep_k2", 4096, 4096, 64, 2, 1.0),
    _mk(4, "lstm1500_n8", 6000, 3000, 100, 10, 0.05, N=8),
    _mk(4, "lstm1500_n32", 6000, 3000, 100, 10, 0.05, N=32),
    _mk(4, "lstm1500_n128", 6000, 3000, 100, 10, 0.05, N=128),
    _mk(5, "fc6_b1", 4096, 25088, 64, 6, 0.01, dtype="f16", N=1),
    _mk(5, "fc6_b16", 4096, 25088, 64, 6, 0.01, dtype="f16", N=16),
    # Sec. 4.1 benchmark shape, 32 banks per row -> bank 256
    _mk(6, "bench16k_k128", 16384, 8192, 256, 128, 1.0),
    _mk(6, "bench16k_k64", 16384, 8192, 256, 64, 1.0),
    _mk(6, "bench16k_k32", 16384, 8192, 256, 32, 1.0),
    _mk(6, "bench16k_k16", 16384, 8192, 256, 16, 1.0),
    _mk(6, "bench16k_k8", 16384, 8192, 256, 8, 1.0),
    # Sec. 4.2: convolution as a matrix product over im2col columns, VGG-16 layer shapes
    # (Table 2): out-channels x (in-channels * 3 * 3), one column per output pixel
    _mk(9, "conv5_n196", 512, 4608, 64, 16, 0.02, N=196),
    _mk(9, "conv4_n784", 512, 4608, 64, 16, 0.02, N=784),
    _mk(9, "conv2_n12544", 128, 576, 64, 16, 0.05, N=12544),
    # the large-N end (Table 2's first rows, where the paper's kernel loses to dense):
    # conv1_2, 64 x (64 * 3 * 3), one column per pixel of a 224 x 224 output
    _mk(9, "conv1_n50176", 64, 576, 64, 16, 0.05, N=50176),
    # Table 4's axes on the LSTM gate matrix: balance range 25 / 50 / 100 at 60 % .. 80 %
    _mk(8, "lstm1500_b25_k10", 6000, 3000, 25, 10, 0.05),
    _mk(8, "lstm1500_b25_k5", 6000, 3000, 25, 5, 0.05),
    _mk(8, "lstm1500_b50_k20", 6000, 3000, 50, 20, 0.05),
    _mk(8, "lstm1500_b50_k15", 6000, 3000, 50, 15, 0.05),
    _mk(8, "lstm1500_b50_k10", 6000, 3000, 50, 10, 0.05),
    _mk(8, "lstm1500_b100_k40", 6000, 3000, 100, 40, 0.05),
    _mk(8, "lstm1500_b100_k30", 6000, 3000, 100, 30, 0.05),
    _mk(8, "lstm1500_b100_k20", 6000, 3000, 100, 20, 0.05),
    # Sec. 4.3's second recurrent model: hidden size 1024 (input size taken as 1024), 87.5 %
    _mk(7, "bilstm1024", 4096, 2048, 64, 8, 0.05),
    # balance ranges over 256 (16-bit offsets): Sec. 4.1's matrix with 16 and 8 banks per row
    _mk(10, "bench16k_b512_k64", 16384, 8192, 512, 64, 1.0),
    _mk(10, "bench16k_b1024_k128", 16384, 8192, 1024, 128, 1.0),
    _mk(10, "bench16k_b512_k64_n8", 16384, 8192, 512, 64, 1.0, N=8),
    _mk(6, "bench16k_k128_n8", 16384, 8192, 256, 128, 1.0, N=8),
    _mk(6, "bench16k_k32_n8", 16384, 8192, 256, 32, 1.0, N=8),
    _mk(6, "bench16k_k8_n8", 16384, 8192, 256, 8, 1.0, N=8),
]}


def draw_weights(M: int, K: int, sigma: float, dtype: str, seed: int) -> np.ndarray:
    """M x K weights ~ N(0, sigma) in fp32; for "f16" rounded to nearest-even
    binary16 on the host, and that rounded array IS the input."""
    rng = np.random.Generator(np.random.PCG64(seed))
    W = rng.standard_normal((M, K), dtype=np.float32)
    W *= np.float32(sigma)
    if dtype == "f16":
        return W.astype(np.float16)
    if dtype != "f32":
        raise ValueError(dtype)
    return W


def draw_activations(K: int, N: int, seed: int) -> np.ndarray:
    """x ~ U(-1, 1) fp32: shape [K] for N == 1, else [K, N] row-major."""
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    X = rng.random((K, N), dtype=np.float32)
    X = X * np.float32(2.0) - np.float32(1.0)
    return X[:, 0].copy() if N == 1 else X


def draw_lstm_inputs(H: int, I: int, T: int, seed: int):
    """Inputs of T LSTM steps besides the gate matrix: X [T, I] ~ U(-1, 1), h0 [H] and
    c0 [H] ~ U(-1, 1), bias [4H] ~ U(-0.5, 0.5), all fp32."""
    rng = np.random.Generator(np.random.PCG64(seed + 104729))
    u = lambda shape, a: (rng.random(shape, dtype=np.float32) * np.float32(2 * a) - np.float32(a))
    return u((T, I), 1.0), u((H,), 1.0), u((H,), 1.0), u((4 * H,), 0.5)


def make(name_or_workload, rows: int | None = None):
    """(workload, W, X) for a named workload; `rows` keeps only the first rows
    of W (a bounded sample with the same row structure)."""
    wl = WORKLOADS[name_or_workload] if isinstance(name_or_workload, str) else name_or_workload
    W = draw_weights(wl.M, wl.K, wl.sigma, wl.dtype, wl.seed)
    if rows is not None:
        W = np.ascontiguousarray(W[:rows])
    X = draw_activations(wl.K, wl.N, wl.seed)
    return wl, W, X


def tie_heavy_weights(M: int, K: int, levels: int, dtype: str, seed: int) -> np.ndarray:
    """Weights drawn from a few magnitudes with random signs, so nearly every
    bank has ties at the cut: exercises the lower-offset rule."""
    rng = np.random.Generator(np.random.PCG64(seed))
    mag = rng.integers(0, levels, size=(M, K)).astype(np.float32) * np.float32(0.25)
    sign = rng.integers(0, 2, size=(M, K)).astype(np.float32) * 2 - 1
    W = mag * sign  # includes +0.0 and -0.0
    return W.astype(np.float16) if dtype == "f16" else W.astype(np.float32)
