"""Balanced-Sparsity multiply for AMD MI355X (gfx950): thin Python binding over
the C-ABI library ``libbs.so`` (hand-written HIP kernels).

``bs_prune_pack``, ``bs_spmv``, ``bs_spmm`` and the dense baselines take torch
tensors that live on the GPU and only marshal arguments; every step runs in
the HIP kernels.  The native library is loaded on first use and a missing
library is an error, never a fallback.
"""
from __future__ import annotations

_BINDING_NAMES = (
    "bs_init", "bs_prune_pack", "bs_spmv", "bs_spmv_ex", "bs_spmv_plan", "bs_spmm", "bs_spmm_static", "bs_spmm_static_limit", "bs_spmm_workspace_bytes", "bs_spmm_plan",
    "bs_dense_gemv", "bs_dense_gemm", "bs_lstm_step", "bs_lstm_sequence", "bs_reprune", "bs_idx_bytes_wide", "bs_prune_pack_wide", "bs_spmv_wide",
    "bs_spmm_workspace_bytes_wide", "bs_spmm_wide", "bs_nnz", "bs_vals_bytes", "bs_idx_bytes",
    "bs_status_str", "BsError", "PreparedSpmv", "load_library", "library_path",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)


__all__ = list(_BINDING_NAMES)
