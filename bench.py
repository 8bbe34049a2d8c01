#!/usr/bin/env python3
"""Benchmark of the Balanced-Sparsity multiply on one MI355X.

A step is one pass of the inference hot path over one synthetic batch: one
``bs_spmv`` (or ``bs_spmm`` for workloads with N > 1) on the packed matrix,
which ``bs_prune_pack`` wrote on the GPU before the timed region (pruning is a
one-time, model-load step; it is timed separately and reported under
``extras``).  The default workload is the LSTM-1500 gate matrix, 6000 x 3000,
banks of 100 keeping 10 (90 % sparse), batch 1.

The timed region is exactly K steps between two HIP events on the launch
stream; ``value`` and ``roofline.achieved`` are both algorithmic bytes x K /
that wall time (gaps between launches included, so the kernel's own duration is
at most this).  A second pass over the same K launches attaches a pair of
events to every launch, which receive that kernel's own begin/end time stamps;
its statistics are reported under ``extras`` (that method cannot report less
than about 3.9 us, the figure it gives for an empty kernel).
"Cold" (default) rotates over enough copies of vals/idx to exceed twice the
256 MB last-level cache, so every launch streams from HBM; ``--warm`` reuses one
copy (cache resident; reported as such, never as HBM bandwidth).

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
LLC_BYTES = 256 << 20
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (see profiles/);
# None until measured for that workload.
MEASURED_TRAFFIC = {
    # profiles/spmv_lstm1500_hbm_traffic.md: 4496.8 KiB fetched x 1.993 (copy-kernel
    # calibration) + 23.4 KiB written
    ("lstm1500", "cold"): 9_252_196,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="lstm1500")
    ap.add_argument("--warm", action="store_true", help="reuse one copy of the matrix (cache resident)")
    ap.add_argument("--eager", action="store_true", help="time Python-side launches, no HIP graph")
    ap.add_argument("--no-extras", action="store_true", help="skip the secondary measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    return ap.parse_args()


class HipEvents:
    """Raw hipEvent_t pairs, so single launches can be timed by their own time stamps."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float),
                                                 ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            if self.hip.hipEventCreate(ctypes.byref(a)) or self.hip.hipEventCreate(ctypes.byref(b)):
                raise RuntimeError("hipEventCreate failed")
            self.pairs.append((a.value, b.value))

    def us(self, i):
        t = ctypes.c_float()
        a, b = self.pairs[i]
        rc = self.hip.hipEventElapsedTime(ctypes.byref(t), ctypes.c_void_p(a), ctypes.c_void_p(b))
        if rc:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return t.value * 1e3

    def close(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(ctypes.c_void_p(a))
            self.hip.hipEventDestroy(ctypes.c_void_p(b))
        self.pairs = []


def region_us(torch, fn, n):
    """Wall time per call of n back-to-back calls between two events on the launch stream."""
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    s.record()
    for i in range(n):
        fn(i)
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) * 1e3 / n


def graph_us(torch, fn, n):
    """Time per call of n calls captured into one graph and replayed: the protocol of `value`,
    free of the host's per-call cost (which would inflate kernels of a few microseconds).
    Falls back to eager launches if the calls cannot be captured."""
    try:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            fn(0)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(n):
                fn(i)
        g.replay()
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        g.replay()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) * 1e3 / n
    except Exception:
        torch.cuda.synchronize()
        return region_us(torch, fn, n)


OTHER_WORKLOADS = ("tiny", "sweep_k32", "sweep_k16", "sweep_k8", "sweep_k4", "sweep_k2",
                   "lstm1500_n8", "lstm1500_n32", "lstm1500_n128", "fc6_b1", "fc6_b16",
                   # Table 4's axes: balance range 25 / 50 / 100 at 60 % .. 80 % on the LSTM matrix
                   "lstm1500_b25_k10", "lstm1500_b25_k5", "lstm1500_b50_k20", "lstm1500_b50_k15",
                   "lstm1500_b50_k10", "lstm1500_b100_k40", "lstm1500_b100_k30", "lstm1500_b100_k20",
                   "bilstm1024",
                   # Sec. 4.2: convolution layers as products over im2col columns
                   "conv5_n196", "conv4_n784", "conv2_n12544",
                   # Sec. 4.1's matrix shape, 50 % .. 97 % sparse, batch 1 and 8
                   "bench16k_k128", "bench16k_k64", "bench16k_k32", "bench16k_k16", "bench16k_k8",
                   "bench16k_k128_n8", "bench16k_k32_n8", "bench16k_k8_n8")


def quick_measure(torch, np, bs, workloads, dev, name, o_time, launches=200):
    """One workload, cold, `launches` graph-replayed launches: time per launch.
    o_time = measured launch floor, for eq. (5)'s ideal time."""
    wl, W, X = workloads.make(name)
    Wd = torch.from_numpy(W).to(dev)
    Xd = torch.from_numpy(np.ascontiguousarray(X)).to(dev)
    vals, idx = bs.bs_prune_pack(Wd, wl.bank, wl.k)
    alg = wl.spmv_bytes()
    R = max(2, -(-2 * LLC_BYTES // alg) + 1)
    copies = [(vals, idx)] + [(vals.clone(), idx.clone()) for _ in range(R - 1)]
    spmm = wl.N > 1
    Y = torch.empty((wl.M, wl.N) if spmm else (wl.M,), dtype=torch.float32, device=dev)
    if spmm:
        code = bs.BS_F16 if wl.dtype == "f16" else bs.BS_F32
        ws = torch.empty(max(16, bs.bs_spmm_workspace_bytes(code, wl.M, wl.K, wl.bank, wl.k, wl.N)),
                         dtype=torch.uint8, device=dev)

    def launch_all():
        if spmm:
            for i in range(launches):
                v, ix = copies[i % R]
                bs.bs_spmm(v, ix, wl.bank, Xd, out=Y, workspace=ws)
        else:
            cs = [bs.PreparedSpmv(v, ix, wl.bank, Xd, Y) for v, ix in copies]
            for i in range(launches):
                cs[i % R]()

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        launch_all()                                  # warm-up outside any graph
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        launch_all()
    g.replay()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    g.replay()
    e.record()
    torch.cuda.synchronize()
    us = s.elapsed_time(e) * 1e3 / launches
    res = {"us": round(us, 2), "GBps": round(alg / us / 1e3, 1),
           "frac_of_8TBps": round(alg / us / 1e3 / HBM_PEAK_GBS, 3)}
    if spmm:
        res["TFLOPs"] = round(wl.flops() / us / 1e6, 2)
    # dense baseline, cold as well
    Rd = max(2, -(-2 * LLC_BYTES // wl.dense_bytes()) + 1)
    Wc = [Wd] + [Wd.clone() for _ in range(min(Rd, 8) - 1)]
    n_d = 10 if spmm else 50
    fn = (lambda i: bs.bs_dense_gemm(Wc[i % len(Wc)], Xd, out=Y)) if spmm else \
         (lambda i: bs.bs_dense_gemv(Wc[i % len(Wc)], Xd, out=Y))
    for i in range(2):
        fn(i)
    d_us = graph_us(torch, fn, n_d)
    res["dense_us"] = round(d_us, 1)
    res["speedup_vs_dense"] = round(d_us / us, 2)
    # context: the vendor library's dense product on the same matrix (torch.matmul ->
    # rocBLAS / hipBLASLt; fp16 weights multiply an fp16 copy of X there)
    try:
        Xl = Xd if wl.dtype == "f32" else Xd.half()
        Yl = torch.empty(Y.shape, dtype=Xl.dtype, device=dev)
        lib = lambda i: torch.matmul(Wc[i % len(Wc)], Xl, out=Yl)
        for i in range(3):
            lib(i)
        res["dense_library_us"] = round(graph_us(torch, lib, n_d), 1)
        res["speedup_vs_faster_dense"] = round(min(d_us, res["dense_library_us"]) / us, 2)
    except Exception as exc:
        res["dense_library_error"] = str(exc)[:80]
    # eq. (5): the dense time scaled by the kept fraction, launch overhead not scaled
    res["ideal_us_eq5"] = round(max(d_us - o_time, 0.0) * (1 - wl.sparsity) + o_time, 2)
    # pruning + packing this matrix (W rotates as for the dense baseline)
    p_out = (torch.empty_like(vals), torch.empty_like(idx))
    pfn = lambda i: bs.bs_prune_pack(Wc[i % len(Wc)], wl.bank, wl.k, out=p_out)
    pfn(0)
    p_us = graph_us(torch, pfn, 6)
    res["prune_pack_us"] = round(p_us, 1)
    res["prune_pack_GBps"] = round((W.nbytes + wl.nnz * (wl.val_bytes + 1)) / p_us / 1e3, 1)
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 "
              "(the path would shard by rows, but no multi-GPU code exists)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1811_00206_amd import binding as bs
    from paper_1811_00206_amd import workloads

    if not os.path.exists(bs.library_path()):
        from paper_1811_00206_amd.build import build_library
        build_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    wl, W, X = workloads.make(args.workload)
    K, W_steps = args.steps, args.warmup
    Wd = torch.from_numpy(W).to(dev)
    Xd = torch.from_numpy(np.ascontiguousarray(X)).to(dev)
    vals, idx = bs.bs_prune_pack(Wd, wl.bank, wl.k)        # the product path packs on the GPU
    torch.cuda.synchronize()

    alg_bytes = wl.spmv_bytes()
    if args.warm:
        R = 1
    else:
        R = max(2, -(-2 * LLC_BYTES // alg_bytes) + 1)
    copies = [(vals, idx)] + [(vals.clone(), idx.clone()) for _ in range(R - 1)]
    spmm = wl.N > 1
    if spmm:
        Y = torch.empty((wl.M, wl.N), dtype=torch.float32, device=dev)
        ws_bytes = bs.bs_spmm_workspace_bytes(bs.BS_F16 if wl.dtype == "f16" else bs.BS_F32,
                                              wl.M, wl.K, wl.bank, wl.k, wl.N)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    else:
        Y = torch.empty(wl.M, dtype=torch.float32, device=dev)

    events = None if spmm else HipEvents(K)
    # arguments marshalled once per matrix copy: a step is then one C-ABI call
    calls = None if spmm else [bs.PreparedSpmv(v, ix, wl.bank, Xd, Y) for v, ix in copies]

    def step(i, timed=False):
        if spmm:
            v, ix = copies[i % R]
            bs.bs_spmm(v, ix, wl.bank, Xd, out=Y, workspace=ws)
        elif timed:
            a, b = events.pairs[i]
            calls[i % R](a, b)
        else:
            calls[i % R]()

    for i in range(W_steps):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region A: exactly K steps between two events on the launch stream.
    # The K launches are captured once into a HIP graph (the deployment form of a
    # launch-bound loop) and replayed inside the region; --eager launches them
    # from Python instead.
    mode = "eager"
    graph = None
    if not args.eager:
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                if spmm:
                    for i in range(K):
                        step(i)
                else:
                    gcalls = [bs.PreparedSpmv(v, ix, wl.bank, Xd, Y) for v, ix in copies]
                    for i in range(K):
                        gcalls[i % R]()
            graph.replay()                       # one untimed replay
            torch.cuda.synchronize()
            mode = "hip graph of K launches"
        except Exception as exc:                 # capture unsupported: say so, time eagerly
            print(f"bench.py: graph capture failed ({exc}); timing eager launches", file=sys.stderr)
            graph = None
    t_wall0 = time.perf_counter()
    if graph is not None:
        s_ev, e_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        s_ev.record()
        graph.replay()
        e_ev.record()
        torch.cuda.synchronize()
        us_per_step = s_ev.elapsed_time(e_ev) * 1e3 / K
    else:
        us_per_step = region_us(torch, step, K)
    t_wall = time.perf_counter() - t_wall0

    # The kernel's average launch duration is taken from that same region: wall time
    # between the two events / K.  Launch gaps are inside it, so it is an upper bound
    # of the kernel's own duration (rocprofv3's per-dispatch average is the check).
    kern_us = us_per_step
    kern_note = ("HIP events around the K launches of the timed region / K"
                 + (" (slab kernel + reduce kernel per step)" if spmm else ""))

    # ---- region B (spmv only, reported under extras): the same K launches again,
    # each with its own pair of events that receive that launch's begin/end time
    # stamps.  Attaching events slows the host side, so launches are spaced out.
    if not spmm:
        region_us(torch, lambda i: step(i, timed=True), K)
        durs = np.array([events.us(i) for i in range(K)])
    value = alg_bytes / us_per_step / 1e3                  # GB/s
    achieved = alg_bytes / kern_us / 1e3

    out = {
        "metric": "bs_spmv achieved HBM GB/s" if not spmm else "bs_spmm achieved HBM GB/s",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W_steps,
        "ms_per_step": round(us_per_step / 1e3, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if wl.dtype == "f32" else "f16 storage, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: W {wl.M}x{wl.K} {wl.dtype}, bank {wl.bank}, keep {wl.k} "
                               f"({100 * wl.sparsity:.3g}% sparse), batch {wl.N}",
                   "residency": "warm (one copy, cache resident)" if args.warm else
                                f"cold (rotating over {R} copies, {R * alg_bytes / 1e6:.0f} MB)",
                   "launch": mode,
                   "algorithmic_bytes_per_step": alg_bytes,
                   "flop_per_step": wl.flops()},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_TRAFFIC.get((wl.name, "warm" if args.warm else "cold")),
                     "kernel_us": round(kern_us, 3), "how": kern_note},
    }

    extras = {"gflops": round(wl.flops() / us_per_step / 1e3, 1),
              "host_wall_s_timed_region": round(t_wall, 3)}
    if not spmm:
        extras["per_launch_stamp_us_min_med_mean_p90"] = [
            round(float(v), 2) for v in (durs.min(), np.median(durs), durs.mean(),
                                         np.percentile(durs, 90))]

    if not args.no_extras:
        ev = HipEvents(64)

        def kernel_us_of(v, ix, x, y, bank, n=64):
            for i in range(n):
                bs.bs_spmv(v, ix, bank, x, out=y, start_event=ev.pairs[i][0],
                           stop_event=ev.pairs[i][1])
            torch.cuda.synchronize()
            return float(np.median([ev.us(i) for i in range(n)]))

        # floor of the time-stamp method: a one-row matrix (nothing to stream)
        v1 = torch.zeros((1, wl.nb, wl.k), dtype=vals.dtype, device=dev)
        i1 = torch.zeros((1, wl.nb, wl.k), dtype=torch.uint8, device=dev)
        y1 = torch.empty(1, dtype=torch.float32, device=dev)
        if not spmm:
            extras["launch_floor_us"] = round(kernel_us_of(v1, i1, Xd, y1, wl.bank), 2)
            # the same matrix from cache (one copy): what an LSTM time step loop sees
            w_us = kernel_us_of(vals, idx, Xd, Y, wl.bank)
            extras["warm_kernel_us"] = round(w_us, 2)
            extras["warm_GBps_cache_resident"] = round(alg_bytes / w_us / 1e3, 1)
            # ... and in the protocol of `value` (a graph of launches back to back), which
            # does not carry the time-stamp method's floor
            gw = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gw):
                for _ in range(64):
                    bs.bs_spmv(vals, idx, wl.bank, Xd, out=Y)
            gw.replay()
            torch.cuda.synchronize()
            s1, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s1.record()
            for _ in range(10):
                gw.replay()
            e1.record()
            torch.cuda.synchronize()
            wg_us = s1.elapsed_time(e1) * 1e3 / 640
            extras["warm_us_per_launch_graph"] = round(wg_us, 3)
            extras["warm_GBps_per_launch_graph"] = round(alg_bytes / wg_us / 1e3, 1)
            del gw

        def avg_us(fn, n):
            for _ in range(3):
                fn(0)
            return graph_us(torch, fn, n)

        # dense baseline on the unpruned-shape matrix, same residency protocol
        dense_bytes = wl.dense_bytes()
        Rd = 1 if args.warm else max(2, -(-2 * LLC_BYTES // dense_bytes) + 1)
        Wc = [Wd] + [Wd.clone() for _ in range(Rd - 1)]
        if spmm:
            d_us = avg_us(lambda i: bs.bs_dense_gemm(Wc[i % Rd], Xd, out=Y), 20)
        else:
            d_us = avg_us(lambda i: bs.bs_dense_gemv(Wc[i % Rd], Xd, out=Y), 200)
        del Wc
        extras["dense_us"] = round(d_us, 2)
        extras["dense_GBps"] = round(dense_bytes / d_us / 1e3, 1)
        extras["speedup_vs_dense"] = round(d_us / us_per_step, 2)   # both: region time per launch
        # eq. (5) of the paper with the measured dense time and the measured launch floor
        o_time = extras.get("launch_floor_us", 0.0)
        extras["ideal_us_eq5"] = round((d_us - o_time) * (1 - wl.sparsity) + o_time, 2)
        # one-time pruning + packing of the dense matrix
        p_out = (torch.empty_like(vals), torch.empty_like(idx))
        p_us = avg_us(lambda i: bs.bs_prune_pack(Wd, wl.bank, wl.k, out=p_out), 10)
        p_bytes = W.nbytes + wl.nnz * (wl.val_bytes + 1)
        extras["prune_pack_us"] = round(p_us, 1)
        extras["prune_pack_GBps"] = round(p_bytes / p_us / 1e3, 1)
        # one more pruning round on the packed matrix: half the weights of every bank
        if wl.k >= 2:
            k2 = wl.k // 2
            r_out = bs.bs_reprune(vals, idx, wl.bank, k2)
            torch.cuda.synchronize()
            gr = torch.cuda.CUDAGraph()       # a 9 us kernel: replayed from a graph, as the products are
            with torch.cuda.graph(gr):
                for _ in range(20):
                    bs.bs_reprune(vals, idx, wl.bank, k2, out=r_out)
            gr.replay()
            torch.cuda.synchronize()
            r_us = region_us(torch, lambda i: gr.replay(), 5) / 20
            extras["reprune_to_half_us"] = round(r_us, 1)
            extras["reprune_GBps"] = round((wl.nnz + wl.M * (wl.K // wl.bank) * k2) *
                                           (wl.val_bytes + 1) / r_us / 1e3, 1)
        ev.close()

        # the machine's floor, measured with the library's helper kernels in the same
        # protocol (a graph of launches): an empty launch, a kernel that only reads this
        # workload's bytes (cold, rotating buffers), and a large streaming read
        try:
            def floor_graph_us(launch, n):
                side2 = torch.cuda.Stream()
                with torch.cuda.stream(side2):
                    for i in range(min(n, 8)):
                        launch(i)
                torch.cuda.synchronize()
                gp = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gp):
                    for i in range(n):
                        launch(i)
                gp.replay()
                torch.cuda.synchronize()
                return region_us(torch, lambda i: gp.replay(), 3) / n

            floor = {}
            floor["empty_launch_us"] = round(floor_graph_us(lambda i: bs.bs_probe_empty(750, 256), 1000), 3)
            same = (alg_bytes + 15) // 16 * 16
            n_same = max(2, -(-2 * LLC_BYTES // same) + 1)
            bufs = [torch.empty(same, dtype=torch.uint8, device=dev) for _ in range(n_same)]
            for b_ in bufs:
                b_.fill_(1)
            t_same = floor_graph_us(lambda i: bs.bs_probe_stream_read(bufs[i % n_same]), 2 * n_same)
            floor["stream_read_same_bytes_us"] = round(t_same, 3)
            floor["stream_read_same_bytes_GBps"] = round(same / t_same / 1e3, 1)
            del bufs
            big = 288 << 20
            bufs = [torch.empty(big, dtype=torch.uint8, device=dev) for _ in range(3)]
            for b_ in bufs:
                b_.fill_(1)
            t_big = floor_graph_us(lambda i: bs.bs_probe_stream_read(bufs[i % 3]), 12)
            floor["stream_read_288MB_us"] = round(t_big, 2)
            floor["stream_read_288MB_GBps"] = round(big / t_big / 1e3, 1)
            floor["value_over_same_bytes_stream"] = round(t_same / us_per_step, 3)
            del bufs
            # what an LDS gather costs (the SpMM kernels' inner loop): 256 workgroups of 768
            # lanes that only issue 16-byte LDS reads; ns per wavefront read and compute unit
            reads, thr = 16000, 768
            t0 = floor_graph_us(lambda i: bs.bs_probe_lds_gather(thr, 0, 16, 8), 4)   # fill + launch only
            lds = {}
            for key, pattern, lanes in (("adjacent_1KB", 0, 16), ("rows_of_256B", 1, 16),
                                        ("rows_of_128B", 1, 8), ("rows_of_64B", 1, 4), ("rows_of_32B", 1, 2)):
                t = floor_graph_us(lambda i: bs.bs_probe_lds_gather(thr, pattern, lanes, reads), 4)
                lds[key] = round((t - t0) * 1e3 / ((reads - 8) * thr / 64), 3)
            floor["lds_gather_ns_per_wavefront_read_per_cu"] = lds
            extras["machine_floor"] = floor
        except Exception as exc:                 # never lose the headline line
            extras["machine_floor_error"] = str(exc)[:200]

        # fused LSTM time steps (Sec. 4.3's language model: H = I = 1500 is this very gate
        # matrix): T dependent steps replayed from one graph, weights cache resident as in
        # a real recurrence; per step = the sparse product + bias, gates and cell update
        if not spmm and wl.M % 4 == 0 and wl.K > wl.M // 4:
            try:
                Hn, T = wl.M // 4, 64
                In = wl.K - Hn
                Xs_h, h0_h, c0_h, b_h = workloads.draw_lstm_inputs(Hn, In, T, wl.seed)
                Xs, h0, c0, bias = (torch.from_numpy(t).to(dev) for t in (Xs_h, h0_h, c0_h, b_h))
                H_all = torch.empty((T, Hn), dtype=torch.float32, device=dev)
                side = torch.cuda.Stream()
                with torch.cuda.stream(side):
                    bs.bs_lstm_sequence(vals, idx, wl.bank, Xs, h0, bias, c0, H_all=H_all)
                torch.cuda.synchronize()
                gl = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gl):
                    bs.bs_lstm_sequence(vals, idx, wl.bank, Xs, h0, bias, c0, H_all=H_all)
                gl.replay()
                torch.cuda.synchronize()
                s2, e2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                s2.record()
                for _ in range(10):
                    gl.replay()
                e2.record()
                torch.cuda.synchronize()
                l_us = s2.elapsed_time(e2) * 1e3 / (10 * T)
                extras["lstm_step_us_cache_resident"] = round(l_us, 3)
                extras["lstm_steps_per_graph"] = T
                extras["lstm_step_vs_dense_gemv_us"] = round(d_us, 2)
            except Exception as exc:             # never lose the headline line
                extras["lstm_error"] = str(exc)[:200]

        # the paper's own timings of the same layers (Tables 1-3), as context only: another
        # GPU (an NVIDIA part the paper does not name), trained weights, precision not stated
        extras["paper_context_us"] = {
            "hardware": "unnamed NVIDIA GPU (paper, Sec. 4); not a target",
            "table1_lstm_2x1500": {"dense": 294.1, "balanced_80pct": 120.2},
            "table2_vgg_fc6_4096x25088": {"dense": 979.9, "balanced_93pct": 231.1},
            "table2_vgg_fc7_4096x4096": {"dense": 265.5, "balanced_93pct": 70.3},
            "table3_bilstm_1024": {"dense": 117.9, "balanced_87.5pct": 83.9},
            "eq5_launch_overhead": 10.0,
        }

        # the other configurations of the metric, same protocol (cold, graph of launches),
        # fewer launches: {us per launch, GB/s of algorithmic bytes, dense baseline us}
        if not args.warm and args.workload == "lstm1500":
            del copies, calls
            others = {}
            for name in OTHER_WORKLOADS:
                try:
                    others[name] = quick_measure(torch, np, bs, workloads, dev, name, o_time)
                except Exception as exc:             # never lose the headline line
                    others[name] = {"error": str(exc)[:200]}
                torch.cuda.empty_cache()
            extras["other_workloads_cold"] = others
    out["extras"] = extras

    if not args.no_cpu:
        from oracle import bs_ref
        v_h, i_h = vals.cpu().numpy(), idx.cpu().numpy()
        threads = min(16, bs_ref.host_threads())
        fn = (lambda: bs_ref.spmm(v_h, i_h, wl.bank, X, threads=threads)) if spmm else \
             (lambda: bs_ref.spmv(v_h, i_h, wl.bank, X, threads=threads))
        fn()
        t0 = time.perf_counter()
        n_calls = 0
        while True:
            fn()
            n_calls += 1
            el = time.perf_counter() - t0
            if el > 10.0:
                break
        out["cpu_baseline"] = {"value": round(alg_bytes * n_calls / el / 1e9, 3), "unit": "GB/s",
                               "cores": threads, "kind": "oracle",
                               "sample": f"{n_calls} full products of the same workload "
                                         f"in {el:.1f} s (fp64 accumulate, rows split over threads)",
                               "us_per_call": round(el / n_calls * 1e6, 1)}
    if events:
        events.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
