#!/usr/bin/env python3
"""Benchmark of the Balanced-Sparsity multiply on one MI355X.

A step is one pass of the inference hot path over one synthetic batch: one
``bs_spmv`` (or ``bs_spmm`` for workloads with N > 1) on the packed matrix,
which ``bs_prune_pack`` wrote on the GPU before the timed region (pruning is a
one-time, model-load step; it is timed separately and reported under
``extras``).  The default workload is the LSTM-1500 gate matrix, 6000 x 3000,
banks of 100 keeping 10 (90 % sparse), batch 1.

The timed region is exactly K steps on the launch stream, captured into one HIP
graph together with a short pre-roll and two one-lane kernels that store the
GPU's wall clock right before the first and right after the last of the K
launches (events cannot be recorded inside a captured graph on this runtime, and
events around the replay also time the launching of the graph itself: 8 us, which
is 10 % of a 20-step region and nothing of a 2000-step one).  ``value`` and
``roofline.achieved`` are both algorithmic bytes x K / that time (gaps between
launches included, so the kernel's own duration is at most this); the time of
the whole replay between two HIP events is reported beside it.
"Cold" (default): the launches rotate over enough copies of vals/idx to exceed
twice the 256 MB last-level cache, and a 768 MB streaming read of unrelated
memory is enqueued right before every timed replay, so no timed launch finds its
matrix in a cache whatever K is; ``config.residency`` states the bytes the timed
launches touch.  ``--warm`` reuses one copy (cache resident; reported as such,
never as HBM bandwidth).  The machine's floor for the same bytes (a kernel that
only reads them, same protocol, same run) is reported inside ``roofline``.

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
EVICT_BYTES = 768 << 20
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (the two commands
# and the copy-kernel calibration are in profiles/spmv_lstm1500_hbm_traffic.md).  A figure
# belongs to one kernel instantiation; it is reported only while bs_spmv_plan still names
# that instantiation for the workload.
MEASURED_TRAFFIC = {
    # FETCH_SIZE 4494.0 KiB x 1.9932 (the copy kernels' calibration) + WRITE_SIZE 23.4 KiB
    ("lstm1500", "cold"): {"kernel": "spmv_kernel<float,4,32,3> 250 x 768", "bytes": 9_196_322},
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
    ap.add_argument("--copies", type=int, default=0,
                    help="rotate over this many copies of the packed matrix (default: enough to exceed "
                         "twice the last-level cache)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: time bs_spmv_ex on --workload over launch shapes "
                         "(lanes per row x rows per workgroup), cold, same protocol, plus empty kernels and "
                         "read-only kernels of several shapes; prints one JSON object")
    ap.add_argument("--only", default="", help="comma-separated other workloads to measure under extras "
                                               "(default: all of them)")
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


EAGER_FALLBACKS = []     # what had to be timed as eager launches (reported under extras)


class Evictor:
    """A streaming read of EVICT_BYTES of unrelated memory (three times the last-level cache).
    Enqueued right before a timed replay, on the same stream, it leaves neither L2 nor the
    last-level cache holding anything the replay is about to read; reads leave no dirty lines
    behind, so the timed region does not pay for write-backs either."""

    def __init__(self, torch, probe, dev):
        self.buf = torch.empty(EVICT_BYTES, dtype=torch.uint8, device=dev)
        self.buf.fill_(1)
        self.probe = probe

    def __call__(self):
        self.probe.probe_stream_read(self.buf)


class GraphTimer:
    """Times n calls of a function inside one captured graph with the GPU's own wall clock:
    graph = [pre-roll calls] [stamp] [the n calls] [stamp].  The pre-roll (calls n, n+1, ... of
    the same function, i.e. other copies of the data when the caller rotates) brings the
    machine to its steady state; the stamps are one-lane kernels that store the constant-rate
    wall clock (100 MHz here), so launching the graph is not inside the interval.  The interval
    of two stamps with nothing between them is measured once and subtracted."""

    PREROLL = 32

    def __init__(self, torch, probe, dev):
        self.torch, self.probe = torch, probe
        self.slots = torch.zeros(8, dtype=torch.int64, device=dev)
        self.khz = probe.wall_clock_khz()
        self.gap_us = 0.0
        if self.khz > 0:
            # two adjacent stamps behind a pre-roll of empty kernels (the steady state the
            # timed launches see; the first launches of a replay are slower)
            g = self._capture(lambda i: probe.probe_empty(1, 64), 0, self.PREROLL, "stamp gap")
            if g is not None:
                self.gap_us = min(self._replay(g, None)[0] for _ in range(5))

    def _capture(self, fn, n, preroll, what):
        torch = self.torch
        try:
            if n or preroll:
                side = torch.cuda.Stream()
                with torch.cuda.stream(side):
                    fn(0)
                torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for i in range(preroll):
                    fn(n + i)
                self.probe.probe_timestamp(self.slots, 0)
                for i in range(n):
                    fn(i)
                self.probe.probe_timestamp(self.slots, 1)
            g.replay()
            torch.cuda.synchronize()
            return g
        except Exception as exc:
            torch.cuda.synchronize()
            EAGER_FALLBACKS.append(f"{what}: {str(exc)[:120]}")
            print(f"bench.py: graph capture failed for {what!r} ({exc}); timing eager launches",
                  file=sys.stderr)
            return None

    def _replay(self, g, evict):
        """(us between the two stamps, us between two events around the whole replay)"""
        torch = self.torch
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        if evict is not None:
            evict()
        s.record()
        g.replay()
        e.record()
        torch.cuda.synchronize()
        t0, t1 = self.slots[:2].tolist()
        return (t1 - t0) / self.khz * 1e3, s.elapsed_time(e) * 1e3

    def capture(self, fn, n, what, preroll=None):
        """A graph of n timed calls (after a pre-roll), replayed once untimed; None if the calls
        cannot be captured or the wall clock's rate is unknown."""
        if self.khz <= 0:
            return None
        pre = self.PREROLL if preroll is None else preroll
        g = self._capture(fn, n, pre, what)
        return None if g is None else (g, n, pre)

    def replay_us(self, cap, evict=None):
        """One replay: (us per timed call by the stamps, us per call of the whole replay by events)."""
        g, n, pre = cap
        stamps, events = self._replay(g, evict)
        return max(stamps - self.gap_us, 0.0) / n, events / (n + pre)

    def us(self, fn, n, what, evict=None, preroll=8, best_of=1):
        """Time per call of n calls; falls back to eager launches between events."""
        cap = self.capture(fn, n, what, preroll)
        if cap is None:
            return region_us(self.torch, fn, n)
        return min(self.replay_us(cap, evict)[0] for _ in range(best_of))


OTHER_WORKLOADS = ("tiny", "sweep_k32", "sweep_k16", "sweep_k8", "sweep_k4", "sweep_k2",
                   "lstm1500_n8", "lstm1500_n32", "lstm1500_n128", "fc6_b1", "fc6_b16",
                   # Table 4's axes: balance range 25 / 50 / 100 at 60 % .. 80 % on the LSTM matrix
                   "lstm1500_b25_k10", "lstm1500_b25_k5", "lstm1500_b50_k20", "lstm1500_b50_k15",
                   "lstm1500_b50_k10", "lstm1500_b100_k40", "lstm1500_b100_k30", "lstm1500_b100_k20",
                   "bilstm1024",
                   # Sec. 4.2: convolution layers as products over im2col columns
                   "conv5_n196", "conv4_n784", "conv2_n12544", "conv1_n50176",
                   # Sec. 4.1's matrix shape, 50 % .. 97 % sparse, batch 1 and 8
                   "bench16k_k128", "bench16k_k64", "bench16k_k32", "bench16k_k16", "bench16k_k8",
                   "bench16k_k128_n8", "bench16k_k32_n8", "bench16k_k8_n8",
                   # balance ranges over 256 (16-bit offsets): 16 and 8 banks per row
                   "bench16k_b512_k64", "bench16k_b1024_k128", "bench16k_b512_k64_n8")


def rotation(alg_bytes):
    """Copies of a buffer of alg_bytes needed to exceed twice the last-level cache."""
    return max(2, -(-2 * LLC_BYTES // alg_bytes) + 1)


def quick_measure(torch, np, bs, workloads, dev, name, o_time, evict, timer, launches=200):
    """One workload, cold, `launches` graph-replayed launches: time per launch.
    o_time = measured launch floor, for eq. (5)'s ideal time."""
    wl, W, X = workloads.make(name)
    wide = wl.idx_bytes == 2            # balance range over 256: the calls with 16-bit offsets
    prune, spmv_call, spmm_call = ((bs.bs_prune_pack_wide, bs.bs_spmv_wide, bs.bs_spmm_wide) if wide else
                                   (bs.bs_prune_pack, bs.bs_spmv, bs.bs_spmm))
    Wd = torch.from_numpy(W).to(dev)
    Xd = torch.from_numpy(np.ascontiguousarray(X)).to(dev)
    vals, idx = prune(Wd, wl.bank, wl.k)
    alg = wl.spmv_bytes()
    R = rotation(alg)
    copies = [(vals, idx)] + [(vals.clone(), idx.clone()) for _ in range(R - 1)]
    spmm = wl.N > 1
    Y = torch.empty((wl.M, wl.N) if spmm else (wl.M,), dtype=torch.float32, device=dev)
    if spmm:
        code = bs.BS_F16 if wl.dtype == "f16" else bs.BS_F32
        need = (bs.bs_spmm_workspace_bytes_wide if wide else bs.bs_spmm_workspace_bytes)(
            code, wl.M, wl.K, wl.bank, wl.k, wl.N)
        ws = torch.zeros(max(16, need), dtype=torch.uint8, device=dev)
        fn = lambda i: spmm_call(copies[i % R][0], copies[i % R][1], wl.bank, Xd, out=Y, workspace=ws)
    elif wide:
        fn = lambda i: spmv_call(copies[i % R][0], copies[i % R][1], wl.bank, Xd, out=Y)
    else:
        cs = [bs.PreparedSpmv(v, ix, wl.bank, Xd, Y) for v, ix in copies]
        fn = lambda i: cs[i % R]()
    us = timer.us(fn, launches, name, evict)
    res = {"us": round(us, 2), "GBps": round(alg / us / 1e3, 1),
           "frac_of_8TBps": round(alg / us / 1e3 / HBM_PEAK_GBS, 3)}
    if spmm:
        res["TFLOPs"] = round(wl.flops() / us / 1e6, 2)
    # dense baselines, cold as well: the hand-written kernel and, as context, the vendor
    # library's dense product on the same matrix (torch.matmul -> rocBLAS / hipBLASLt; fp16
    # weights multiply an fp16 copy of X there).  The speedup printed first is against the
    # faster of the two.
    Rd = rotation(wl.dense_bytes())
    Wc = [Wd] + [Wd.clone() for _ in range(min(Rd, 8) - 1)]
    n_d = 10 if spmm else 50
    dfn = (lambda i: bs.bs_dense_gemm(Wc[i % len(Wc)], Xd, out=Y)) if spmm else \
          (lambda i: bs.bs_dense_gemv(Wc[i % len(Wc)], Xd, out=Y))
    d_us = timer.us(dfn, n_d, name + " dense", evict)
    lib_us = None
    try:
        Xl = Xd if wl.dtype == "f32" else Xd.half()
        Yl = torch.empty(Y.shape, dtype=Xl.dtype, device=dev)
        lib = lambda i: torch.matmul(Wc[i % len(Wc)], Xl, out=Yl)
        for i in range(3):
            lib(i)
        lib_us = timer.us(lib, n_d, name + " dense (vendor library)", evict)
    except Exception as exc:
        res["dense_library_error"] = str(exc)[:80]
    res["speedup_vs_faster_dense"] = round(min(d_us, lib_us if lib_us else d_us) / us, 2)
    res["dense_us"] = round(d_us, 1)
    if lib_us:
        res["dense_library_us"] = round(lib_us, 1)
    res["speedup_vs_own_dense"] = round(d_us / us, 2)
    # eq. (5): the dense time scaled by the kept fraction, launch overhead not scaled
    res["ideal_us_eq5"] = round(max(d_us - o_time, 0.0) * (1 - wl.sparsity) + o_time, 2)
    # pruning + packing this matrix (W rotates as for the dense baseline)
    p_out = (torch.empty_like(vals), torch.empty_like(idx))
    pfn = lambda i: prune(Wc[i % len(Wc)], wl.bank, wl.k, out=p_out)
    p_us = timer.us(pfn, 6, name + " prune_pack", evict, preroll=2)
    res["prune_pack_us"] = round(p_us, 1)
    res["prune_pack_GBps"] = round((W.nbytes + wl.nnz * (wl.val_bytes + wl.idx_bytes)) / p_us / 1e3, 1)
    return res


def spmv_kernel_name(bs, wl):
    """The instantiation bs_spmv launches for this workload, as the profiles name it."""
    code = bs.BS_F16 if wl.dtype == "f16" else bs.BS_F32
    p = bs.bs_spmv_plan(code, wl.M, wl.K, wl.bank, wl.k)
    if p["slab_kernel"]:
        return "spmv_slab_kernel", p
    vt = "__half" if wl.dtype == "f16" else "float"
    return f"spmv_kernel<{vt},{p['ch']},{p['lpr']},{p['u']}> {p['workgroups']} x {p['threads']}", p


def sweep(args, torch, np, bs, probe, workloads, dev):
    """Launch-shape sweep of bs_spmv_ex on one workload, cold, graph of 400 launches, best of 3."""
    wl, W, X = workloads.make(args.workload)
    Wd = torch.from_numpy(W).to(dev)
    vals, idx = bs.bs_prune_pack(Wd, wl.bank, wl.k)
    del Wd
    xd = torch.from_numpy(np.ascontiguousarray(X)).to(dev)
    alg = wl.spmv_bytes()
    R = rotation(alg)
    copies = [(vals, idx)] + [(vals.clone(), idx.clone()) for _ in range(R - 1)]
    y = torch.empty(wl.M, dtype=torch.float32, device=dev)
    evict = Evictor(torch, probe, dev)
    timer = GraphTimer(torch, probe, dev)
    n = 400
    code = bs.BS_F16 if wl.dtype == "f16" else bs.BS_F32

    def timed(fn):
        cap = timer.capture(fn, n, "sweep")
        if cap is None:
            return None
        return round(min(timer.replay_us(cap, evict)[0] for _ in range(3)), 3)

    out = {"workload": wl.name, "algorithmic_bytes": alg, "launches_per_graph": n, "copies": R,
           "default": {"plan": bs.bs_spmv_plan(code, wl.M, wl.K, wl.bank, wl.k)}}
    cs = [bs.PreparedSpmv(v, ix, wl.bank, xd, y) for v, ix in copies]
    out["default"]["us"] = timed(lambda i: cs[i % R]())
    print(f"default {out['default']}", file=sys.stderr, flush=True)
    table = []
    for lpr in (4, 8, 16, 32, 64):
        for thr in (64, 128, 256, 384, 512, 768, 1024):
            if thr % lpr:
                continue
            try:
                plan = bs.bs_spmv_plan(code, wl.M, wl.K, wl.bank, wl.k, lpr, thr // lpr)
            except bs.BsError:
                continue
            cs = [bs.PreparedSpmv(v, ix, wl.bank, xd, y, lpr, thr // lpr) for v, ix in copies]
            us = timed(lambda i: cs[i % R]())
            row = {"lanes_per_row": lpr, "rows_per_wg": thr // lpr, "threads": thr,
                   "workgroups": plan["workgroups"], "chunk_slots": plan["u"], "us": us,
                   "GBps": round(alg / us / 1e3, 1) if us else None}
            table.append(row)
            print(row, file=sys.stderr, flush=True)
    out["shapes"] = table
    # the floor for the same bytes, several shapes of the read-only kernel
    same = (alg + 15) // 16 * 16
    bufs = [torch.empty(same, dtype=torch.uint8, device=dev) for _ in range(R)]
    for b_ in bufs:
        b_.fill_(1)
    out["read_only_us_by_pieces_per_lane"] = {
        str(pc): timed(lambda i: probe.probe_stream_read(bufs[i % R], pc)) for pc in (1, 2, 4, 8)}
    del bufs
    out["empty_kernel_us"] = {f"{g}x{t}": timed(lambda i: probe.probe_empty(g, t))
                              for g in (1, 64, 256, 750, 2207, 8828) for t in (64, 256, 1024)}
    print(json.dumps(out))
    return 0


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
    from paper_1811_00206_amd import probe
    from paper_1811_00206_amd import workloads

    if not os.path.exists(bs.library_path()) or not os.path.exists(probe.library_path()):
        from paper_1811_00206_amd.build import build_library
        build_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    bs.bs_init()
    if args.sweep:
        return sweep(args, torch, np, bs, probe, workloads, dev)

    wl, W, X = workloads.make(args.workload)
    K, W_steps = args.steps, args.warmup
    Wd = torch.from_numpy(W).to(dev)
    Xd = torch.from_numpy(np.ascontiguousarray(X)).to(dev)
    vals, idx = bs.bs_prune_pack(Wd, wl.bank, wl.k)        # the product path packs on the GPU
    torch.cuda.synchronize()

    alg_bytes = wl.spmv_bytes()
    R = 1 if args.warm else max(rotation(alg_bytes), args.copies)
    copies = [(vals, idx)] + [(vals.clone(), idx.clone()) for _ in range(R - 1)]
    evict = None if args.warm else Evictor(torch, probe, dev)
    spmm = wl.N > 1
    if spmm:
        Y = torch.empty((wl.M, wl.N), dtype=torch.float32, device=dev)
        ws_bytes = bs.bs_spmm_workspace_bytes(bs.BS_F16 if wl.dtype == "f16" else bs.BS_F32,
                                              wl.M, wl.K, wl.bank, wl.k, wl.N)
        ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
        kernel_name, plan = "bs_spmm", {}
    else:
        Y = torch.empty(wl.M, dtype=torch.float32, device=dev)
        kernel_name, plan = spmv_kernel_name(bs, wl)

    # arguments marshalled once per matrix copy: a step is then one C-ABI call
    calls = None if spmm else [bs.PreparedSpmv(v, ix, wl.bank, Xd, Y) for v, ix in copies]

    def step(i):
        if spmm:
            v, ix = copies[i % R]
            bs.bs_spmm(v, ix, wl.bank, Xd, out=Y, workspace=ws)
        else:
            calls[i % R]()

    for i in range(W_steps):
        step(i)
    torch.cuda.synchronize()

    # ---- the timed region: exactly K steps between two events on the launch stream.
    # The K launches are captured once into a HIP graph (the deployment form of a
    # launch-bound loop), replayed once untimed, and replayed inside the region; --eager
    # launches them from Python instead.  Cold runs enqueue the evicting read right before
    # the first event, so the K launches start with empty caches and (rotating over R
    # copies) never come back to a copy before 2 x the last-level cache has gone by.
    mode = "eager"
    timer = GraphTimer(torch, probe, dev)
    # pre-roll launches continue the rotation (copies K, K+1, ...), so with K < R they touch
    # copies the timed launches do not
    graph = None if args.eager else timer.capture(step, K, "headline")
    replay_events_us = None
    t_wall0 = time.perf_counter()
    if graph is not None:
        mode = (f"hip graph: {graph[2]} pre-roll launches, wall-clock stamp, the K launches, "
                "wall-clock stamp")
        us_per_step, replay_events_us = timer.replay_us(graph, evict)
    else:
        if evict is not None:
            evict()
        us_per_step = region_us(torch, step, K)
    t_wall = time.perf_counter() - t_wall0
    # the same region a few more times (extras): how far one sample of K steps can be off
    trials = []
    if graph is not None and not args.no_extras:
        trials = [round(timer.replay_us(graph, evict)[0], 3) for _ in range(4)]

    value = alg_bytes / us_per_step / 1e3                  # GB/s
    n_launched = K + (graph[2] if graph is not None else 0)
    touched = min(K, R) * alg_bytes
    if args.warm:
        residency = "warm (one copy, cache resident)"
    else:
        residency = (f"cold: {EVICT_BYTES >> 20} MB of unrelated memory streamed right before the timed "
                     f"region; its {K} launches read {min(K, R)} distinct copies of vals/idx "
                     f"({touched / 1e6:.0f} MB)"
                     + (f", a copy comes round again after {R - 1} others ({(R - 1) * alg_bytes / 1e6:.0f} MB, "
                        f"over twice the {LLC_BYTES >> 20} MB last-level cache)" if K > R else
                        ", each exactly once"))

    traffic = None
    rec = MEASURED_TRAFFIC.get((wl.name, "warm" if args.warm else "cold"))
    if rec and rec["kernel"] == kernel_name:
        traffic = rec["bytes"]

    roofline = {"bound": "hbm", "achieved": round(value, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(value / HBM_PEAK_GBS, 4),
                "traffic": traffic,
                "kernel": kernel_name,
                "kernel_us": round(us_per_step, 3),
                "how": ("GPU wall-clock stamps (one-lane kernels inside the captured graph) right before "
                        "and after the K launches, minus the interval of two adjacent stamps, / K"
                        if graph is not None else "HIP events around K eager launches / K"),
                "stamp_gap_us": round(timer.gap_us, 3),
                "replay_events_us_per_launch": (round(replay_events_us, 3) if replay_events_us else None)}

    # ---- the machine's floor in the same protocol and the same run: an empty kernel of
    # the product's launch shape, and a kernel that only reads the product's algorithmic
    # bytes (rotating buffers, same eviction, same K).
    if graph is not None and not args.warm:
        try:
            same = (alg_bytes + 15) // 16 * 16
            bufs = [torch.empty(same, dtype=torch.uint8, device=dev) for _ in range(R)]
            for b_ in bufs:
                b_.fill_(1)
            g_floor = timer.capture(lambda i: probe.probe_stream_read(bufs[i % R]), K, "floor: read-only kernel")
            if g_floor is not None:
                floor_us = min(timer.replay_us(g_floor, evict)[0] for _ in range(3))
                roofline["floor_us"] = round(floor_us, 3)
                roofline["floor_GBps"] = round(same / floor_us / 1e3, 1)
                roofline["frac_of_floor"] = round(floor_us / us_per_step, 3)
                roofline["floor"] = ("a kernel that only reads the same number of bytes (16 bytes per "
                                     "lane, one piece per lane), same protocol (pre-roll, stamps, K "
                                     "launches), same eviction, rotating buffers; best of 3")
                # ... and the same kernel when it also stores as many words as the product has
                # results (one lane in every few stores its sum to consecutive words)
                n_out = wl.M * wl.N
                every = max(1, (same // 16) // n_out)
                sink = torch.zeros((same // 16 + 256) // every + 2, dtype=torch.int32, device=dev)
                g_fs = timer.capture(lambda i: probe.probe_stream_read(bufs[i % R], 1, sink=sink, store_mode=1,
                                                                       store_every=every),
                                     K, "floor: read-and-store kernel")
                if g_fs is not None:
                    fs_us = min(timer.replay_us(g_fs, evict)[0] for _ in range(3))
                    roofline["floor_with_result_stores_us"] = round(fs_us, 3)
                    roofline["frac_of_floor_with_result_stores"] = round(fs_us / us_per_step, 3)
                del g_fs, sink
            del bufs, g_floor
            grid, thr = (plan.get("workgroups") or 256), (plan.get("threads") or 256)
            g_empty = timer.capture(lambda i: probe.probe_empty(int(grid), int(thr)), max(K, 200),
                                    "floor: empty kernel")
            if g_empty is not None:
                roofline["empty_launch_us"] = round(
                    min(timer.replay_us(g_empty)[0] for _ in range(3)), 3)
            del g_empty
        except Exception as exc:                 # never lose the headline line
            roofline["floor_error"] = str(exc)[:200]

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
                   "residency": residency,
                   "bytes_touched_by_timed_launches": touched,
                   "launches_per_replay": n_launched,
                   "launch": mode,
                   "algorithmic_bytes_per_step": alg_bytes,
                   "flop_per_step": wl.flops()},
        "roofline": roofline,
    }

    extras = {"gflops": round(wl.flops() / us_per_step / 1e3, 1),
              "host_wall_s_timed_region": round(t_wall, 3)}
    if trials:
        extras["further_trials_us_per_step"] = trials

    if not args.no_extras:
        d_us, o_time = float("nan"), roofline.get("empty_launch_us", 0.0)
        try:                                     # never lose the headline line
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
                # the same matrix from cache (one copy): what an LSTM time step loop sees,
                # in the protocol of `value` (a graph of launches back to back)
                gw = timer.capture(lambda i: bs.bs_spmv(vals, idx, wl.bank, Xd, out=Y), 64, "warm product")
                if gw is not None:
                    wg_us = min(timer.replay_us(gw)[0] for _ in range(5))
                    extras["warm_us_per_launch_graph"] = round(wg_us, 3)
                    extras["warm_GBps_per_launch_graph"] = round(alg_bytes / wg_us / 1e3, 1)
                del gw

            # dense baseline on the unpruned-shape matrix, same residency protocol
            dense_bytes = wl.dense_bytes()
            Rd = 1 if args.warm else rotation(dense_bytes)
            Wc = [Wd] + [Wd.clone() for _ in range(Rd - 1)]
            if spmm:
                d_us = timer.us(lambda i: bs.bs_dense_gemm(Wc[i % Rd], Xd, out=Y), 20, "dense gemm", evict)
            else:
                d_us = timer.us(lambda i: bs.bs_dense_gemv(Wc[i % Rd], Xd, out=Y), 200, "dense gemv", evict)
            del Wc
            extras["dense_us"] = round(d_us, 2)
            extras["dense_GBps"] = round(dense_bytes / d_us / 1e3, 1)
            extras["speedup_vs_dense"] = round(d_us / us_per_step, 2)   # both: region time per launch
            # eq. (5) of the paper with the measured dense time and the measured launch floor
            o_time = roofline.get("empty_launch_us", extras.get("launch_floor_us", 0.0))
            extras["ideal_us_eq5"] = round((d_us - o_time) * (1 - wl.sparsity) + o_time, 2)
            # one-time pruning + packing of the dense matrix
            p_out = (torch.empty_like(vals), torch.empty_like(idx))
            p_us = timer.us(lambda i: bs.bs_prune_pack(Wd, wl.bank, wl.k, out=p_out), 10, "prune_pack", evict, preroll=2)
            p_bytes = W.nbytes + wl.nnz * (wl.val_bytes + 1)
            extras["prune_pack_us"] = round(p_us, 1)
            extras["prune_pack_GBps"] = round(p_bytes / p_us / 1e3, 1)
            # one more pruning round on the packed matrix: half the weights of every bank
            if wl.k >= 2:
                k2 = wl.k // 2
                r_out = bs.bs_reprune(vals, idx, wl.bank, k2)
                r_us = timer.us(lambda i: bs.bs_reprune(vals, idx, wl.bank, k2, out=r_out), 20, "reprune", preroll=2)
                extras["reprune_to_half_us"] = round(r_us, 1)
                extras["reprune_GBps"] = round((wl.nnz + wl.M * (wl.K // wl.bank) * k2) *
                                               (wl.val_bytes + 1) / r_us / 1e3, 1)
            ev.close()
        except Exception as exc:
            extras["baselines_error"] = str(exc)[:200]

        # more of the machine's floor: a large streaming read, LDS gather rates, and the
        # grid-wide barrier a persistent multi-step kernel would need once per step
        try:
            floor = {}
            big = 288 << 20
            bufs = [torch.empty(big, dtype=torch.uint8, device=dev) for _ in range(3)]
            for b_ in bufs:
                b_.fill_(1)
            t_big = timer.us(lambda i: probe.probe_stream_read(bufs[i % 3]), 12, "floor: 288 MB read", preroll=3)
            floor["stream_read_288MB_us"] = round(t_big, 2)
            floor["stream_read_288MB_GBps"] = round(big / t_big / 1e3, 1)
            del bufs
            # what storing costs a kernel of this size: the read-only kernel of the product's bytes
            # with different store patterns (cold, the protocol of `value`)
            same = (alg_bytes + 15) // 16 * 16
            if not args.warm and same // 16 <= 16384 * 256:
                Rf = rotation(same)
                bufs = [torch.empty(same, dtype=torch.uint8, device=dev) for _ in range(Rf)]
                for b_ in bufs:
                    b_.fill_(1)
                sink = torch.zeros(((same // 16 + 255) // 256 + 1) * 32, dtype=torch.int32, device=dev)
                n_out = wl.M * wl.N
                every = max(1, (same // 16) // n_out)
                stores = {}
                for key, mode, ev_ in (("no_store", 0, 1),
                                       (f"one_word_per_{every}_lanes_plain_store", 1, every),
                                       (f"one_word_per_{every}_lanes_nontemporal_store", 2, every),
                                       (f"one_word_per_{every}_lanes_agent_scope_store", 3, every),
                                       ("one_word_per_32_lanes_plain_store", 1, 32),
                                       ("one_instruction_per_workgroup_32_adjacent_words", 4, 32),
                                       ("one_instruction_per_workgroup_1_word", 4, 1)):
                    cap = timer.capture(lambda i: probe.probe_stream_read(bufs[i % Rf], 1, sink=sink, store_mode=mode,
                                                                          store_every=ev_), 400, "floor: stores")
                    if cap is not None:
                        stores[key] = round(min(timer.replay_us(cap, evict)[0] for _ in range(3)), 3)
                floor["read_same_bytes_and_store_us"] = stores
                del bufs, sink
            # what an LDS gather costs: 256 workgroups of 768 lanes that only issue LDS reads;
            # ns per wavefront read and compute unit
            reads, thr = 16000, 768
            t0 = timer.us(lambda i: probe.probe_lds_gather(thr, 0, 16, 8), 4, "floor: lds fill", preroll=1)
            lds = {}
            for key, pattern, lanes in (("b128_adjacent_1KB", 0, 16), ("b128_rows_of_256B", 1, 16),
                                        ("b128_rows_of_128B", 1, 8), ("b128_rows_of_64B", 1, 4),
                                        ("b128_rows_of_32B", 1, 2), ("b32_random_word_per_lane", 2, 16),
                                        ("b32_random_row_word_is_lane", 3, 16)):
                t = timer.us(lambda i: probe.probe_lds_gather(thr, pattern, lanes, reads), 4,
                             "floor: lds gather", preroll=1)
                lds[key] = round((t - t0) * 1e3 / ((reads - 8) * thr / 64), 3)
            floor["lds_gather_ns_per_wavefront_read_per_cu"] = lds
            # grid barrier: workgroups -> us per round (256 lanes each, a 6 KB vector read and
            # rewritten per round as an LSTM-1500 step would; bounded waits)
            sync = torch.zeros(4, dtype=torch.int32, device=dev)
            hbuf = torch.zeros(2 * 1500, dtype=torch.float32, device=dev)
            bar = {}
            n_rounds = 500
            for wgs in (32, 64, 128, 256):
                for bmode, tag in ((0, "acquire_polls"), (1, "relaxed_polls")):
                    sync.zero_()
                    us = region_us(torch, lambda i: probe.probe_grid_barrier(wgs, 256, n_rounds, 1500, bmode,
                                                                             sync, hbuf), 1) / n_rounds
                    arrivals, aborted = (int(v) for v in sync[:2].tolist())
                    bar[f"{wgs}_wgs_{tag}"] = {"us_per_round": round(us, 2),
                                               "complete": arrivals == n_rounds * wgs and not aborted}
            floor["grid_barrier"] = bar
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
                gl = timer.capture(lambda i: bs.bs_lstm_sequence(vals, idx, wl.bank, Xs, h0, bias, c0,
                                                                 H_all=H_all), 1, "lstm sequence", preroll=1)
                if gl is not None:
                    l_us = min(timer.replay_us(gl)[0] for _ in range(5)) / T
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
            only = [n for n in args.only.split(",") if n]
            others = {}
            for name in (only or OTHER_WORKLOADS):
                if name not in workloads.WORKLOADS:
                    continue
                try:
                    others[name] = quick_measure(torch, np, bs, workloads, dev, name, o_time, evict, timer)
                except Exception as exc:             # never lose the headline line
                    others[name] = {"error": str(exc)[:200]}
                torch.cuda.empty_cache()
            extras["other_workloads_cold"] = others
    if EAGER_FALLBACKS:
        extras["timed_as_eager_launches"] = EAGER_FALLBACKS
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
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
