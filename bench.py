#!/usr/bin/env python3
"""Benchmark of the W1A6 linear forward (rotate+quantize, then binary GEMM + PSP + dequant).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-extra]

A step is one pass of the whole hot path over one batch of synthetic activations: one
bwla_decode_forward call (rotation, codes, binary GEMM, PSP branch, dequantization: one kernel
launch where the library has a single-launch kernel for the shape, else the launches of
bwla_rotate_quant and bwla_linear_forward back to back).  Successive steps use different packed
copies of the layer, 512 MB of them, as the layers of a model are all distinct; and every timed
region starts behind a pass over a 768 MB buffer, so whatever the number of steps the sign bits
stream from HBM, not from the 256 MB last-level cache.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E
INT8_PEAK_TOPS = 5000.0       # dense INT8 MFMA
CACHE_DEFEAT_BYTES = 512 << 20
FLUSH_BYTES = 768 << 20
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "pmc_hbm_traffic.txt")


def measured_traffic():
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE in separate
    runs, each scaled by what the same counter reads for a plain device copy of known size in the
    same run), read from the tracked summary of those runs: its lines
        traffic <workload> <kernel> <fetch bytes> <write bytes>
    Returns {(workload, kernel): bytes}; empty when the summary is missing."""
    out = {}
    try:
        with open(TRAFFIC_FILE) as f:
            for ln in f:
                p = ln.split()
                if len(p) == 5 and p[0] == "traffic":
                    out[(p[1], p[2])] = int(p[3]) + int(p[4])
    except OSError:
        pass
    return out


def linear_forward_bytes(cfg) -> int:
    """Algorithmic HBM bytes of one bwla_linear_forward launch: sign bits, alpha, V (fp16),
    codes, per-token scale and code sum, T, and the fp32 output."""
    M, K, N, r = cfg.M, cfg.K, cfg.N, cfg.r
    return N * K // 8 + 2 * N + 2 * N * r + M * K + 8 * M + 4 * M * r + 4 * M * N


def rotate_quant_bytes(cfg) -> int:
    """Algorithmic bytes of one bwla_rotate_quant call: X, the factors, U (fp16), codes,
    scale, code sum and T."""
    xb = 2 if cfg.x_dtype == "bf16" else 4
    return cfg.M * cfg.K * xb + 4 * (cfg.n1 ** 2 + cfg.n2 ** 2) + 2 * cfg.K * cfg.r + cfg.M * cfg.K \
        + 8 * cfg.M + 4 * cfg.M * cfg.r


def layer_bytes(cfg) -> int:
    """Algorithmic bytes of the whole layer: everything either call reads or writes once."""
    return linear_forward_bytes(cfg) + rotate_quant_bytes(cfg)


def gemm_ops(cfg) -> int:
    return 2 * cfg.M * cfg.N * cfg.K


_flush_buf = None
_flush_sink = None


def flush_caches(torch):
    """One streaming read of 768 MB on the current stream: afterwards neither the L2s nor the 256 MB
    last-level cache hold anything of the layers.  (A read, not a read-modify-write: the dirty lines a
    writing pass leaves behind drain to HBM during the next few hundred microseconds and slowed the
    first forty or so layer launches behind it by 1 us each -- which a timed region of 20 steps carried
    in full and one of 400 steps hardly at all.)"""
    global _flush_buf, _flush_sink
    from paper_2605_00422_amd import binding as B
    if _flush_buf is None:
        _flush_buf = torch.zeros(FLUSH_BYTES // 4, dtype=torch.int32, device="cuda:0")
        _flush_sink = torch.zeros(1 << 16, dtype=torch.int32, device="cuda:0")
    B.probe_hbm_read(_flush_buf, _flush_sink)


class Workload:
    """One layer on the GPU with `copies` packed replicas and preallocated outputs."""

    def __init__(self, cfg, copies=None, centered=False, act_bits=6, asym=False, nibble=False):
        import numpy as np
        import torch
        from paper_2605_00422_amd import binding as B
        from paper_2605_00422_amd import inputs as syn
        self.cfg, self.B, self.torch = cfg, B, torch
        self.act_bits = act_bits
        self.nibble = nibble          # 4-bit codes packed two to a byte between the two calls
        dev = "cuda:0"
        d = syn.make_layer(cfg)
        self.data = d
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        U = t(d.U) if cfg.r > 0 else None
        V = t(d.V) if cfg.r > 0 else None
        # centered: binarization with the row shift, on weights with a per-channel offset
        W = syn.shifted_weights(d) if centered else d.W
        first = B.pack_weights(t(W), t(d.R1), t(d.R2), U, V, cfg.n1, cfg.n2, centered=centered, asym=asym)
        torch.cuda.synchronize()
        nbytes = first.blob.numel()
        if copies is None:
            copies = max(2, math.ceil(CACHE_DEFEAT_BYTES / nbytes))
        self.layers = [first]
        for _ in range(copies - 1):
            blob = first.blob.clone()
            desc = B.BwlaLayer.from_buffer_copy(first.desc)
            desc.d_blob = blob.data_ptr()
            self.layers.append(B.PackedLayer(desc, blob))
        X = t(d.X)
        self.X = X.to(torch.bfloat16) if cfg.x_dtype == "bf16" else X
        self.act = B.Activations(first, cfg.M)
        self.Y = torch.empty((cfg.M, cfg.N), dtype=torch.float32, device=dev)
        # 1 where bwla_decode_forward has a single-launch kernel for the shape (at any code width)
        self.launches = B.decode_forward_launches(first, cfg.M, cfg.x_dtype == "bf16")
        if nibble:
            self.q4 = torch.empty((cfg.M, cfg.K // 2), dtype=torch.uint8, device=dev)
            self.launches = 2
        torch.cuda.synchronize()

    def step(self, i):
        L = self.layers[i % len(self.layers)]
        if self.nibble:
            self.B.rotate_quant(L, self.X, self.act, self.act_bits)
            self.B.pack_codes_a4(self.act.q, self.q4)
            self.B.linear_forward_a4(L, self.q4, self.act, self.Y)
            return
        self.B.decode_forward(L, self.X, self.act, self.Y, act_bits=self.act_bits)

    def only_rotate(self, i):
        self.B.rotate_quant(self.layers[i % len(self.layers)], self.X, self.act, self.act_bits)

    def only_forward(self, i):
        if self.nibble:
            self.B.linear_forward_a4(self.layers[i % len(self.layers)], self.q4, self.act, self.Y)
            return
        self.B.linear_forward(self.layers[i % len(self.layers)], self.act, self.Y)

    def only_forward_gated(self, i):
        """The same GEMM with the MLP gate applied to neighbouring outputs before the store
        (bf16 h, M x N/2); up to 16 tokens no scratch is needed."""
        if not hasattr(self, "H"):
            self.H = self.torch.empty((self.cfg.M, self.cfg.N // 2), dtype=self.torch.bfloat16, device="cuda:0")
        self.B.linear_forward_swiglu(self.layers[i % len(self.layers)], self.act, self.H)

    def time_loop(self, fn, steps, warmup):
        """Average milliseconds per call of fn over `steps` back-to-back calls, bracketed by
        events on the stream the kernels are launched on (torch's current stream)."""
        torch = self.torch
        for i in range(warmup):
            fn(i)
        flush_caches(torch)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            fn(warmup + i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    def time_graph(self, fn, steps, warmup, replays=5):
        """The same K calls captured once into a HIP graph and replayed: per-call milliseconds
        without host launch overhead (how a decode loop would be deployed).  `replays` timed
        replays, each behind a cache flush; returns (median, minimum).  The span of the K calls is
        read off the GPU's constant 100 MHz counter by two one-wavefront launches captured in front
        of and behind them (the gap to the first call and from the last count as the gaps between
        calls do); events around the replay measure the same span plus the replay's own start on the
        GPU -- some 25 us, which K = 400 calls do not notice and K = 20 would carry as 1 us each; that
        figure is kept as last_graph_events_ms and reported beside the other."""
        torch = self.torch
        for i in range(max(warmup, 3)):
            fn(i)
        torch.cuda.synchronize()
        B = self.B
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        t0 = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        t1 = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        with torch.cuda.stream(s):
            with torch.cuda.graph(g, stream=s):
                B.probe_clock(t0)
                for i in range(steps):
                    fn(warmup + i)
                B.probe_clock(t1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ms, ms_ev = [], []
        for _ in range(replays):
            flush_caches(torch)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            ms_ev.append(e0.elapsed_time(e1) / steps)
            ms.append((t1.item() - t0.item()) * 1e-5 / steps)          # ticks of 10 ns -> ms
        ms.sort()
        ms_ev.sort()
        self.last_graph_events_ms = ms_ev[len(ms_ev) // 2]
        return ms[len(ms) // 2], ms[0]


def measure(cfg, steps, warmup, use_graph=True, centered=False, act_bits=6, asym=False, nibble=False):
    w = Workload(cfg, centered=centered, act_bits=act_bits, asym=asym, nibble=nibble)
    out = {"workload": cfg.name + ("+row_shift" if centered else "") + (f"+a{act_bits}" if act_bits != 6 else "")
           + ("+asym" if asym else "") + ("+nibbles" if nibble else ""),
           "M": cfg.M, "K": cfg.K, "N": cfg.N, "r": cfg.r,
           "kron": f"{cfg.n1}x{cfg.n2}", "layer_copies": len(w.layers), "launches_per_layer": w.launches}
    if nibble:
        w.step(0)            # the packed codes exist before the GEMM is timed on its own
    ms_step = w.time_loop(w.step, steps, warmup)
    ms_fwd = w.time_loop(w.only_forward, steps, warmup)
    ms_rot = w.time_loop(w.only_rotate, steps, warmup)
    out["stream"] = {"us_per_layer": ms_step * 1e3, "us_linear_forward": ms_fwd * 1e3,
                     "us_rotate_quant": ms_rot * 1e3}
    if use_graph:
        try:
            gs, gs_min = w.time_graph(w.step, steps, warmup)
            gs_events = w.last_graph_events_ms
            gf, _ = w.time_graph(w.only_forward, steps, warmup)
            gr, _ = w.time_graph(w.only_rotate, steps, warmup)
            out["graph"] = {"us_per_layer": gs * 1e3, "us_per_layer_min": gs_min * 1e3,
                            "us_per_layer_events": gs_events * 1e3,
                            "us_linear_forward": gf * 1e3, "us_rotate_quant": gr * 1e3}
            if cfg.name.startswith("cfg1_7b_gateup") and cfg.M <= 16:
                out["graph"]["us_linear_forward_gated"] = w.time_graph(w.only_forward_gated, steps, warmup)[0] * 1e3
        except Exception as ex:  # graph capture is an optimisation of the launch path only
            out["graph"] = {"error": repr(ex)[:200]}
    return w, out


def best_of(res):
    """The faster of the stream loop and the graph replay (median) of the whole layer."""
    best, mode = res["stream"], "stream"
    if "graph" in res and "us_per_layer" in res["graph"] and res["graph"]["us_per_layer"] < best["us_per_layer"]:
        best, mode = res["graph"], "graph"
    return best, mode


class Peaks:
    """What this GPU reaches on a pure streaming read of a given size and on a loop of INT8 MFMAs
    only (the library's two measurement kernels), timed like the workloads: events on the
    launch stream around a graph replay, every read launch on a window of a 768 MB buffer that the launches before it
    did not touch."""

    def __init__(self, torch, B):
        self.torch, self.B = torch, B
        flush_caches(torch)
        self.sink = torch.zeros(16384, dtype=torch.int32, device="cuda:0")
        self._read = {}
        self._mfma = None

    def hbm_read_gbps(self, nbytes, launches=40):
        nbytes = max(4096, min(int(nbytes), FLUSH_BYTES // 3) // 4096 * 4096)
        if nbytes in self._read:
            return self._read[nbytes]
        torch = self.torch
        buf = _flush_buf.view(torch.uint8)
        nwin = FLUSH_BYTES // nbytes
        launches = max(1, min(launches, nwin - 1))      # the buffer's tail is what the flush wrote last
        wins = [buf[i * nbytes:(i + 1) * nbytes] for i in range(launches)]
        self.B.probe_hbm_read(wins[0], self.sink)
        torch.cuda.synchronize()
        # replayed from a graph like the workloads, so that host launch overhead is not in the figure
        g = torch.cuda.CUDAGraph()
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            with torch.cuda.graph(g, stream=st):
                for wv in wins:
                    self.B.probe_hbm_read(wv, self.sink)
        torch.cuda.synchronize()
        best = 0.0
        for _ in range(3):
            flush_caches(torch)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            best = max(best, nbytes * launches / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        self._read[nbytes] = best
        return best

    def mfma_int8_tops(self):
        if self._mfma is None:
            torch = self.torch
            self.B.probe_mfma_int8(1000, self.sink)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ops = self.B.probe_mfma_int8(20000, self.sink)
            e1.record()
            torch.cuda.synchronize()
            self._mfma = ops / (e0.elapsed_time(e1) * 1e-3) / 1e12
        return self._mfma


def microbench(torch, B):
    """Latencies the decode path lives with, measured with the library's probe launches: the period
    of back-to-back launches of a kernel that does nothing (from a graph, like the workloads), and the
    latency of one dependent load that misses every cache / that hits the L2."""
    n = 400
    g = torch.cuda.CUDAGraph()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        B.probe_empty_launch()
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=st):
            for _ in range(n):
                B.probe_empty_launch()
    torch.cuda.synchronize()
    period = 1e9
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        period = min(period, e0.elapsed_time(e1) * 1e3 / n)
    out = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    flush_caches(torch)
    buf = _flush_buf.view(torch.uint8)
    iters = 2000
    # cold: a new 4 KiB page region every load (stride 1 MiB + 4 KiB over the flushed buffer's head)
    B.probe_load_latency(buf[:FLUSH_BYTES // 2], (1 << 20) + 4096, 300, out)
    torch.cuda.synchronize()
    miss = out[0].item() * 10.0 / 300
    small = buf[:1 << 20]
    B.probe_load_latency(small, 128, (1 << 20) // 128, out)       # first walk brings the MiB into the L2
    B.probe_load_latency(small, 128, iters, out)
    torch.cuda.synchronize()
    l2 = out[0].item() * 10.0 / iters
    return {"empty_launch_period_us": period, "dependent_load_ns": {"miss": miss, "l2_hit": l2},
            "what": "graph of 400 launches of an empty kernel (256 x 512 threads); one lane's dependent 4-byte loads, "
                    "1 MiB + 4 KiB apart over a flushed 384 MiB buffer / 128 bytes apart over 1 MiB read just before"}


def roofline_for(cfg, launches, us_layer, us_forward, peaks, traffic, workload=None):
    """Roofline of the dominant kernel: the single-launch decode kernel where it serves the layer
    (then the kernel is the layer), else the binary GEMM inside bwla_linear_forward; with the
    whole layer (all launches, all bytes or operations) against the same peak beside it."""
    workload = workload or cfg.name
    hbm_bound = layer_bytes(cfg) / (HBM_PEAK_GBPS * 1e9) >= gemm_ops(cfg) / (INT8_PEAK_TOPS * 1e12)
    if launches == 1:
        kernel, t, nbytes = "decode_layer_kernel", us_layer * 1e-6, layer_bytes(cfg)
    else:
        kernel = "gemm_decode_bs_kernel" if cfg.M <= 16 else "gemm_prefill_direct_kernel"
        t, nbytes = us_forward * 1e-6, linear_forward_bytes(cfg)
    tl = us_layer * 1e-6
    if hbm_bound:
        a = nbytes / t / 1e9
        pm = peaks.hbm_read_gbps(nbytes) if peaks else None
        r = {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": a / HBM_PEAK_GBPS,
             "traffic": traffic.get((workload, kernel)), "kernel": kernel, "bytes_per_launch": nbytes,
             "us_per_launch": t * 1e6,
             "peak_measured": pm, "frac_of_measured": (a / pm if pm else None),
             "peak_measured_what": "one streaming-read launch of the same number of bytes, cold",
             "peak_measured_large": (peaks.hbm_read_gbps(FLUSH_BYTES // 3) if peaks else None),
             "layer": {"achieved": layer_bytes(cfg) / tl / 1e9, "frac": layer_bytes(cfg) / tl / 1e9 / HBM_PEAK_GBPS,
                       "bytes": layer_bytes(cfg), "us": us_layer, "launches": launches}}
        return r
    a = gemm_ops(cfg) / t / 1e12
    pm = peaks.mfma_int8_tops() if peaks else None
    return {"bound": "mfma", "achieved": a, "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": a / INT8_PEAK_TOPS,
            "traffic": traffic.get((workload, kernel)), "kernel": kernel, "ops_per_launch": gemm_ops(cfg),
            "us_per_launch": t * 1e6,
            "peak_measured": pm, "frac_of_measured": (a / pm if pm else None),
            "peak_measured_what": "a launch of INT8 16x16x64 MFMAs on register operands only",
            "layer": {"achieved": gemm_ops(cfg) / tl / 1e12, "frac": gemm_ops(cfg) / tl / 1e12 / INT8_PEAK_TOPS,
                      "ops": gemm_ops(cfg), "us": us_layer, "launches": launches}}


def side_kernel_report(cfg, us_rotate):
    """bwla_rotate_quant beside the GEMM: its algorithmic bytes and flops against the same
    peaks.  With one token it is a single workgroup and latency bound; it is reported so that
    the share of the layer time it takes is visible."""
    t = us_rotate * 1e-6
    flops = 2 * cfg.M * cfg.K * (cfg.n1 + cfg.n2) + 2 * cfg.M * cfg.K * cfg.r
    return {"kernel": "bwla_rotate_quant", "us_per_launch": us_rotate,
            "bytes_per_launch": rotate_quant_bytes(cfg), "gbps": rotate_quant_bytes(cfg) / t / 1e9,
            "flops_per_launch": flops, "tflops": flops / t / 1e12}


def quantizer_report(torch, rounds=2, svd_iters=20):
    """The offline quantizer (paper App. A.1 Algorithm 2) on a synthetic Gaussian matrix of the default
    workload's shape: time per round of {EM, PSP, two Procrustes updates}, the loss after every
    sub-step, and how the OKT transform of all rows (three fp64 GEMMs and the centering, each a pass
    over the n x m array) sits against HBM."""
    from paper_2605_00422_amd import quantizer_binding as qb
    n, n1, n2, k = 11008, 64, 64, 32
    m = n1 * n2
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    W = torch.randn(n, m, device="cuda", dtype=torch.float32, generator=g) * 0.02
    ws = torch.zeros(qb.workspace_size(n, m, n1, n2, k), dtype=torch.uint8, device="cuda")
    f32 = lambda *s: torch.empty(*s, dtype=torch.float32, device="cuda")
    f64 = lambda *s: torch.empty(*s, dtype=torch.float64, device="cuda")
    R1, R2, Wrot, U, V, c, s2 = f32(n1, n1), f32(n2, n2), f32(n, m), f32(m, k), f32(n, k), f64(n), f64(n)
    hist = f64(1 + 3 * rounds)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    ms = timed(lambda: qb.quantize_layer(W, n1, n2, k, rounds, R1, R2, Wrot, U, V, c, s2, hist, ws,
                                         svd_iters=svd_iters, svd_tol=0.0), 2)
    W64, X, A, Bt = W.double(), f64(n, m), torch.zeros(n, k, dtype=torch.float64, device="cuda"), \
        torch.zeros(m, k, dtype=torch.float64, device="cuda")
    r1, r2 = R1.double(), R2.double()
    ms_okt = timed(lambda: qb.okt_rows(W64, A, Bt, r1, r2, X, None, ws), 5)
    passes = 8 * n * m * 8            # W - M, two GEMM stages, centering: each reads and writes n x m fp64
    # the down projection of the same block (128 x 86 factors: the polar factors of the Procrustes
    # updates come from the Newton-Schulz iteration there, not from the Jacobi SVD)
    del W64, X, A, Bt, Wrot, U, V
    dn, d1, d2 = 4096, 128, 86
    dm = d1 * d2
    Wd = torch.randn(dn, dm, device="cuda", dtype=torch.float32, generator=g) * 0.02
    wsd = ws[:qb.workspace_size(dn, dm, d1, d2, k)] if qb.workspace_size(dn, dm, d1, d2, k) <= ws.numel() else \
        torch.zeros(qb.workspace_size(dn, dm, d1, d2, k), dtype=torch.uint8, device="cuda")
    dR1, dR2, dWrot, dU, dV, dc, ds2 = f32(d1, d1), f32(d2, d2), f32(dn, dm), f32(dm, k), f32(dn, k), f64(dn), f64(dn)
    dhist = f64(1 + 3 * rounds)
    ms_down = timed(lambda: qb.quantize_layer(Wd, d1, d2, k, rounds, dR1, dR2, dWrot, dU, dV, dc, ds2, dhist, wsd,
                                              svd_iters=svd_iters, svd_tol=0.0), 2)
    down = {"workload": f"Gaussian {dn} x {dm} (Kronecker {d1} x {d2}), rank {k}", "ms_per_round": ms_down / rounds,
            "loss_history": [float(v) for v in dhist.cpu()]}
    return {"workload": f"Gaussian {n} x {m} (Kronecker {n1} x {n2}), rank {k}", "dtype": "f64",
            "rounds": rounds, "svd_iters_per_round": svd_iters, "ms_total": ms, "ms_per_round": ms / rounds,
            "loss_history": [float(v) for v in hist.cpu()],
            "okt_rows": {"ms": ms_okt, "bound": "hbm", "bytes_moved": passes,
                         "achieved": passes / (ms_okt * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                         "frac": passes / (ms_okt * 1e-3) / 1e9 / 8000.0,
                         "flops": 2 * n * m * (n1 + n2 + k)},
            "down_projection": down}


def cpu_baseline(w, budget_s=12.0):
    """The CPU oracle (as it stands) on the same workload: online path only (the binarized
    matrix is prepared once, like the packed layer on the GPU)."""
    import numpy as np
    from oracle import bwla_oracle as orc
    cfg, d = w.cfg, w.data
    sgn, alpha = orc.binarize_rows(d.W)
    alpha16 = orc.to_fp16(alpha)
    rows_n = cfg.M if cfg.M <= 64 else 64
    rows = np.arange(rows_n)
    U = d.U if cfg.r > 0 else None
    V = d.V if cfg.r > 0 else None
    orc.forward_rows(d.X, d.R1, d.R2, sgn, alpha16, U, V, rows)       # warm-up
    n, t0 = 0, time.perf_counter()
    while True:
        orc.forward_rows(d.X, d.R1, d.R2, sgn, alpha16, U, V, rows)
        n += 1
        el = time.perf_counter() - t0
        if el > budget_s or n >= 200:
            break
    per_call = el / n
    us_layer = per_call * (cfg.M / rows_n) * 1e6
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    sample = (f"{n} repeats of the oracle's online path on {rows_n} of {cfg.M} token rows of {cfg.name}"
              + ("" if rows_n == cfg.M else f", scaled by {cfg.M}/{rows_n}"))
    return {"value": us_layer, "unit": "us/layer", "cores": int(cores), "kind": "oracle", "sample": sample,
            "host_cpus": os.cpu_count()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="cfg1_decode7b")
    ap.add_argument("--no-extra", action="store_true", help="skip the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the measured-ceiling launches")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device copies (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_00422_amd import binding as B
    from paper_2605_00422_amd import inputs as syn
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.load()          # raises if the HIP library has not been built: there is no fallback

    all_cfgs = dict(syn.CONFIGS)
    for M in (1, 64, 4096):
        for c in syn.block70b_configs(M):
            all_cfgs[c.name] = c
    for c in syn.block7b_configs(1):
        all_cfgs[c.name] = c
    cfg = all_cfgs[args.workload]

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    traffic = measured_traffic()
    peaks = None if args.no_peaks else Peaks(torch, B)
    w, res = measure(cfg, args.steps, args.warmup, not args.no_graph)
    best, mode = best_of(res)
    us_layer = best["us_per_layer"]
    us_fwd = best["us_linear_forward"]
    roof = roofline_for(cfg, w.launches, us_layer, us_fwd, peaks, traffic)
    line = {
        "metric": "us/layer, W1A6 linear forward (rotate+quant, binary GEMM + PSP + dequant)",
        "value": us_layer, "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": us_layer / 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8",
        "dtype_detail": "int8 codes x 1-bit weights -> int32 on INT8 MFMA; rotation on bf16/fp16-split MFMA with fp32 accumulation, fp32 epilogue",
        "data": "synthetic",
        "config": {"workload": cfg.name, "M": cfg.M, "K": cfg.K, "N": cfg.N, "r": cfg.r,
                   "kron": f"{cfg.n1}x{cfg.n2}", "x_dtype": cfg.x_dtype, "launch_mode": mode,
                   "launches_per_layer": w.launches, "layer_copies": res["layer_copies"],
                   "cache_flush_bytes": FLUSH_BYTES},
        "effective_tops": gemm_ops(cfg) / (us_layer * 1e-6) / 1e12,
        "hbm_gbps_layer": layer_bytes(cfg) / (us_layer * 1e-6) / 1e9,
        "us_two_calls": {"us_linear_forward": us_fwd, "us_rotate_quant": best["us_rotate_quant"]},
        "timings": {k: res[k] for k in ("stream", "graph") if k in res},
        "roofline": roof,
        "side_kernels": [side_kernel_report(cfg, best["us_rotate_quant"])],
    }
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(w)
    del w
    torch.cuda.empty_cache()

    if not args.no_extra:
        extra = []
        names = ["cfg1_7b_q_m1", "cfg1_7b_down_m1", "cfg1_7b_qkv_m1", "cfg1_7b_gateup_m1", "cfg2_qwen32b_up_m16",
                 "cfg3_qwen32b_down_m2048", "cfg4_70b_gate_m1", "cfg4_70b_down_m1", "cfg4_70b_q_m64",
                 "cfg4_70b_gate_m64", "cfg4_70b_down_m64", "cfg4_70b_q_m4096", "cfg4_70b_gate_m4096",
                 "cfg4_70b_down_m4096"]
        # (name, layer binarized with the row shift: the shift term rides as one more low-rank column)
        # and 8-bit activation codes, the width of the paper's speed run: same kernels, same bytes)
        # and per-token asymmetric codes with the row shift, the paper's own setting: three more columns)
        # and 4-bit codes (paper Table 3) at the prefill shape: one per byte, and two per byte)
        variants = [(n, False, 6, False, False) for n in names] + [("cfg1_decode7b", True, 6, False, False),
                                                                   ("cfg1_decode7b", False, 8, False, False),
                                                                   ("cfg1_decode7b", True, 6, True, False),
                                                                   ("cfg3_qwen32b_down_m2048", False, 4, False, False),
                                                                   ("cfg3_qwen32b_down_m2048", False, 4, False, True)]
        for nm, shift, bits, asym, nibble in variants:
            if nm == cfg.name and not shift and bits == 6 and not asym:
                continue
            c = all_cfgs[nm]
            st = max(10, min(args.steps, 200 if c.M <= 64 else (20 if c.M <= 2048 else 10)))
            ww, r = measure(c, st, max(3, min(args.warmup, st // 4)), not args.no_graph, centered=shift,
                            act_bits=bits, asym=asym, nibble=nibble)
            if nibble:
                r["code_bytes_per_launch"] = c.M * c.K // 2
            if shift or asym:
                c = dataclasses.replace(c, r=c.r + int(shift) + 2 * int(asym))   # bytes of the extra columns of V and T
            b, _ = best_of(r)
            r["roofline"] = roofline_for(c, ww.launches, b["us_per_layer"], b["us_linear_forward"], peaks, traffic,
                                         workload=r["workload"])
            if not nibble and bits == 4:
                r["code_bytes_per_launch"] = c.M * c.K
            r["side_kernels"] = [side_kernel_report(c, b["us_rotate_quant"])]
            r["effective_tops"] = gemm_ops(c) / (b["us_per_layer"] * 1e-6) / 1e12
            extra.append(r)
            del ww
            torch.cuda.empty_cache()
        line["other_workloads"] = extra
        # the prefill shape's roofline (INT8 MFMA bound) beside the headline's (HBM bound)
        pre = [e for e in extra if e["workload"] == "cfg3_qwen32b_down_m2048"]
        if pre:
            line["roofline_prefill"] = dict(pre[0]["roofline"], workload=pre[0]["workload"])
        # the seven linear layers of a 7B decoder block at one token: called one by one (q, k, v, o,
        # gate, up, down), and with the projections that read the same activations packed as one
        # layer (qkv, o, gate|up, down)
        us = {e["workload"]: best_of(e)[0]["us_per_layer"] for e in extra}
        us[cfg.name] = us_layer
        need = ("cfg1_7b_q_m1", "cfg1_decode7b", "cfg1_7b_down_m1", "cfg1_7b_qkv_m1", "cfg1_7b_gateup_m1")
        if all(k in us for k in need):
            line["block7b_m1"] = {
                "us_seven_layers": 4 * us["cfg1_7b_q_m1"] + 2 * us["cfg1_decode7b"] + us["cfg1_7b_down_m1"],
                "us_four_merged_layers": us["cfg1_7b_qkv_m1"] + us["cfg1_7b_q_m1"] + us["cfg1_7b_gateup_m1"]
                                         + us["cfg1_7b_down_m1"]}
            gu = [e for e in extra if e["workload"] == "cfg1_7b_gateup_m1"]
            if gu and "us_linear_forward_gated" in gu[0].get("graph", {}):
                # bwla_linear_forward_swiglu in place of bwla_linear_forward for gate|up: h leaves the
                # GEMM as bf16, ready for the down projection's rotation
                line["block7b_m1"]["us_gateup_forward"] = gu[0]["graph"]["us_linear_forward"]
                line["block7b_m1"]["us_gateup_forward_gated"] = gu[0]["graph"]["us_linear_forward_gated"]
        line["quantizer"] = quantizer_report(torch)
    if peaks is not None:
        line["microbench"] = microbench(torch, B)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
