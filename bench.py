#!/usr/bin/env python3
"""Benchmark of the Walsh-Hadamard output layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-extras]

One "step" is one pass of the whole hot path over one batch: wht_affine_forward followed by
wht_affine_backward (forward only for forward-only workloads), inputs resident in HBM.  The last
line printed is one JSON object: whole-job tokens/s, the HBM-roofline figure of the dominant kernel
(measured here with events on the launch stream), and the CPU oracle timed on this host's cores on
a bounded sample of the same workload.  Extra keys carry the other workloads, the plain-copy
ceiling and the same-shape dense W_O GEMM.
"""
import argparse
import ctypes
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=150,
                    help="untimed steps first; after idling the GPU's shader clock dips for ~40 steps of this load")
    ap.add_argument("--workload", default="C5_large")
    ap.add_argument("--no-extras", action="store_true", help="headline workload only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--schedule", choices=["default", "butterfly"], default="default",
                    help="butterfly: force the butterfly schedule for bf16, d >= 1024 (WHT_AFFINE_SCHEDULE)")
    args = ap.parse_args()
    if args.schedule == "butterfly":
        os.environ["WHT_AFFINE_SCHEDULE"] = "butterfly"       # read by the library when it is loaded
    return args


def io_bytes(dtype):
    return 2 if dtype == "bf16" else 4


def algorithmic_bytes(N, d, dtype, which):
    """HBM bytes the method itself must move per launch: forward reads x and writes y (+ alpha,
    beta); backward reads x, dy, writes dx (+ alpha read, dalpha/dbeta written)."""
    s = io_bytes(dtype)
    if which == "fwd":
        return 2 * N * d * s + 8 * d
    return 3 * N * d * s + 12 * d


class Bench:
    def __init__(self, torch, wht, synth, name, sets=None):
        import numpy as np
        self.torch, self.wht = torch, wht
        w = synth.WORKLOADS[name]
        self.w = w
        tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        per_set = (4 if w.backward else 2) * w.N * w.d * io_bytes(w.dtype)
        # rotate buffer sets so that consecutive steps cannot be served by the 256 MB Infinity Cache;
        # at least three, because the kernels' time also depends (by a few per cent) on the address
        # distances between the tensors, which differ from set to set
        self.sets = sets if sets is not None else max(3, min(8, -(-(1 << 30) // per_set)))
        g = torch.Generator(device="cuda").manual_seed(0)
        rng = np.random.Generator(np.random.PCG64(0))
        self.alpha = torch.from_numpy(rng.uniform(0.5, 1.5, w.d).astype(np.float32)).cuda()
        self.beta = torch.from_numpy((0.02 * rng.standard_normal(w.d)).astype(np.float32)).cuda()
        self.x, self.dy, self.y, self.dx = [], [], [], []
        for _ in range(self.sets):
            x = torch.randn(w.N, w.d, device="cuda", dtype=torch.float32, generator=g)
            if w.outliers:
                mask = torch.rand(w.N, w.d, device="cuda", generator=g) < 0.01
                x = torch.where(mask, x * 20.0, x)
            self.x.append(x.to(tdt))
            self.y.append(torch.empty(w.N, w.d, device="cuda", dtype=tdt))
            if w.backward:
                self.dy.append(torch.randn(w.N, w.d, device="cuda", dtype=torch.float32, generator=g).to(tdt))
                self.dx.append(torch.empty(w.N, w.d, device="cuda", dtype=tdt))
            del x
        self.dalpha = torch.empty(w.d, device="cuda")
        self.dbeta = torch.empty(w.d, device="cuda")
        code = wht.DTYPE_BF16 if w.dtype == "bf16" else wht.DTYPE_F32
        need = wht.wht_affine_backward_workspace_bytes(w.N, w.d, code) if w.backward else 0
        self.ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

    def fwd(self, i):
        k = i % self.sets
        self.wht.wht_affine_forward(self.x[k], self.alpha, self.beta, y=self.y[k])

    def bwd(self, i):
        k = i % self.sets
        self.wht.wht_affine_backward(self.dy[k], self.x[k], self.alpha, dx=self.dx[k], dalpha=self.dalpha,
                                     dbeta=self.dbeta, workspace=self.ws)

    def run(self, steps, warmup):
        """Times `steps` whole steps (wall clock between synchronisations) and, inside the same
        region, every forward and backward call with events on the launch stream (StreamEvent: an
        event record is itself a few microseconds of stream time, which the step time includes)."""
        torch = self.torch
        for i in range(warmup):
            self.fwd(i)
            if self.w.backward:
                self.bwd(i)
        ev = [[StreamEvent(torch) for _ in range(3)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            ev[i][0].record()
            self.fwd(i)
            ev[i][1].record()
            if self.w.backward:
                self.bwd(i)
                ev[i][2].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        fwd_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
        bwd_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / steps if self.w.backward else None
        return (t1 - t0) * 1e3 / steps, fwd_ms, bwd_ms

    def series(self, calls=50, warmup=5):
        """Per-call time of each entry point called back to back, `calls` times between one pair of
        events: no event between the launches, so this is what a caller that does not time single
        launches sees.  Returns (fwd_ms, bwd_ms or None)."""
        torch = self.torch
        out = []
        for fn in (self.fwd, self.bwd if self.w.backward else None):
            if fn is None:
                out.append(None)
                continue
            for i in range(warmup):
                fn(i)
            a, b = StreamEvent(torch), StreamEvent(torch)
            torch.cuda.synchronize()
            a.record()
            for i in range(calls):
                fn(i)
            b.record()
            torch.cuda.synchronize()
            out.append(a.elapsed_time(b) / calls)
        return tuple(out)


def paper_protocol(bench, runs=3, iters=50, warmup=10):
    """The paper's timing protocol (Sec. 5, captions of Tables 4 and 5: mean and standard deviation
    over 3 runs of 50 iterations each), after 10 untimed steps: per entry point the mean of the
    three per-run averages and their standard deviation, from events on the launch stream."""
    torch, w = bench.torch, bench.w
    for i in range(warmup):
        bench.fwd(i)
        if w.backward:
            bench.bwd(i)
    per_run = {"fwd": [], "bwd": [], "step": []}
    for _ in range(runs):
        ev = [[StreamEvent(torch) for _ in range(3)] for _ in range(iters)]
        torch.cuda.synchronize()
        for i in range(iters):
            ev[i][0].record()
            bench.fwd(i)
            ev[i][1].record()
            if w.backward:
                bench.bwd(i)
            ev[i][2].record()
        torch.cuda.synchronize()
        per_run["fwd"].append(sum(e[0].elapsed_time(e[1]) for e in ev) / iters)
        per_run["bwd"].append(sum(e[1].elapsed_time(e[2]) for e in ev) / iters)
        per_run["step"].append(ev[0][0].elapsed_time(ev[-1][2]) / iters)
    out = {"workload": w.name, "warmup": warmup, "runs": runs, "iterations_per_run": iters}
    for key, which in (("fwd", "fwd"), ("bwd", "bwd")):
        if key == "bwd" and not w.backward:
            continue
        mean = statistics.mean(per_run[key])
        out[key + "_ms_mean"] = mean
        out[key + "_ms_std"] = statistics.stdev(per_run[key])
        out[key + "_frac_hbm_peak"] = algorithmic_bytes(w.N, w.d, w.dtype, which) / (mean * 1e-3) / 1e9 / HBM_PEAK_GBS
    out["step_ms_mean"] = statistics.mean(per_run["step"])
    out["step_ms_std"] = statistics.stdev(per_run["step"])
    out["tokens_per_s"] = w.N / (out["step_ms_mean"] * 1e-3)
    return out


def add_series(row, w, fwd_ms, bwd_ms):
    """Back-to-back per-call times (Bench.series) into a workload's summary row."""
    row["fwd_ms_back_to_back"] = round(fwd_ms, 5)
    row["fwd_frac_hbm_peak_back_to_back"] = algorithmic_bytes(w.N, w.d, w.dtype, "fwd") / (fwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS
    if bwd_ms is not None:
        row["bwd_ms_back_to_back"] = round(bwd_ms, 5)
        row["bwd_frac_hbm_peak_back_to_back"] = algorithmic_bytes(w.N, w.d, w.dtype, "bwd") / (bwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS


def event_cost(torch, n=200):
    """Microseconds between two consecutive event records with nothing between them: what one
    record costs on the stream, for the events this benchmark uses and for torch.cuda.Event."""
    out = {}
    for key, make in (("stream_event_us", lambda: StreamEvent(torch)),
                      ("torch_event_us", lambda: torch.cuda.Event(enable_timing=True))):
        ev = [make() for _ in range(n)]
        torch.cuda.synchronize()
        for e in ev:
            e.record()
        torch.cuda.synchronize()
        gaps = [ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(n // 4, n - 1)]
        out[key] = sum(gaps) / len(gaps)
    return out


def summarize(w, step_ms, fwd_ms, bwd_ms):
    out = {
        "workload": w.name, "N": w.N, "d": w.d, "io_dtype": w.dtype,
        "ms_per_step": round(step_ms, 5),
        "tokens_per_s": w.N / (step_ms * 1e-3),
        "fwd_ms": round(fwd_ms, 5),
        "fwd_tokens_per_s": w.N / (fwd_ms * 1e-3),
        "fwd_GBs": algorithmic_bytes(w.N, w.d, w.dtype, "fwd") / (fwd_ms * 1e-3) / 1e9,
    }
    out["fwd_frac_hbm_peak"] = out["fwd_GBs"] / HBM_PEAK_GBS
    if bwd_ms is not None:
        out["bwd_ms"] = round(bwd_ms, 5)
        out["bwd_GBs"] = algorithmic_bytes(w.N, w.d, w.dtype, "bwd") / (bwd_ms * 1e-3) / 1e9
        out["bwd_frac_hbm_peak"] = out["bwd_GBs"] / HBM_PEAK_GBS
    return out


_copy_lib = None


def _bench_lib():
    global _copy_lib
    if _copy_lib is None:
        from paper_2603_08343_amd.build import COPY_LIB
        _copy_lib = ctypes.CDLL(COPY_LIB)
        _copy_lib.wht_bench_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        _copy_lib.wht_bench_copy.restype = ctypes.c_int
        _copy_lib.wht_bench_empty.argtypes = [ctypes.c_void_p]
        _copy_lib.wht_bench_empty.restype = ctypes.c_int
        _copy_lib.wht_bench_clock_probe.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        _copy_lib.wht_bench_clock_probe.restype = ctypes.c_int
        _copy_lib.wht_bench_event_create.argtypes = []
        _copy_lib.wht_bench_event_create.restype = ctypes.c_void_p
        _copy_lib.wht_bench_event_record.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        _copy_lib.wht_bench_event_record.restype = ctypes.c_int
        _copy_lib.wht_bench_event_elapsed_ms.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        _copy_lib.wht_bench_event_elapsed_ms.restype = ctypes.c_float
        _copy_lib.wht_bench_event_destroy.argtypes = [ctypes.c_void_p]
        _copy_lib.wht_bench_event_destroy.restype = ctypes.c_int
    return _copy_lib


class StreamEvent:
    """HIP timing event without the system-scope fence (libwht_copybench.so), recorded on torch's
    current stream.  torch.cuda.Event creates events with the default flags, whose record costs
    4.5 us of stream time; this one costs 3.3 us and reads a kernel 0.9 us long instead of 2.8 us."""

    def __init__(self, torch):
        self._torch = torch
        self._h = _bench_lib().wht_bench_event_create()
        if not self._h:
            raise RuntimeError("wht_bench_event_create failed")

    def record(self):
        if _bench_lib().wht_bench_event_record(self._h, self._torch.cuda.current_stream().cuda_stream) != 0:
            raise RuntimeError("wht_bench_event_record failed")

    def elapsed_time(self, other) -> float:
        ms = _bench_lib().wht_bench_event_elapsed_ms(self._h, other._h)
        if ms < 0:
            raise RuntimeError("wht_bench_event_elapsed_ms failed")
        return ms

    def __del__(self):
        try:
            _bench_lib().wht_bench_event_destroy(self._h)
        except Exception:
            pass


def bench_empty(torch):
    """One launch of an empty kernel on torch's current stream (the launch path's per-call floor)."""
    if _bench_lib().wht_bench_empty(torch.cuda.current_stream().cuda_stream) != 0:
        raise RuntimeError("wht_bench_empty failed")


def bench_clock_probe(torch, out):
    """Enqueue a short probe kernel that writes (shader-clock ticks, 100 MHz ticks) of a fixed spin
    into out[0:2] (int64 GPU tensor): the shader clock at that point of the stream."""
    if _bench_lib().wht_bench_clock_probe(out.data_ptr(), torch.cuda.current_stream().cuda_stream) != 0:
        raise RuntimeError("wht_bench_clock_probe failed")


def bench_copy(torch, src, dst):
    """dst <- src with the bench-only streaming copy kernel (libwht_copybench.so: 16 bytes per lane,
    non-temporal both ways; not part of the layer's library)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    rc = _bench_lib().wht_bench_copy(src.data_ptr(), dst.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"wht_bench_copy: status {rc}")


def copy_ceiling(torch, nbytes=1 << 30, iters=20):
    src = [torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(2)]
    dst = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    for i in range(3):
        bench_copy(torch, src[i % 2], dst[i % 2])
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for i in range(iters):
        bench_copy(torch, src[i % 2], dst[i % 2])
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / iters
    return {"bytes_moved": 2 * nbytes, "ms": ms, "GBs": 2 * nbytes / (ms * 1e-3) / 1e9}


def dense_wo(torch, w, iters=10):
    """Same-shape dense output projection on the same GPU (hipBLASLt through torch.matmul):
    forward y = x W^T + b; backward dx = dy W, dW = dy^T x, db = sum dy."""
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    x = torch.randn(w.N, w.d, device="cuda", dtype=tdt)
    W = torch.randn(w.d, w.d, device="cuda", dtype=tdt) / (w.d ** 0.5)
    b = torch.zeros(w.d, device="cuda", dtype=tdt)
    dy = torch.randn(w.N, w.d, device="cuda", dtype=tdt) if w.backward else None

    def fwd():
        return torch.addmm(b, x, W.t())

    def bwd():
        return dy @ W, dy.t() @ x, dy.sum(dim=0)

    def timeit(fn):
        for _ in range(2):
            fn()
        a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(iters):
            fn()
        e.record()
        torch.cuda.synchronize()
        return a.elapsed_time(e) / iters

    out = {"fwd_ms": timeit(fwd), "fwd_flops": 2.0 * w.N * w.d * w.d}
    out["fwd_TFLOPs"] = out["fwd_flops"] / (out["fwd_ms"] * 1e-3) / 1e12
    if w.backward:
        out["bwd_ms"] = timeit(bwd)
        out["fwd_bwd_ms"] = out["fwd_ms"] + out["bwd_ms"]
    return out


def cpu_baseline(synth, w, target_seconds):
    """The CPU oracle as it stands (butterfly path, OpenMP over tokens), on a bounded sample of the
    same workload: the first n tokens of the seeded recipe, passes repeated until about
    `target_seconds` of oracle time has been spent; the mean pass time is reported."""
    import oracle

    n = min(w.N, 4096)
    inp = synth.make_inputs(n, w.d, w.dtype, seed=0, backward=w.backward, outliers=w.outliers)

    def one():
        t0 = time.perf_counter()
        oracle.forward(inp.x, inp.alpha, inp.beta, "fast")
        if w.backward:
            oracle.backward(inp.dy, inp.x, inp.alpha, "fast")
        return time.perf_counter() - t0

    one()                                                 # first call loads the library
    spent, passes = 0.0, 0
    while spent < target_seconds and passes < 1000:
        spent += one()
        passes += 1
    secs = spent / passes
    cores = oracle.num_threads()
    # the same sample on one core, for about a fifth of the time
    single = None
    try:
        oracle.set_num_threads(1)
        spent1, passes1 = 0.0, 0
        while spent1 < target_seconds / 5 and passes1 < 50:
            spent1 += one()
            passes1 += 1
        single = n / (spent1 / passes1)
    finally:
        oracle.set_num_threads(cores)
    return {"value": n / secs, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "single_core_value": single,
            "sample": f"first {n} of {w.N} tokens of {w.name} (d={w.d}, {w.dtype} inputs, "
                      f"{'forward+backward' if w.backward else 'forward'}), fp64 butterfly oracle, "
                      f"mean of {passes} passes, {spent:.1f} s of CPU time in total"}


def decode_latency(torch, wht, synth, iters=1000):
    """Per-call time of the decode shapes (one new token per sequence, d = 4096), two ways:
    back-to-back calls through the Python binding (launch path included), and the same calls
    captured once into a HIP graph and replayed (GPU-side time per call, no host launch path);
    next to them the same-shape dense GEMV/GEMM."""
    rows = []
    for name in ("C4_decode_n1", "C4_decode_n16", "C4_decode_n64", "C4_decode_n256"):
        w = synth.WORKLOADS[name]
        b = Bench(torch, wht, synth, name, sets=1)
        for i in range(20):
            b.fwd(i)
        a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for i in range(iters):
            b.fwd(i)
        e.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(e) * 1e3 / iters
        dense = dense_wo(torch, w, iters=200)
        row = {"N": w.N, "d": w.d, "wht_affine_us_per_call": us, "dense_wo_us_per_call": dense["fwd_ms"] * 1e3,
               "wht_affine_us_per_call_graph": None, "dense_wo_us_per_call_graph": None,
               "wht_affine_residual_stats_us_per_call_graph": None,
               "empty_kernel_us_per_call_graph": None, "copy_same_bytes_us_per_call_graph": None}
        try:
            per_graph = 50
            xd = torch.randn(w.N, w.d, device="cuda", dtype=torch.bfloat16)
            Wd = torch.randn(w.d, w.d, device="cuda", dtype=torch.bfloat16) / (w.d ** 0.5)
            bd = torch.zeros(w.d, device="cuda", dtype=torch.bfloat16)
            yd = torch.empty_like(xd)
            rd = torch.randn(w.N, w.d, device="cuda", dtype=torch.bfloat16)
            ss = torch.empty(w.N, device="cuda", dtype=torch.float32)
            for key, fn in (("wht_affine_us_per_call_graph", lambda: b.fwd(0)),
                            # the layer as the attention block calls it when decoding: residual add fused,
                            # in place on the residual stream, with the following RMS norm's statistic
                            ("wht_affine_residual_stats_us_per_call_graph",
                             lambda: wht.wht_affine_forward_residual_stats(b.x[0], b.alpha, b.beta, rd, y=rd, sumsq=ss)),
                            ("dense_wo_us_per_call_graph", lambda: torch.addmm(bd, xd, Wd.t())),
                            # floors of a call on this GPU: a kernel that does nothing, and a plain copy
                            # of the same x -> y bytes (one memory round trip, no arithmetic)
                            ("empty_kernel_us_per_call_graph", lambda: bench_empty(torch)),
                            ("copy_same_bytes_us_per_call_graph", lambda: bench_copy(torch, xd, yd))):
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    for _ in range(3):
                        fn()
                torch.cuda.current_stream().wait_stream(side)
                torch.cuda.synchronize()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    for _ in range(per_graph):
                        fn()
                for _ in range(3):
                    graph.replay()
                torch.cuda.synchronize()
                a.record()
                for _ in range(20):
                    graph.replay()
                e.record()
                torch.cuda.synchronize()
                row[key] = a.elapsed_time(e) * 1e3 / (20 * per_graph)
        except Exception as exc:                      # graph capture is a measurement nicety only
            row["graph_note"] = f"graph replay not measured: {type(exc).__name__}: {exc}"[:200]
        rows.append(row)
    return rows


def graph_replay_step(torch, b, steps):
    """The same forward+backward step captured once into a HIP graph (one step per rotating buffer
    set) and replayed: the step without the host launch path and with the inter-kernel gaps the
    graph executor leaves.  The entry points allocate and synchronise nothing, so they capture as
    they are."""
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(b.sets):
                b.fwd(i)
                if b.w.backward:
                    b.bwd(i)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(b.sets):
                b.fwd(i)
                if b.w.backward:
                    b.bwd(i)
        replays = max(1, -(-steps // b.sets))
        for _ in range(max(1, 150 // b.sets)):
            graph.replay()
        a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(replays):
            graph.replay()
        e.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(e) / (replays * b.sets)
        return {"ms_per_step": ms, "tokens_per_s": b.w.N / (ms * 1e-3), "steps_per_graph": b.sets,
                "replays": replays}
    except Exception as exc:                          # a measurement nicety only
        return {"note": f"graph replay not measured: {type(exc).__name__}: {exc}"[:200]}


def attention_block_context(torch, wht, iters=20):
    """The layer where the paper uses it: one attention block (QKV projection, causal attention, output
    layer, residual add) at the paper's four model widths (Table 2) and its two inference shapes
    (prefill: batch 1024 x 64 tokens; decode: batch 2048, one new token against a 128-token cache),
    forward, bf16, random weights.  Everything but the output layer is stock torch (hipBLASLt GEMM,
    scaled_dot_product_attention) and identical in both variants; the output layer is either the
    dense W_O (addmm with the residual as its additive input) or wht_affine_forward_residual."""
    import torch.nn.functional as F
    rows = []
    g = torch.Generator(device="cuda").manual_seed(0)
    for size, d, heads in (("Tiny", 768, 12), ("Small", 1024, 16), ("Base", 1536, 16), ("Large", 2048, 16)):
        dh = d // heads
        wqkv = (torch.randn(3 * d, d, device="cuda", generator=g) / d ** 0.5).to(torch.bfloat16)
        wo = (torch.randn(d, d, device="cuda", generator=g) / d ** 0.5).to(torch.bfloat16)
        alpha = torch.rand(d, device="cuda", generator=g) + 0.5
        beta = 0.02 * torch.randn(d, device="cuda", generator=g)
        for phase, B, T, L in (("prefill", 1024, 64, 64), ("decode", 2048, 1, 128)):
            x = torch.randn(B, T, d, device="cuda", generator=g).to(torch.bfloat16)
            kc = torch.randn(B, heads, L, dh, device="cuda", generator=g).to(torch.bfloat16)
            vc = torch.randn(B, heads, L, dh, device="cuda", generator=g).to(torch.bfloat16)
            resid = x.view(B * T, d)
            out = torch.empty(B * T, d, device="cuda", dtype=torch.bfloat16)

            def heads_out():
                qkv = F.linear(x, wqkv).view(B, T, 3, heads, dh)
                q = qkv[:, :, 0].transpose(1, 2)
                if phase == "prefill":
                    k, v = qkv[:, :, 1].transpose(1, 2), qkv[:, :, 2].transpose(1, 2)
                    o = F.scaled_dot_product_attention(q, k, v, is_causal=True)
                else:
                    o = F.scaled_dot_product_attention(q, kc, vc)
                return o.transpose(1, 2).reshape(B * T, d)

            def dense_block():
                return torch.addmm(resid, heads_out(), wo.t())

            def wht_block():
                return wht.wht_affine_forward_residual(heads_out(), alpha, beta, resid, y=out)

            ho = heads_out()

            def timeit(fn):
                for _ in range(5):
                    fn()
                a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                a.record()
                for _ in range(iters):
                    fn()
                e.record()
                torch.cuda.synchronize()
                return a.elapsed_time(e) / iters

            row = {"size": size, "d_model": d, "heads": heads, "phase": phase, "tokens": B * T,
                   "block_dense_ms": timeit(dense_block), "block_wht_ms": timeit(wht_block),
                   "output_layer_dense_ms": timeit(lambda: torch.addmm(resid, ho, wo.t())),
                   "output_layer_wht_ms": timeit(lambda: wht.wht_affine_forward_residual(ho, alpha, beta, resid, y=out))}
            row["block_speedup"] = row["block_dense_ms"] / row["block_wht_ms"]
            row["output_layer_speedup"] = row["output_layer_dense_ms"] / row["output_layer_wht_ms"]
            rows.append(row)
            del x, kc, vc, out, ho
        del wqkv, wo
        torch.cuda.empty_cache()
    return rows


def fused_residual(torch, wht, synth, name, steps=100, warmup=100):
    """y = resid + alpha (.) Hx + beta in one kernel (3 N d s bytes) against the unfused pair:
    the layer's forward followed by torch's in-place add on the residual stream (5 N d s bytes);
    and the same kernel also delivering sum_j y^2 per token (the following RMS norm's statistic)."""
    w = synth.WORKLOADS[name]
    b = Bench(torch, wht, synth, name)
    tdt = b.x[0].dtype
    resid = [torch.randn(w.N, w.d, device="cuda").to(tdt) for _ in range(b.sets)]

    def fused(i):
        k = i % b.sets
        wht.wht_affine_forward_residual(b.x[k], b.alpha, b.beta, resid[k], y=b.y[k])

    def unfused(i):
        k = i % b.sets
        wht.wht_affine_forward(b.x[k], b.alpha, b.beta, y=b.y[k])
        resid[k].add_(b.y[k])

    sumsq = torch.empty(w.N, dtype=torch.float32, device="cuda")

    def fused_stats(i):
        k = i % b.sets
        wht.wht_affine_forward_residual_stats(b.x[k], b.alpha, b.beta, resid[k], y=b.y[k], sumsq=sumsq)

    out = {"workload": name}
    for key, fn in (("fused", fused), ("fused_stats", fused_stats), ("unfused", unfused)):
        for i in range(warmup):
            fn(i)
        a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for i in range(steps):
            fn(i)
        e.record()
        torch.cuda.synchronize()
        out[key + "_ms"] = a.elapsed_time(e) / steps
    bytes_fused = 3 * w.N * w.d * io_bytes(w.dtype)
    out["fused_GBs"] = bytes_fused / (out["fused_ms"] * 1e-3) / 1e9
    out["fused_frac_hbm_peak"] = out["fused_GBs"] / HBM_PEAK_GBS
    return out


def recorded_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` as measured with rocprofv3 counters
    (FETCH_SIZE + WRITE_SIZE, calibrated on the copy kernel) and recorded in the committed summary
    under profiles/; None when no such record exists."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(path):
            if "TRAFFIC_JSON" in line:
                rec = json.loads(line.split("TRAFFIC_JSON", 1)[1])
                if rec.get("workload") == workload and rec.get("kernel") == kernel:
                    return rec["traffic_bytes_per_launch"]
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (tokens are independent, so "
              "the layer shards by splitting N; only dalpha/dbeta would need an all-reduce). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2603_08343_amd as wht
    from paper_2603_08343_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    from paper_2603_08343_amd.build import ensure_built
    ensure_built()                                        # compiles only if nothing is built yet
    wht.library()                                         # fail loudly if the HIP library is missing
    w = synth.WORKLOADS[args.workload]

    bench = Bench(torch, wht, synth, args.workload)
    step_ms, fwd_ms, bwd_ms = bench.run(args.steps, args.warmup)
    head = summarize(w, step_ms, fwd_ms, bwd_ms)
    sets = bench.sets
    # the paper's protocol on the same buffers, after the headline so that it cannot warm it up
    protocol = None if args.no_extras else [paper_protocol(bench)]
    graph_step = None if args.no_extras else graph_replay_step(torch, bench, args.steps)
    if not args.no_extras:
        add_series(head, w, *bench.series())
    del bench
    torch.cuda.empty_cache()

    # roofline of the dominant kernel: backward where the workload has one
    dom = "bwd" if w.backward else "fwd"
    dom_ms = bwd_ms if w.backward else fwd_ms
    dom_bytes = algorithmic_bytes(w.N, w.d, w.dtype, dom)
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    dom_kernel = ("backward_teams_kernel" if w.d in (3072, 4096, 6144, 8192) and w.dtype == "bf16" else "backward_kernel") \
        if w.backward else "forward_kernel"
    roofline = {"bound": "hbm",
                "kernel": dom_kernel + (" (+ reduce_partials_kernel: the interval timed is the whole "
                                        "wht_affine_backward call)" if w.backward else ""),
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": recorded_traffic(w.name, dom_kernel),
                "traffic_source": "recorded, not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                  "summary committed under profiles/ (TRAFFIC_JSON line); null if none",
                "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": dom_ms,
                "timing": "mean interval between events (no system-scope fence) recorded on the launch stream "
                          "right before and right after each call, over the timed steps; such an interval reads "
                          "about 1 us more than the kernels in it take"}

    result = {
        "metric": "wht_affine_fwd_bwd_tokens_per_s" if w.backward else "wht_affine_fwd_tokens_per_s",
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        # what the path computes in: float32 vector arithmetic and float32 accumulation; on the
        # matrix-core schedule (bf16 I/O, d >= 1024) a float32 value enters a +-1 matrix round as two
        # bfloat16 terms hi + lo (relative error <= 2^-17), the round's products being exact
        "dtype": "f32 (matrix-core rounds on bf16 hi+lo pairs, f32 accumulate)" if w.dtype == "bf16" and w.d >= 768
                 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: N={w.N} tokens, d={w.d}, {w.dtype} I/O, "
                               f"{'forward+backward' if w.backward else 'forward'}",
                   "io_dtype": w.dtype, "buffer_sets_rotated": sets},
        "roofline": roofline,
        "headline": head,
    }

    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(synth, w, args.cpu_seconds)
    else:
        result["cpu_baseline"] = None

    if not args.no_extras:
        extras = {}
        extras["copy_ceiling"] = copy_ceiling(torch)
        extras["event_record_cost"] = event_cost(torch)
        others = [n for n in ("C4b_roofline", "C5_large", "C2_train", "C3_prefill",
                              "W_tiny_768", "W_base_1536", "W_wide_6144") if n != args.workload]
        extras["workloads"] = []
        for name in others:
            b = Bench(torch, wht, synth, name)
            s, f, bw = b.run(max(10, args.steps // 2), 5)
            extras["workloads"].append(summarize(synth.WORKLOADS[name], s, f, bw))
            add_series(extras["workloads"][-1], synth.WORKLOADS[name], *b.series())
            del b
            torch.cuda.empty_cache()
        if args.workload != "C4b_roofline":
            b = Bench(torch, wht, synth, "C4b_roofline")
            protocol.append(paper_protocol(b))
            del b
            torch.cuda.empty_cache()
        extras["paper_protocol_3x50"] = protocol
        ceil = extras["copy_ceiling"]["GBs"]
        for row in [head] + extras["workloads"]:
            row["fwd_frac_copy_ceiling"] = row["fwd_GBs"] / ceil
            if "bwd_GBs" in row:
                row["bwd_frac_copy_ceiling"] = row["bwd_GBs"] / ceil
        extras["fused_residual_forward"] = [fused_residual(torch, wht, synth, n) for n in ("C5_large", "C4b_roofline")]
        extras["headline_step_graph_replay"] = graph_step
        try:
            extras["attention_block_context"] = attention_block_context(torch, wht)
        except Exception as exc:                      # stock-torch harness around the layer: optional
            extras["attention_block_context"] = {"note": f"not measured: {type(exc).__name__}: {exc}"[:200]}
        extras["decode"] = decode_latency(torch, wht, synth)
        extras["dense_wo_same_shape"] = dense_wo(torch, w)
        extras["dense_wo_same_shape"]["workload"] = w.name
        result["extras"] = extras

    print(json.dumps(result))


if __name__ == "__main__":
    main()
