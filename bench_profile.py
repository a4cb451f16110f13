"""Helpers around rocprofv3 for the Walsh-Hadamard output layer's kernels.

Three sub-commands:

  drive      launch a short, fixed sequence on one workload -- the plain copy kernel on a buffer of
             known size (the calibration reference for the HBM byte counters), then forward and
             backward a few times -- so that a counter pass (rocprofv3 --pmc ...) stays short:
                 rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT -o fetch -- \
                     python3 bench_profile.py drive --workload C5_large
  summarize  turn the CSV files of a kernel-trace run and of counter passes into the short text
             summary kept under profiles/ (per-kernel average duration; HBM bytes per launch scaled
             by what the same counter reads for the copy kernel; VALU / MFMA / LDS activity):
                 python3 bench_profile.py summarize --workload C5_large \
                     --kernel-stats OUT/kt/kt_kernel_stats.csv --kernel-trace OUT/kt/kt_kernel_trace.csv \
                     --pmc OUT/*/*_counter_collection.csv

  series     the first steps of forward + backward after the GPU has idled, each step timed with
             events and followed by a probe of the shader clock: shows the clock transient that a
             short benchmark run sits in
                 python3 bench_profile.py series --workload C5_large --steps 80
             with --copy the steps are plain copies of 512 MiB (the bench-only copy kernel) instead:
             the transient without the layer's arithmetic

Nothing here is on the product path (the file sits beside bench.py, outside the package).
"""
import argparse
import collections
import csv
import glob
import json
import sys

COPY_BYTES = 1 << 30          # the copy kernel reads 1 GiB and writes 1 GiB
NUM_SIMD = 256 * 4            # MI355X: 256 CUs x 4 SIMDs
NUM_XCD = 8                   # GRBM_GUI_ACTIVE comes back summed over the 8 XCDs


def drive(args):
    import os
    if args.schedule == "butterfly":
        os.environ["WHT_AFFINE_SCHEDULE"] = "butterfly"       # read by the library when it is loaded
    import numpy as np
    import torch
    import bench
    import paper_2603_08343_amd as wht
    from paper_2603_08343_amd import synth

    w = synth.WORKLOADS[args.workload]
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    g = torch.Generator(device="cuda").manual_seed(0)
    x = torch.randn(w.N, w.d, device="cuda", generator=g).to(tdt)
    dy = torch.randn(w.N, w.d, device="cuda", generator=g).to(tdt)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    rng = np.random.Generator(np.random.PCG64(0))
    alpha = torch.from_numpy(rng.uniform(0.5, 1.5, w.d).astype(np.float32)).cuda()
    beta = torch.from_numpy((0.02 * rng.standard_normal(w.d)).astype(np.float32)).cuda()
    src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    for _ in range(args.steps):
        bench.bench_copy(torch, src, dst)
    for _ in range(args.steps):
        wht.wht_affine_forward(x, alpha, beta, y=y)
    for _ in range(args.steps):
        wht.wht_affine_backward(dy, x, alpha, dx=dx)
    torch.cuda.synchronize()
    print(f"drove {args.steps} x (copy 1 GiB, forward, backward) on {w.name}", flush=True)


def series(args):
    """fwd+bwd steps from an idle GPU: per step the two entry points' times (events) and the shader
    clock right after the step (probe kernel: shader-clock ticks per 100 MHz tick)."""
    import time
    import torch
    import bench
    import paper_2603_08343_amd as wht
    from paper_2603_08343_amd import synth

    K = args.steps
    if args.copy:
        n = 512 << 20
        src = [torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(3)]
        dst = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(3)]
        probes = torch.zeros(K, 2, dtype=torch.int64, device="cuda")
        ev = [[bench.StreamEvent(torch) for _ in range(2)] for _ in range(K)]
        torch.cuda.synchronize()
        time.sleep(args.idle)
        for i in range(K):
            ev[i][0].record()
            bench.bench_copy(torch, src[i % 3], dst[i % 3])
            ev[i][1].record()
            bench.bench_clock_probe(torch, probes[i])
        torch.cuda.synchronize()
        p = probes.cpu().numpy()
        print(f"plain copy of 512 MiB (copy_kernel, bench-only library); {K} steps after {args.idle} s of idling")
        print("step copy_us shader_MHz")
        for i in range(K):
            print(f"{i:4d} {ev[i][0].elapsed_time(ev[i][1]) * 1e3:7.1f} {100.0 * p[i][0] / max(1, p[i][1]):8.0f}")
        return
    w = synth.WORKLOADS[args.workload]
    b = bench.Bench(torch, wht, synth, args.workload)
    probes = torch.zeros(K, 2, dtype=torch.int64, device="cuda")
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    torch.cuda.synchronize()
    time.sleep(args.idle)
    for i in range(K):
        ev[i][0].record()
        b.fwd(i)
        ev[i][1].record()
        if w.backward:
            b.bwd(i)
        ev[i][2].record()
        bench.bench_clock_probe(torch, probes[i])
    torch.cuda.synchronize()
    p = probes.cpu().numpy()
    print(f"workload {w.name}: N={w.N} d={w.d} {w.dtype} I/O; {K} steps after {args.idle} s of idling")
    print("step  fwd_us  bwd_us  shader_MHz")
    rows = []
    for i in range(K):
        f = ev[i][0].elapsed_time(ev[i][1]) * 1e3
        g = ev[i][1].elapsed_time(ev[i][2]) * 1e3 if w.backward else 0.0
        mhz = 100.0 * p[i][0] / max(1, p[i][1])
        rows.append((f, g, mhz))
        print(f"{i:4d} {f:7.1f} {g:7.1f} {mhz:8.0f}")
    lo, hi = 5, min(K, 25)
    print(f"mean of steps {lo}..{hi - 1} (the window a run with 5 warm-up and 20 timed steps sees): "
          f"fwd {sum(r[0] for r in rows[lo:hi]) / (hi - lo):.1f} us, bwd {sum(r[1] for r in rows[lo:hi]) / (hi - lo):.1f} us, "
          f"clock {sum(r[2] for r in rows[lo:hi]) / (hi - lo):.0f} MHz (min {min(r[2] for r in rows[lo:hi]):.0f})")
    t = rows[max(0, K - 20):]
    print(f"mean of the last {len(t)} steps: fwd {sum(r[0] for r in t) / len(t):.1f} us, bwd {sum(r[1] for r in t) / len(t):.1f} us, "
          f"clock {sum(r[2] for r in t) / len(t):.0f} MHz")


def _ours(name: str) -> bool:
    return "wht::" in name or name.startswith(("copy_kernel", "void copy_kernel"))


def _short(name: str) -> str:
    name = name.replace("void wht::", "").replace("wht::", "")
    return name.split("(")[0].strip()


def summarize(args):
    from paper_2603_08343_amd import synth
    w = synth.WORKLOADS[args.workload]
    s = 2 if w.dtype == "bf16" else 4
    algo = {"forward_kernel": 2 * w.N * w.d * s + 8 * w.d, "forward_once_kernel": 2 * w.N * w.d * s + 8 * w.d,
            "backward_kernel": 3 * w.N * w.d * s + 12 * w.d,
            "backward_teams_kernel": 3 * w.N * w.d * s + 12 * w.d}
    out = [f"workload {w.name}: N={w.N} d={w.d} {w.dtype} I/O"]

    if args.kernel_stats:
        out.append("")
        out.append("kernel-trace --stats (ns): name, calls, average, min, max, % of GPU time")
        for row in csv.DictReader(open(args.kernel_stats)):
            if _ours(row["Name"]):
                out.append(f"  {_short(row['Name']):48s} calls {row['Calls']:>5s}  avg {float(row['AverageNs']):10.0f}"
                           f"  min {row['MinNs']:>8s}  max {row['MaxNs']:>8s}  {row['Percentage']}%")

    if args.kernel_trace:
        # the benchmark's timed region is its last `--last` steps: the launches before it are the
        # untimed warm-up, during which the clocks are still settling
        per_kernel = collections.defaultdict(list)
        for row in csv.DictReader(open(args.kernel_trace)):
            if _ours(row["Kernel_Name"]):
                per_kernel[_short(row["Kernel_Name"])].append(
                    (int(row["Start_Timestamp"]), int(row["End_Timestamp"]) - int(row["Start_Timestamp"])))
        out.append("")
        out.append(f"kernel-trace, last {args.last} launches of each kernel (the benchmark's timed region), ns:")
        for k, launches in sorted(per_kernel.items()):
            tail = [d for _, d in sorted(launches)[-args.last:]]
            out.append(f"  {k:48s} calls {len(tail):>5d}  avg {sum(tail) / len(tail):10.0f}"
                       f"  min {min(tail):>8d}  max {max(tail):>8d}")

    counters = collections.defaultdict(lambda: collections.defaultdict(list))
    durations = collections.defaultdict(list)
    for pattern in args.pmc or []:
        for path in glob.glob(pattern):
            for row in csv.DictReader(open(path)):
                if not _ours(row["Kernel_Name"]):
                    continue
                k = _short(row["Kernel_Name"])
                counters[k][row["Counter_Name"]].append(float(row["Counter_Value"]))
                durations[k].append(float(row["End_Timestamp"]) - float(row["Start_Timestamp"]))
    if counters:
        out.append("")
        out.append("counter passes (mean per dispatch; kernels run serialised under --pmc)")
        copy = counters.get("copy_kernel", {})
        scale = {}
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            if c in copy:
                mean = sum(copy[c]) / len(copy[c])
                scale[c] = COPY_BYTES / (mean * 1024.0)
                out.append(f"  calibration: copy_kernel moves {COPY_BYTES} B each way; {c} reads {mean:.0f} KiB"
                           f" -> scale factor {scale[c]:.4f}")
        for k, cs in sorted(counters.items()):
            out.append(f"  {k}")
            dur_ns = sum(durations[k]) / len(durations[k])
            for c, vals in sorted(cs.items()):
                out.append(f"      {c:28s} {sum(vals) / len(vals):16.0f}")
            base = k.split("<")[0]
            traffic = 0.0
            have = 0
            for c in ("FETCH_SIZE", "WRITE_SIZE"):
                if c in cs and c in scale:
                    b = sum(cs[c]) / len(cs[c]) * 1024.0 * scale[c]
                    traffic += b
                    have += 1
                    out.append(f"      {c} scaled: {b:.4e} B per launch")
            if have == 2 and base in algo:
                out.append(f"      HBM traffic {traffic:.4e} B per launch vs algorithmic {algo[base]:.4e} B"
                           f" (ratio {traffic / algo[base]:.3f})")
                out.append("      TRAFFIC_JSON " + json.dumps({"kernel": base, "workload": w.name,
                                                               "traffic_bytes_per_launch": traffic}))
            if "SQ_ACTIVE_INST_VALU" in cs and "GRBM_GUI_ACTIVE" in cs:
                gui = sum(cs["GRBM_GUI_ACTIVE"]) / len(cs["GRBM_GUI_ACTIVE"]) / NUM_XCD
                valu = sum(cs["SQ_ACTIVE_INST_VALU"]) / len(cs["SQ_ACTIVE_INST_VALU"])
                out.append(f"      VALU busy = 4*SQ_ACTIVE_INST_VALU / (GRBM_GUI_ACTIVE/{NUM_XCD} * {NUM_SIMD} SIMDs)"
                           f" = {4 * valu / (gui * NUM_SIMD) * 100:.1f} %")
                if "SQ_VALU_MFMA_BUSY_CYCLES" in cs:
                    mf = sum(cs["SQ_VALU_MFMA_BUSY_CYCLES"]) / len(cs["SQ_VALU_MFMA_BUSY_CYCLES"])
                    out.append(f"      MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE/{NUM_XCD} * {NUM_SIMD})"
                               f" = {mf / (gui * NUM_SIMD) * 100:.1f} %")
            if "SQ_LDS_BANK_CONFLICT" in cs and "SQ_ACTIVE_INST_LDS" in cs:
                a = sum(cs["SQ_ACTIVE_INST_LDS"]) / len(cs["SQ_ACTIVE_INST_LDS"])
                b = sum(cs["SQ_LDS_BANK_CONFLICT"]) / len(cs["SQ_LDS_BANK_CONFLICT"])
                out.append(f"      LDS bank-conflict cycles / LDS active cycles = {b / a * 100 if a else 0:.1f} %")
            out.append(f"      duration under the counter pass: {dur_ns:.0f} ns")
    text = "\n".join(out) + "\n"
    if args.out:
        with open(args.out, "a") as f:
            f.write(text)
    sys.stdout.write(text)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    d = sub.add_parser("drive")
    d.add_argument("--workload", default="C5_large")
    d.add_argument("--steps", type=int, default=3)
    d.add_argument("--schedule", choices=["default", "butterfly"], default="default")
    d.set_defaults(fn=drive)
    c = sub.add_parser("series")
    c.add_argument("--workload", default="C5_large")
    c.add_argument("--steps", type=int, default=80)
    c.add_argument("--idle", type=float, default=1.0, help="seconds of idling before the first step")
    c.add_argument("--copy", action="store_true", help="time plain 512 MiB copies instead of the layer")
    c.set_defaults(fn=series)
    s = sub.add_parser("summarize")
    s.add_argument("--workload", default="C5_large")
    s.add_argument("--kernel-stats")
    s.add_argument("--kernel-trace", help="kt_kernel_trace.csv of the same run")
    s.add_argument("--last", type=int, default=100, help="launches per kernel in the timed region")
    s.add_argument("--pmc", nargs="*")
    s.add_argument("--out")
    s.set_defaults(fn=summarize)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
