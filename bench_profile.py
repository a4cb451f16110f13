"""Helpers around rocprofv3 for the Walsh-Hadamard output layer's kernels.

Two sub-commands:

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


def _short(name: str) -> str:
    name = name.replace("void wht::", "").replace("wht::", "")
    return name.split("(")[0].strip()


def summarize(args):
    from paper_2603_08343_amd import synth
    w = synth.WORKLOADS[args.workload]
    s = 2 if w.dtype == "bf16" else 4
    algo = {"forward_kernel": 2 * w.N * w.d * s + 8 * w.d, "backward_kernel": 3 * w.N * w.d * s + 12 * w.d}
    out = [f"workload {w.name}: N={w.N} d={w.d} {w.dtype} I/O"]

    if args.kernel_stats:
        out.append("")
        out.append("kernel-trace --stats (ns): name, calls, average, min, max, % of GPU time")
        for row in csv.DictReader(open(args.kernel_stats)):
            if "wht::" in row["Name"]:
                out.append(f"  {_short(row['Name']):48s} calls {row['Calls']:>5s}  avg {float(row['AverageNs']):10.0f}"
                           f"  min {row['MinNs']:>8s}  max {row['MaxNs']:>8s}  {row['Percentage']}%")

    if args.kernel_trace:
        # the benchmark's timed region is its last `--last` steps: the launches before it are the
        # untimed warm-up, during which the clocks are still settling
        per_kernel = collections.defaultdict(list)
        for row in csv.DictReader(open(args.kernel_trace)):
            if "wht::" in row["Kernel_Name"]:
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
                if "wht::" not in row["Kernel_Name"]:
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
    d.set_defaults(fn=drive)
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
