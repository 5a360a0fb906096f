"""Turns a `rocprofv3 --kernel-trace --stats` run of bench.py into the short summary under profiles/.

On the GPU machine, from /tmp with TMPDIR=/tmp:
    rocprofv3 --kernel-trace --stats --output-format csv -d <dir> -- python3 bench.py <ARGS> > <dir>/bench.json
    python3 -m paper_2401_11469_amd.trace_summary <dir> <dir>/bench.json profiles/<name>.md "<ARGS>"
"""
from __future__ import annotations

import csv
import glob
import json
import os
import sys


def short(k: str) -> str:
    k = k.replace("zr::(anonymous namespace)::", "").replace("void ", "")
    if ">(" in k and "_kernel<" in k:
        k = k[:k.index(">(") + 1]
        return k[:-4] + ">" if k.startswith("fast_kernel<") and k.endswith(", 0>") else k
    return k.split("(")[0]


def main(d: str, bench_json: str, out_md: str, args: str) -> None:
    stats = glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True)[0]
    rows = list(csv.DictReader(open(stats)))
    bench = json.loads(open(bench_json).read().strip().splitlines()[-1])
    out = [f"# rocprofv3 kernel trace: bench.py {args}", "",
           f"Workload: {bench['config']['workload']}", "",
           "Command (GPU box, from /tmp with TMPDIR=/tmp):", "",
           f"    rocprofv3 --kernel-trace --stats --output-format csv -d <dir> -- python3 bench.py {args} > <dir>/bench.json",
           f"    python3 -m paper_2401_11469_amd.trace_summary <dir> <dir>/bench.json {out_md} \"{args}\"", "",
           "The run executes warm-up + timed steps + the per-kernel event pass (a step = one selection launch, then forward and "
           "backward of every projection at the step's seeded ratio), so every instantiation below mixes several shapes and ratios.", "",
           "| kernel | calls | total ms | avg us | % |", "|---|---:|---:|---:|---:|"]
    for r in rows:
        if float(r["Percentage"]) < 0.05:
            continue
        out.append(f"| `{short(r['Name'])}` | {r['Calls']} | {float(r['TotalDurationNs']) / 1e6:.2f} | "
                   f"{float(r['AverageNs']) / 1e3:.1f} | {float(r['Percentage']):.2f} |")
    rf = bench["roofline"]
    out += ["", "bench.py's own figures in the same run (HIP events on the launch stream; profiling serialises nothing here, the "
            "kernels of a step already run back to back on one stream):", "",
            f"- value: {bench['value']:.1f} TFLOP/s over kept work, {bench['ms_per_step']:.3f} ms per step",
            f"- dominant kernel by summed duration: `{rf['kernel']}`: {rf['launches']} products, average {rf['avg_launch_ms'] * 1e3:.1f} us, "
            f"{rf['achieved']:.1f} TFLOP/s = {rf['frac'] * 100:.1f} % of the {rf['peak']:.0f} TFLOP/s MFMA peak of the dtype"]
    for k, v in bench["kernels"].items():
        out.append(f"- `{k}`: {v['launches']} products in the event pass, average {v['avg_ms'] * 1e3:.1f} us, {v['tflops']:.1f} TFLOP/s")
    ex = bench.get("extract") or {}
    if ex.get("avg_ms"):
        out.append(f"- extraction (`{ex['kernel']}`): average {ex['avg_ms'] * 1e3:.1f} us, {ex['GB/s']:.0f} GB/s (timed on its own in the event pass)")
    out.append("")
    out.append("A product that the schedule cuts into a big-tile panel and a 128 x 128 remainder panel (or into the two launches of a "
               "split contraction) appears as two kernels in the table above and as one entry, named after both, in bench.py's list.")
    with open(out_md, "w") as f:
        f.write("\n".join(out) + "\n")
    print("\n".join(out))


if __name__ == "__main__":
    main(sys.argv[1], sys.argv[2], sys.argv[3], sys.argv[4])
