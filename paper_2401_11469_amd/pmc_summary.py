"""Turns rocprofv3 --pmc outputs of bench.py into the counter summary under profiles/.

Run on the GPU machine, from /tmp with TMPDIR=/tmp, one counter set per run (rocprofv3 does
not split counters over passes), each as
    rocprofv3 --pmc <counters> --output-format csv -d <dir>/<tag> -- python3 bench.py <ARGS>
with the tags and counter sets of PASSES below, and for the two byte counters also
    rocprofv3 --pmc FETCH_SIZE  ... -d <dir>/fetch_copy -- python3 bench.py --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE  ... -d <dir>/write_copy -- python3 bench.py --calibrate-copy
then
    python3 -m paper_2401_11469_amd.pmc_summary <dir> <commit>
writes profiles/pmc_counters.json (read by bench.py) and profiles/pmc_counters.md.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH_ARGS = "--steps 10 --warmup 2 --no-cpu-baseline --no-sweep --no-secondary --no-aux"
PASSES = {
    "mfma": "SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_BUSY_CU_CYCLES SQ_WAVE_CYCLES "
            "SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_INSTS_LDS SQ_ACTIVE_INST_LDS GRBM_GUI_ACTIVE",
    "vmem": "SQ_INSTS_VMEM_RD SQ_INST_CYCLES_VMEM_RD SQ_VMEM_TA_ADDR_FIFO_FULL SQ_VMEM_TA_CMD_FIFO_FULL "
            "SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_INST_LEVEL_VMEM SQ_ACTIVE_INST_VMEM GRBM_GUI_ACTIVE",
    "fetch": "FETCH_SIZE",
    "write": "WRITE_SIZE",
}
COPY_KIB = 65536 * 8192 * 2 / 1024          # what bench.py --calibrate-copy reads and writes per dispatch
N_SIMD = 256 * 4
N_XCD = 8                                   # GRBM_GUI_ACTIVE arrives summed over the XCDs


def short(k: str) -> str:
    k = k.replace("zr::(anonymous namespace)::", "").replace("void ", "")
    if ">(" in k and "_kernel<" in k:
        k = k[:k.index(">(") + 1]
        # the trailing phase parameter of the GEMM kernels: 0 (the ordinary launch) is left out,
        # as in the names the library itself reports
        return k[:-4] + ">" if k.startswith("fast_kernel<") and k.endswith(", 0>") else k
    return k.split("(")[0]


def load(d: str):
    """{kernel: {counter: [value per dispatch]}}"""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
        # rocprofv3 writes one row per dispatch and counter: the SUM over the counter's instances
        # (SQ: shader engines x XCDs; TCC: channels x XCDs; GRBM: one per XCD)
        per = collections.defaultdict(float)
        dur = {}
        for row in csv.DictReader(open(f)):
            k = short(row["Kernel_Name"])
            per[(row["Dispatch_Id"], k, row["Counter_Name"])] += float(row["Counter_Value"])
            dur[(row["Dispatch_Id"], k)] = float(row["End_Timestamp"]) - float(row["Start_Timestamp"])
        for (_, k, c), v in per.items():
            acc[k][c].append(v)
        for (_, k), ns in dur.items():
            acc[k]["_duration_ns"].append(ns)
    return acc


def mean(v):
    return sum(v) / len(v) if v else float("nan")


def main(d: str, commit: str) -> None:
    mf, vm = load(os.path.join(d, "mfma")), load(os.path.join(d, "vmem"))
    fe, wr = load(os.path.join(d, "fetch")), load(os.path.join(d, "write"))
    fc, wc = load(os.path.join(d, "fetch_copy")), load(os.path.join(d, "write_copy"))
    copy_k = [k for k in fc if "compact" in k][0]
    kf = COPY_KIB / mean(fc[copy_k]["FETCH_SIZE"])
    kw = COPY_KIB / mean(wc[copy_k]["WRITE_SIZE"])
    kernels = {}
    lines = ["# Hardware counters per kernel: bench.py on the Llama-2-7B TP=4 layer shard (bf16), one MI355X", "",
             f"Recorded at commit {commit}.  Commands (GPU box, from /tmp with TMPDIR=/tmp; one counter set per run):", ""]
    for tag, ctrs in PASSES.items():
        lines.append(f"    rocprofv3 --pmc {ctrs} --output-format csv -d <dir>/{tag} -- python3 bench.py {BENCH_ARGS}")
    lines += ["    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir>/fetch_copy -- python3 bench.py --calibrate-copy",
              "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir>/write_copy -- python3 bench.py --calibrate-copy",
              "    python3 -m paper_2401_11469_amd.pmc_summary <dir> <commit>", "",
              f"Byte counters are scaled by what they read for the calibration copy ({COPY_KIB:.0f} KiB read and written per "
              f"dispatch): FETCH_SIZE x {kf:.3f}, WRITE_SIZE x {kw:.3f}.  Values are means over all dispatches of a kernel in the run "
              "(the GEMM instantiations mix the five projections and the per-step ratios).  MB = 1e6 bytes.", "",
              "MFMA utilisation = SQ_VALU_MFMA_BUSY_CYCLES (summed over all SIMDs) / (GRBM_GUI_ACTIVE per XCD x 1024 SIMDs), "
              "the expression of rocprofv3's own derived metric MfmaUtil (the CSV holds GRBM_GUI_ACTIVE summed over the 8 XCDs, "
              "hence / 8): the share of "
              "SIMD-cycles in which the matrix pipe is busy while the kernel runs, idle compute units included.", "",
              "Clock = GRBM_GUI_ACTIVE per XCD / the dispatch's duration.  The counter window is a few microseconds longer than "
              "the dispatch, so the figure is a few per cent high for kernels of 100 us and meaningless for those of 10-20 us "
              "(they read above the 2.4 GHz the chip can run at).", "",
              "| kernel | dispatches | clock MHz | MFMA util | MFMA MOPS (bf16) / dispatch | LDS bank-conflict cycles / LDS active cycles | "
              "wave cycles waiting on any instruction | VMEM reads issued | TA address-FIFO-full cycles | fetched MB | written MB |",
              "|---|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|"]
    order = sorted(mf, key=lambda k: -sum(mf[k].get("GRBM_GUI_ACTIVE", [0])))
    for k in order:
        if "kernel" not in k:
            continue
        m, v = mf[k], vm.get(k, {})
        gui = mean(m.get("GRBM_GUI_ACTIVE", [])) / N_XCD        # cycles the kernel ran
        busy = mean(m.get("SQ_VALU_MFMA_BUSY_CYCLES", []))
        util = busy / (gui * N_SIMD) if gui and gui == gui else float("nan")
        mhz = gui / mean(m.get("_duration_ns", [])) * 1e3 if m.get("_duration_ns") and gui == gui else float("nan")
        lds_c, lds_a = mean(m.get("SQ_LDS_BANK_CONFLICT", [])), mean(m.get("SQ_LDS_IDX_ACTIVE", []))
        wait, wave = mean(v.get("SQ_WAIT_INST_ANY", [])), mean(m.get("SQ_WAVE_CYCLES", []))
        f = mean(fe.get(k, {}).get("FETCH_SIZE", [])) * kf * 1024 / 1e6
        w = mean(wr.get(k, {}).get("WRITE_SIZE", [])) * kw * 1024 / 1e6
        entry = {"dispatches": len(m.get("GRBM_GUI_ACTIVE", [])),
                 "mfma_util": None if util != util else round(util, 4),
                 "traffic_bytes": None if (f != f or w != w) else int(round((f + w) * 1e6)),
                 "lds_bank_conflict_share": None if not lds_a or lds_a != lds_a else round(lds_c / lds_a, 4),
                 "wait_inst_any_share": None if not wave or wave != wave or wait != wait else round(wait / wave, 4)}
        kernels[k] = entry
        entry["clock_mhz"] = None if mhz != mhz else round(mhz)
        lines.append(f"| `{k}` | {entry['dispatches']} | {mhz:.0f} | {util:.3f} | {mean(m.get('SQ_INSTS_VALU_MFMA_MOPS_BF16', [])):.4g} | "
                     f"{lds_c:.3g} / {lds_a:.3g} | {wait:.3g} of {wave:.3g} | {mean(v.get('SQ_INSTS_VMEM_RD', [])):.4g} | "
                     f"{mean(v.get('SQ_VMEM_TA_ADDR_FIFO_FULL', [])):.3g} | {f:.1f} | {w:.1f} |")
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    with open(os.path.join(ROOT, "profiles", "pmc_counters.json"), "w") as fjson:
        json.dump({"commit": commit, "bench_args": BENCH_ARGS, "fetch_scale": kf, "write_scale": kw, "kernels": kernels},
                  fjson, indent=1, sort_keys=True)
    with open(os.path.join(ROOT, "profiles", "pmc_counters.md"), "w") as fmd:
        fmd.write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else "unknown")
