"""Builds libzr.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libzr.so")
SOURCES = ["zr_api.hip", "zr_select.hip", "zr_impute.hip", "zr_gemm.hip", "zr_gemm_fast.hip", "zr_compact.hip", "zr_priority.hip",
           "zr_probe.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",
    # packed fp32 VALU ops are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


RESOURCES = os.path.join(PKG, "libzr.resources.txt")


def _resource_table(text: str, hipcc: str):
    """Per-kernel register / scratch / LDS figures from the compiler's resource remarks."""
    import re
    rows, cur = [], None
    for line in text.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = {"name": m.group(1)}
            rows.append(cur)
            continue
        m = re.search(r"remark:\s+(VGPRs|AGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|LDS Size \[bytes/block\]): (\d+)", line)
        if m and cur is not None:
            cur[m.group(1).split(" ")[0]] = int(m.group(2))
    if not rows:
        return []
    import shutil
    filt = shutil.which("llvm-cxxfilt") or shutil.which("c++filt") or "c++filt"
    try:
        names = subprocess.run([filt], input="\n".join(r["name"] for r in rows), stdout=subprocess.PIPE,
                               text=True, check=True).stdout.splitlines()
        for r, n in zip(rows, names):
            r["name"] = n.replace("zr::(anonymous namespace)::", "").replace("void ", "")
    except (OSError, subprocess.CalledProcessError):
        pass
    return rows


def build(verbose: bool = True, out: str = LIB) -> str:
    """Compiles the library; also writes the compiler's per-kernel resource usage next to it
    (a kernel of the fast GEMM path that starts to spill loses 15-20 %, silently)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("ZR_EXTRA_HIPCC_FLAGS", "").split()      # experiments only
    cmd = [hipcc, *FLAGS, "-Rpass-analysis=kernel-resource-usage", *extra, "-I", os.path.join(ROOT, "include"),
           "-I", CSRC, *[os.path.join(CSRC, s) for s in SOURCES], "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if out == LIB and res.returncode == 0:
        rows = _resource_table(res.stdout, hipcc)
        with open(RESOURCES, "w") as f:
            f.write("# kernel | VGPRs | AGPRs | scratch bytes/lane | waves/SIMD | LDS bytes/block\n")
            for r in rows:
                f.write(" | ".join([r["name"].split("(")[0] if "<" not in r["name"] else r["name"][:r["name"].rfind(">") + 1]]
                                   + [str(r.get(k, -1)) for k in ("VGPRs", "AGPRs", "ScratchSize", "Occupancy", "LDS")]) + "\n")
    log = "\n".join(l for l in res.stdout.splitlines()
                    if "is not a recognized feature for this target" not in l
                    and "-Rpass-analysis=kernel-resource-usage" not in l)
    # the remark lines come with source echo lines ("  123 | code", "      | ^"): drop those too
    log = "\n".join(l for l in log.splitlines() if not __import__("re").match(r"^\s*\d*\s*\|", l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose and log.strip():
        print(log)
    return out


if __name__ == "__main__":
    build(out=sys.argv[1] if len(sys.argv) > 1 else LIB)
    sys.exit(0)
