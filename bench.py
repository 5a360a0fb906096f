"""Benchmark of the resized tensor-parallel shard GEMMs on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input for
every projection of the workload's layer shard: resize_select (scores ->
kept/dropped index lists), resized_linear_fwd, resized_linear_bwd (dX and dW)
with the scatter + Zero-imputation epilogue.  The step's pruning ratio is
drawn from a seeded sequence over the workload's ratio list (time-varying
straggler contention).  The metric is effective TFLOP/s over the KEPT work
(6*M*K*N*n'/n per projection) with all inputs resident in HBM.

Prints ONE JSON line.  One GPU only.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}     # MI355X dense MFMA peaks
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch (fetched + written) of a GEMM instantiation on the default
# workload, from the hardware counters FETCH_SIZE / WRITE_SIZE of two
# `rocprofv3 --pmc` runs of this file, each scaled by what the same counter
# reads for --calibrate-copy; the summary under profiles/ gives the commands.
# Counters cannot be read from inside the timed run, so the figures live here.
PMC_TRAFFIC_BYTES = {
    "fast_kernel<DmaP, DmaQM, 256, 256, 2, 4>": 246577848,
    "fast_kernel<DmaP, DmaQ, 256, 256, 2, 4>": 309871558,
    "fast_kernel<DmaQ, DmaQ, 192, 256, 2, 4>": 398153916,
    "fast_kernel<DmaP, DmaP, 256, 256, 2, 4>": 257406170,
    "fast_kernel<DmaQ, DmaQ, 128, 128, 2, 2>": 288334151,
    "fast_kernel<DmaP, DmaP, 128, 128, 2, 2>": 132607727,
    "fast_kernel<DmaP, DmaP, 256, 192, 4, 2>": 209274561,
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload id (4 = Llama-2-7B TP=4 layer shard)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain copy of known size (the reference dispatch that scales the HBM "
                         "byte counters of a rocprofv3 --pmc run) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one tensor-parallel task's shard on ONE GPU; --gpus must be 1 "
              "(no collectives or sharding are part of this build)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2401_11469_amd import workloads as wl
    from paper_2401_11469_amd import zr

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[args.config]
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    M = cfg.M

    if args.calibrate_copy:
        # compact_cols_kernel with the identity index list: reads and writes rows*n*2 bytes
        rows, n = 65536, 8192
        src = torch.ones((rows, n), dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        ident = torch.arange(n, dtype=torch.int32, device=dev)
        for _ in range(10):
            zr.extract_kept_columns(src, ident, out=dst)
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
        print(json.dumps({"calibrate_copy": "compact_cols_kernel", "dispatches": 10,
                          "bytes_read_per_dispatch": rows * n * 2, "bytes_written_per_dispatch": rows * n * 2}))
        return 0

    # ---- inputs resident in HBM before any timing ---------------------------
    projs = []
    for pi, pr in enumerate(cfg.projections):
        t = wl.make_tensors(args.config, pi)
        scores = wl.make_scores(args.config, pi, t["W"])
        n = pr.n_axis
        # Column-parallel shards (kept list on the output features) are stored [N x K]
        # ([out, in]), row-parallel ones [K x N]: in both the kept list selects ROWS
        # of the stored weight, which the GEMM loaders gather in flight (no weight copy).
        nk = pr.mode == zr.DROP_N
        Wd = torch.from_numpy(np.ascontiguousarray(t["W"].T) if nk else t["W"]).to(tdt).to(dev)
        projs.append(dict(
            pr=pr, n=n, layout=zr.W_NK if nk else zr.W_KN,
            X=torch.from_numpy(t["X"]).to(tdt).to(dev), W=Wd,
            dY=torch.from_numpy(t["dY"]).to(tdt).to(dev), scores=torch.from_numpy(scores).to(dev),
            Y=torch.empty((M, pr.N), dtype=tdt, device=dev), dX=torch.empty((M, pr.K), dtype=tdt, device=dev),
            dW=torch.empty(tuple(Wd.shape), dtype=tdt, device=dev),
            keep=torch.empty((1, n), dtype=torch.int32, device=dev),
            drop=torch.empty((1, n), dtype=torch.int32, device=dev)))
        del t
    # one scratch buffer shared by all calls (they are ordered on one stream)
    ws_bytes = max(zr.workspace_bytes(M, p["pr"].K, p["pr"].N, p["n"], p["pr"].mode, tdt) for p in projs)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev) if ws_bytes else None
    torch.cuda.synchronize()

    def step_flops(ratio: float) -> float:
        return sum(wl.kept_flops(M, p["pr"].K, p["pr"].N, p["n"],
                                 zr.keep_count(p["n"], wl.ratio_for(cfg, p["pr"], ratio))) for p in projs)

    extracts = []

    def run_step(ratio: float, events=None):
        # the step's selections: one launch for all projections of the shard
        keeps, _ = zr.resize_select_multi([p["scores"] for p in projs],
                                          [wl.ratio_for(cfg, p["pr"], ratio) for p in projs],
                                          keep_idx=[p["keep"] for p in projs], drop_idx=[p["drop"] for p in projs])
        for p, keep in zip(projs, keeps):
            pr = p["pr"]
            full = keep.numel() == p["n"]
            if events is None:
                zr.resized_linear_fwd(p["X"], p["W"], keep, pr.mode, Y=p["Y"], workspace=ws, w_layout=p["layout"])
                # the scratch buffer still holds what this projection's forward extracted
                zr.resized_linear_bwd(p["X"], p["W"], p["dY"], keep, pr.mode, dX=p["dX"], dW=p["dW"], workspace=ws,
                                      w_layout=p["layout"], workspace_holds_forward=True)
            else:
                # one event pair per product, recorded by the library right around the
                # product's own GEMM launch(es) (zr_debug_time_next_product), so that an
                # extraction into the scratch buffer is not charged to the GEMM; the
                # extraction kernel is bracketed separately where it runs on its own
                fl = 2.0 * M * pr.K * pr.N * keep.numel() / p["n"]
                for op in ("fwd", "dX", "dW"):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(); e1.record()            # creates the HIP events
                    zr.debug_time_next_product(e0, e1)
                    if op == "fwd":
                        zr.resized_linear_fwd(p["X"], p["W"], keep, pr.mode, Y=p["Y"], workspace=ws, w_layout=p["layout"])
                    elif op == "dX":
                        zr.resized_linear_bwd(p["X"], p["W"], p["dY"], keep, pr.mode, dX=p["dX"], need_dW=False,
                                              workspace=ws, w_layout=p["layout"])
                    else:
                        zr.resized_linear_bwd(p["X"], p["W"], p["dY"], keep, pr.mode, dW=p["dW"], need_dX=False,
                                              workspace=ws, w_layout=p["layout"], workspace_holds_forward=True)
                    events.append((zr.debug_last_kernel(), fl, e0, e1))
                if ws is not None and not full and tdt == torch.bfloat16:
                    src = p["X"] if pr.mode == zr.DROP_K else p["dY"]
                    width = (keep.numel() + 63) // 64 * 64
                    x0, x1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    x0.record()
                    zr.extract_kept_columns(src, keep, out=ws[:M * width * 2].view(tdt).view(M, width))
                    x1.record()
                    extracts.append((x0, x1))

    ratios = wl.ratio_sequence(args.config, args.warmup + args.steps)

    # ---- timed region: exactly --steps steps, events on the launch stream ----
    for r in ratios[:args.warmup]:
        run_step(r)
    torch.cuda.synchronize()
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    t0.record()
    for r in ratios[args.warmup:]:
        run_step(r)
    t1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    gpu_ms = t0.elapsed_time(t1)
    total_ms = max(gpu_ms, wall * 1e3)        # host-launch-bound runs are charged the wall clock
    flops = sum(step_flops(r) for r in ratios[args.warmup:])
    value = flops / (total_ms * 1e-3) / 1e12

    # ---- per-kernel durations (same steps again, one event pair per launch) --
    events = []
    for r in ratios[args.warmup:]:
        run_step(r, events)
    torch.cuda.synchronize()
    per = {}
    for label, fl, e0, e1 in events:
        d = per.setdefault(label, [0, 0.0, 0.0])
        d[0] += 1
        d[1] += fl
        d[2] += e0.elapsed_time(e1)
    extract_ms = sum(a.elapsed_time(b) for a, b in extracts)
    n_extract = len(extracts)
    kernels = {k: {"launches": v[0], "avg_ms": v[2] / v[0], "tflops": v[1] / (v[2] * 1e-3) / 1e12}
               for k, v in per.items()}
    dom = max(per.items(), key=lambda kv: kv[1][2])
    peak = PEAK_TFLOPS[cfg.dtype]
    dom_tflops = dom[1][1] / (dom[1][2] * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": dom[0], "achieved": dom_tflops, "peak": peak, "unit": "TFLOP/s",
                "frac": dom_tflops / peak,
                "traffic": PMC_TRAFFIC_BYTES.get(dom[0]) if args.config == 4 else None,
                "avg_launch_ms": dom[1][2] / dom[1][0], "launches": dom[1][0],
                "note": "achieved = kept FLOPs of the launches of this instantiation / their summed durations "
                        "(HIP events on the launch stream)"}
    extract = {"kernel": "compact_cols_kernel", "launches": n_extract,
               "avg_ms": extract_ms / n_extract if n_extract else None}

    # ---- time vs ratio (median of a few steps each) --------------------------
    sweep = {}
    if not args.no_sweep:
        base_ms = None
        for r in cfg.ratios:
            ms = []
            for _ in range(5):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                run_step(r)
                b.record()
                torch.cuda.synchronize()
                ms.append(a.elapsed_time(b))
            med = float(np.median(ms))
            if base_ms is None:
                base_ms = med
            fl = step_flops(r)
            sweep[f"{r:.2f}"] = {"ms": med, "tflops": fl / (med * 1e-3) / 1e12,
                                 "frac_peak": fl / (med * 1e-3) / 1e12 / peak,
                                 "speedup_vs_first": base_ms / med,
                                 "kept_fraction": fl / step_flops(cfg.ratios[0])}

    # ---- HBM-bound helpers: selector and stand-alone imputation ----------------
    def timed(fn, n=20):
        for _ in range(3):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    aux = {}
    p0 = projs[0]
    aux["select_single_us"] = {
        f"n={p['n']}": timed(lambda p=p: zr.resize_select(p["scores"], 0.25, keep_idx=p["keep"], drop_idx=p["drop"])) * 1e3
        for p in projs}
    nb, nn = 4096, 4096
    sc = torch.rand((nb, nn), dtype=torch.float32, device=dev)
    kb = torch.empty((nb, nn), dtype=torch.int32, device=dev)
    db = torch.empty((nb, nn), dtype=torch.int32, device=dev)
    ms = timed(lambda: zr.resize_select(sc, 0.25, keep_idx=kb, drop_idx=db), n=5)
    aux["select_batched"] = {"batch": nb, "n": nn, "ms": ms, "GB/s": 8.0 * nb * nn / (ms * 1e-3) / 1e9,
                             "frac_hbm_peak": 8.0 * nb * nn / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "bytes": "algorithmic: 4n read + 4n written per vector"}
    del sc, kb, db
    keep25, _ = zr.resize_select(p0["scores"], 0.25)
    ncols = p0["Y"].shape[1] if p0["pr"].mode == zr.DROP_N else p0["dX"].shape[1]
    buf = p0["Y"] if p0["pr"].mode == zr.DROP_N else p0["dX"]
    prev = torch.zeros_like(buf)
    esz = buf.element_size()
    dropped_bytes = esz * M * (ncols - keep25.numel())
    kept_bytes = esz * M * keep25.numel()
    for name, pol, nbytes in (("zero", zr.ZERO, dropped_bytes), ("same", zr.SAME, 2 * dropped_bytes),
                              ("average", zr.AVERAGE, kept_bytes + dropped_bytes)):
        ms = timed(lambda pol=pol: zr.impute(buf, 1, keep25, pol, prev if pol == zr.SAME else None))
        aux[f"impute_{name}"] = {"shape": [M, ncols], "ratio": 0.25, "ms": ms, "GB/s": nbytes / (ms * 1e-3) / 1e9,
                                 "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    del prev
    # weight-variation scores of every projection (2 snapshots read once each)
    pri = {}
    for p in projs:
        W = p["W"]
        Wprev = W.clone()
        # in both storage layouts the pruned axis is the row axis of the stored matrix
        wsb = torch.empty(max(16, zr.priority_workspace_bytes(W.shape[0], W.shape[1], zr.DROP_K)),
                          dtype=torch.uint8, device=dev)
        out = torch.empty(p["n"], dtype=torch.float32, device=dev)
        assert W.shape[0] == p["n"]
        ms = timed(lambda: zr.priority_scores(W, Wprev, zr.DROP_K, scores=out, workspace=wsb))
        nbytes = 2.0 * W.numel() * W.element_size()
        pri[p["pr"].name] = {"stored_shape": list(W.shape), "scores": "one per stored row",
                             "us": ms * 1e3, "GB/s": nbytes / (ms * 1e-3) / 1e9,
                             "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del Wprev, wsb
    aux["priority_scores"] = pri
    cnt = torch.empty(1, dtype=torch.int32, device=dev)
    aux["count_above_us"] = timed(lambda: zr.count_above(p0["scores"], 0.5, count=cnt)) * 1e3
    if tdt == torch.bfloat16:
        # what the matrix cores sustain on register operands alone (no LDS, no memory): the
        # clock the chip holds under MFMA load, next to the published peak
        mf = {}
        ms = timed(lambda: mf.__setitem__("flops", zr.debug_mfma_rate(2048, 2048)), n=3)
        aux["mfma_register_only"] = {"TFLOP/s": mf["flops"] / (ms * 1e-3) / 1e12,
                                     "frac_published_peak": mf["flops"] / (ms * 1e-3) / 1e12 / peak,
                                     "what": "2048 workgroups x 4 wavefronts x 2048 x 8 independent 32x32x16 bf16 MFMAs, register operands"}

    # ---- CPU oracle on the host cores, bounded sample -------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle
        m_slice = min(M, 3072)          # about 15 s of float64 work on the 16 host threads of a GPU machine
        ratio = 0.25
        work = 0.0
        secs = 0.0
        for pi, pr in enumerate(cfg.projections):
            t = wl.make_tensors(args.config, pi, M=m_slice)
            scores = wl.make_scores(args.config, pi, t["W"])
            r = wl.ratio_for(cfg, pr, ratio)
            c0 = time.perf_counter()
            keep, _ = oracle.resize_select(scores, r)
            oracle.resized_linear_fwd(t["X"], t["W"], keep, pr.mode)
            oracle.resized_linear_bwd(t["X"], t["W"], t["dY"], keep, pr.mode)
            secs += time.perf_counter() - c0
            work += wl.kept_flops(m_slice, pr.K, pr.N, pr.n_axis, len(keep))
        cpu = {"value": work / secs / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"{cfg.name}: all {len(cfg.projections)} projections, select+fwd+bwd at ratio {ratio}, "
                         f"first-M slice of {m_slice} tokens (fresh draw), float64, {secs:.1f} s"}

    line = {
        "metric": "effective TFLOP/s (fwd+bwd) of resized TP shard GEMM vs resize ratio; % MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": total_ms / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: M={M} tokens, projections "
                               + ", ".join(f"{p.name}[{p.K}x{p.N}]{p.parallel}" for p in cfg.projections)
                               + "; per-step ratio drawn (seeded) from " + str(list(cfg.ratios)),
                   "path": "resize_select_multi (one launch for the 5 projections) + resized_linear_fwd + resized_linear_bwd(dX,dW), Zero imputation, "
                           "with the optional scratch buffer for the extracted kept columns of activations (the backward call reuses "
                           "what the forward call of the same projection extracted); column-parallel shards "
                           "stored [N x K], row-parallel [K x N] (the kept list selects rows of the stored weight, no weight copy)"},
        "frac_mfma_peak": value / peak,
        "gpu_ms_per_step": gpu_ms / args.steps, "wall_ms_per_step": wall * 1e3 / args.steps,
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "extract": extract, "by_ratio": sweep, "aux": aux,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
