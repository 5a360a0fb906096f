"""Benchmark of the resized tensor-parallel shard GEMMs on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input for
every projection of the workload's layer shard: resize_select (scores ->
kept/dropped index lists), resized_linear_fwd, resized_linear_bwd (dX and dW)
with the scatter + Zero-imputation epilogue.  The step's pruning ratio is
drawn from a seeded sequence over the workload's ratio list (time-varying
straggler contention).  The metric is effective TFLOP/s over the KEPT work
(6*M*K*N*n'/n per projection) with all inputs resident in HBM.

Prints ONE JSON line.  One GPU only.

Besides the contract fields the line carries:
  roofline      dominant GEMM instantiation: kept FLOPs / summed durations (HIP events on the
                launch stream); `traffic` and `mfma_util` come from the hardware-counter
                summary under profiles/ (null when that file has no entry for the kernel)
  cpu_baseline  the oracle on the host cores on a token slice of the SAME inputs, and with it
                the check of the GPU's outputs of one step against that oracle result
  by_ratio      per ratio: median / p10 / p90 of >= 20 single-step samples, speed-up over
                ratio 0, linearity residual [t(r)/t(0)] / (kept fraction) - 1, and the same
                step without the selection launch
  secondary     labelled figures that are NOT the headline: no scratch buffer (in-flight
                gathers), the [K x N] layout for column-parallel shards, the paper-literal
                sweep (contraction axis pruned on every shard, Sec. 3.1's worked example),
                leading dimensions padded off the 8 KB stride, the step replayed as a HIP graph
  aux           selector / imputation / extraction / priority-score rates against HBM peak
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
PMC_JSON = os.path.join(ROOT, "profiles", "pmc_counters.json")


def load_pmc():
    """Hardware-counter figures per kernel name, written by paper_2401_11469_amd/pmc_summary.py
    from rocprofv3 --pmc runs of this file; {} when the file is absent."""
    try:
        with open(PMC_JSON) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload id (4 = Llama-2-7B TP=4 layer shard)")
    ap.add_argument("--samples", type=int, default=20, help="single-step samples per ratio in by_ratio")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-secondary", action="store_true")
    ap.add_argument("--no-aux", action="store_true")
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
    peak = PEAK_TFLOPS[cfg.dtype]

    if args.calibrate_copy:
        # the extraction kernel with the identity index list: reads and writes rows*n*2 bytes
        rows, n = 65536, 8192
        src = torch.ones((rows, n), dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        ident = torch.arange(n, dtype=torch.int32, device=dev)
        for _ in range(10):
            zr.extract_kept_columns(src, ident, out=dst)
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
        print(json.dumps({"calibrate_copy": "extraction kernel, identity list", "dispatches": 10,
                          "bytes_read_per_dispatch": rows * n * 2, "bytes_written_per_dispatch": rows * n * 2}))
        return 0

    # ---- inputs resident in HBM before any timing ---------------------------
    def padded(rows, cols, pad):
        """[rows x cols] tensor; with pad, a view into a buffer whose rows are pad elements longer."""
        if not pad:
            return torch.empty((rows, cols), dtype=tdt, device=dev)
        return torch.empty((rows, cols + pad), dtype=tdt, device=dev)[:, :cols]

    host = []
    for pi, pr in enumerate(cfg.projections):
        t = wl.make_tensors(args.config, pi)
        host.append(dict(t=t, scores=wl.make_scores(args.config, pi, t["W"])))

    def make_projs(col_layout="NK", col_mode=None, pad=0):
        """Device tensors of the shard.  col_layout: how column-parallel shards are stored;
        col_mode: pruning mode of column-parallel shards (None = the workload's: output features)."""
        projs = []
        for pi, pr in enumerate(cfg.projections):
            t = host[pi]["t"]
            mode = pr.mode if (col_mode is None or pr.parallel != "col") else col_mode
            n = pr.N if mode == zr.DROP_N else pr.K
            nk = pr.parallel == "col" and col_layout == "NK"
            Wh = np.ascontiguousarray(t["W"].T) if nk else t["W"]
            if mode == pr.mode:
                sc = host[pi]["scores"]
            else:       # the other axis of the same weight: L2 norm of each row of W[K x N]
                sc = np.sqrt((t["W"].astype(np.float64) ** 2).sum(axis=1)).astype(np.float32)
            X, dY = padded(M, pr.K, pad), padded(M, pr.N, pad)
            X.copy_(torch.from_numpy(t["X"]).to(tdt))
            dY.copy_(torch.from_numpy(t["dY"]).to(tdt))
            projs.append(dict(
                pr=pr, n=n, mode=mode, layout=zr.W_NK if nk else zr.W_KN, X=X, dY=dY,
                W=torch.from_numpy(Wh).to(tdt).to(dev), scores=torch.from_numpy(sc).to(dev),
                Y=padded(M, pr.N, pad), dX=padded(M, pr.K, pad),
                dW=torch.empty(tuple(Wh.shape), dtype=tdt, device=dev),
                keep=torch.empty((1, n), dtype=torch.int32, device=dev),
                drop=torch.empty((1, n), dtype=torch.int32, device=dev)))
        return projs

    # Headline layout: column-parallel shards (kept list on the output features) are stored
    # [N x K] ([out, in]), row-parallel ones [K x N]: in both the kept list selects ROWS of the
    # stored weight, which the GEMM loaders gather in flight (no weight copy).
    projs = make_projs()
    # one scratch buffer shared by all calls (they are ordered on one stream)
    # (sized for either axis of every projection: the secondary figures prune the other axis too)
    ws_bytes = max(zr.workspace_bytes(M, p["pr"].K, p["pr"].N, max(p["pr"].K, p["pr"].N), zr.DROP_K, tdt) for p in projs)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev) if ws_bytes else None
    torch.cuda.synchronize()

    def step_flops(ratio: float, ps=None) -> float:
        return sum(wl.kept_flops(M, p["pr"].K, p["pr"].N, p["n"],
                                 zr.keep_count(p["n"], wl.ratio_for(cfg, p["pr"], ratio))) for p in (ps or projs))

    def select(ps, ratio):
        return zr.resize_select_multi([p["scores"] for p in ps], [wl.ratio_for(cfg, p["pr"], ratio) for p in ps],
                                      keep_idx=[p["keep"] for p in ps], drop_idx=[p["drop"] for p in ps])[0]

    def run_step(ratio: float, ps=None, use_ws=True, keeps=None):
        """One step: the selections (one launch for all projections), then forward and backward
        of every projection.  keeps: kept lists of an earlier selection (the step without it)."""
        ps = ps or projs
        if keeps is None:
            keeps = select(ps, ratio)
        w = ws if use_ws else None
        for p, keep in zip(ps, keeps):
            zr.resized_linear_fwd(p["X"], p["W"], keep, p["mode"], Y=p["Y"], workspace=w, w_layout=p["layout"])
            # the scratch buffer still holds what this projection's forward extracted
            zr.resized_linear_bwd(p["X"], p["W"], p["dY"], keep, p["mode"], dX=p["dX"], dW=p["dW"], workspace=w,
                                  w_layout=p["layout"], workspace_holds_forward=use_ws)
        return keeps

    extracts = []

    def run_step_events(ratio: float, events):
        # one event pair per product, recorded by the library right around the product's own
        # GEMM launch(es) (zr_debug_time_next_product), so that an extraction into the scratch
        # buffer is not charged to the GEMM; the extraction kernel is bracketed separately
        keeps = select(projs, ratio)
        for p, keep in zip(projs, keeps):
            pr = p["pr"]
            full = keep.numel() == p["n"]
            fl = 2.0 * M * pr.K * pr.N * keep.numel() / p["n"]
            # algorithmic bytes of a product: the kept operand slices read once, the full-shape output written once
            esz = p["X"].element_size()
            nk = keep.numel()
            if p["mode"] == zr.DROP_K:
                nbytes = {"fwd": M * nk + nk * pr.N + M * pr.N, "dX": M * pr.N + nk * pr.N + M * pr.K,
                          "dW": M * nk + M * pr.N + pr.K * pr.N}
            else:
                nbytes = {"fwd": M * pr.K + pr.K * nk + M * pr.N, "dX": M * nk + pr.K * nk + M * pr.K,
                          "dW": M * pr.K + M * nk + pr.K * pr.N}
            for op in ("fwd", "dX", "dW"):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(); e1.record()            # creates the HIP events
                zr.debug_time_next_product(e0, e1)
                if op == "fwd":
                    zr.resized_linear_fwd(p["X"], p["W"], keep, p["mode"], Y=p["Y"], workspace=ws, w_layout=p["layout"])
                elif op == "dX":
                    zr.resized_linear_bwd(p["X"], p["W"], p["dY"], keep, p["mode"], dX=p["dX"], need_dW=False,
                                          workspace=ws, w_layout=p["layout"])
                else:
                    zr.resized_linear_bwd(p["X"], p["W"], p["dY"], keep, p["mode"], dW=p["dW"], need_dX=False,
                                          workspace=ws, w_layout=p["layout"], workspace_holds_forward=True)
                events.append((zr.debug_last_kernel(), fl, e0, e1, float(esz * nbytes[op])))
            if ws is not None and not full and tdt == torch.bfloat16:
                src = p["X"] if p["mode"] == zr.DROP_K else p["dY"]
                width = (keep.numel() + 63) // 64 * 64
                x0, x1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                x0.record()
                zr.extract_kept_columns(src, keep, out=ws[:M * width * 2].view(tdt).view(M, width))
                x1.record()
                extracts.append((x0, x1, 2.0 * M * (src.shape[1] + width)))

    ratios = wl.ratio_sequence(args.config, args.warmup + args.steps)

    def timed_sequence(fn):
        """W warm-up steps, then exactly K steps between events on the launch stream."""
        for r in ratios[:args.warmup]:
            fn(r)
        torch.cuda.synchronize()
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        wall0 = time.perf_counter()
        t0.record()
        for r in ratios[args.warmup:]:
            fn(r)
        t1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - wall0
        return t0.elapsed_time(t1), wall * 1e3

    # ---- timed region: exactly --steps steps ---------------------------------
    gpu_ms, wall_ms = timed_sequence(run_step)
    total_ms = max(gpu_ms, wall_ms)           # host-launch-bound runs are charged the wall clock
    flops = sum(step_flops(r) for r in ratios[args.warmup:])
    value = flops / (total_ms * 1e-3) / 1e12

    # ---- per-kernel durations (same steps again, one event pair per launch) --
    events = []
    for r in ratios[args.warmup:]:
        run_step_events(r, events)
    torch.cuda.synchronize()
    per = {}
    for label, fl, e0, e1, nb in events:
        d = per.setdefault(label, [0, 0.0, 0.0, 0.0])
        d[0] += 1
        d[1] += fl
        d[2] += e0.elapsed_time(e1)
        d[3] += nb
    pmc = load_pmc()
    pmc_k = pmc.get("kernels", {}) if args.config == 4 else {}
    # (algorithmic GB/s and FLOP per byte beside the TFLOP/s: a product below ~310 FLOP/B, such as the
    # GPT-2 shard's `out` projection with a contraction of 256, is bound by HBM, not by the matrix pipes)
    kernels = {k: {"launches": v[0], "avg_ms": v[2] / v[0], "tflops": v[1] / (v[2] * 1e-3) / 1e12,
                   "algorithmic_GB/s": v[3] / (v[2] * 1e-3) / 1e9, "flop_per_byte": v[1] / v[3],
                   "mfma_util": pmc_k.get(k, {}).get("mfma_util")} for k, v in per.items()}
    dom = max(per.items(), key=lambda kv: kv[1][2])
    dom_tflops = dom[1][1] / (dom[1][2] * 1e-3) / 1e12
    dom_pmc = pmc_k.get(dom[0], {})
    roofline = {"bound": "mfma", "kernel": dom[0], "achieved": dom_tflops, "peak": peak, "unit": "TFLOP/s",
                "frac": dom_tflops / peak,
                "traffic": dom_pmc.get("traffic_bytes"), "mfma_util": dom_pmc.get("mfma_util"),
                "counters_from": (f"profiles/pmc_counters.json (recorded at commit {pmc.get('commit', '?')}, "
                                  "not measured in this run)") if dom_pmc else None,
                "avg_launch_ms": dom[1][2] / dom[1][0], "launches": dom[1][0],
                "note": "achieved = kept FLOPs of the launches of this instantiation / their summed durations "
                        "(HIP events on the launch stream)"}
    ex_ms = sum(a.elapsed_time(b) for a, b, _ in extracts)
    ex_bytes = sum(b for _, _, b in extracts)
    extract = {"kernel": "compact_rows_lds_kernel", "launches": len(extracts),
               "avg_ms": ex_ms / len(extracts) if extracts else None,
               "GB/s": ex_bytes / (ex_ms * 1e-3) / 1e9 if extracts else None,
               "frac_hbm_peak": ex_bytes / (ex_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if extracts else None,
               "bytes": "rows x (n read + width written) x 2"}

    # ---- time vs ratio ---------------------------------------------------------
    STEPS_PER_SAMPLE = 3

    def sample_steps(fn, n):
        # a sample = STEPS_PER_SAMPLE steps enqueued back to back (as in the headline loop); with one
        # step per sample the GPU waits for the host between the selection launch and the first
        # product, 30-60 us that no pipelined caller sees
        ms = []
        for _ in range(n):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(STEPS_PER_SAMPLE):
                fn()
            b.record()
            torch.cuda.synchronize()
            ms.append(a.elapsed_time(b) / STEPS_PER_SAMPLE)
        return np.array(ms)

    sweep = {}
    if not args.no_sweep:
        base_ms = None
        fl0 = step_flops(cfg.ratios[0])
        for r in cfg.ratios:
            run_step(r)
            ms = sample_steps(lambda: run_step(r), args.samples)
            keeps = select(projs, r)
            ms_nosel = sample_steps(lambda: run_step(r, keeps=keeps), args.samples)
            med = float(np.median(ms))
            if base_ms is None:
                base_ms = med
            fl = step_flops(r)
            sweep[f"{r:.2f}"] = {"ms": med, "p10": float(np.percentile(ms, 10)), "p90": float(np.percentile(ms, 90)),
                                 "samples": args.samples, "steps_per_sample": STEPS_PER_SAMPLE, "ms_without_select": float(np.median(ms_nosel)),
                                 "tflops": fl / (med * 1e-3) / 1e12, "frac_peak": fl / (med * 1e-3) / 1e12 / peak,
                                 "speedup_vs_first": base_ms / med, "kept_fraction": fl / fl0,
                                 "linearity_residual": (med / base_ms) / (fl / fl0) - 1.0}

    # ---- secondary figures (labelled, never the headline) ----------------------
    secondary = {}
    if not args.no_secondary and tdt == torch.bfloat16:
        def figure(ps, use_ws=True):
            g, w = timed_sequence(lambda r: run_step(r, ps=ps, use_ws=use_ws))
            fl = sum(step_flops(r, ps) for r in ratios[args.warmup:])
            return {"TFLOP/s": fl / (max(g, w) * 1e-3) / 1e12, "ms_per_step": max(g, w) / args.steps}
        secondary["no_scratch_buffer"] = dict(figure(projs, use_ws=False),
                                              what="headline layouts, activations gathered in flight by the tile loaders")
        kn = make_projs(col_layout="KN")
        secondary["kn_layout_drop_n"] = dict(figure(kn), what="column-parallel shards stored [K x N] (the kept list selects "
                                             "single elements of every stored row: element-gather loaders), with scratch")
        secondary["kn_layout_drop_n_no_scratch"] = dict(figure(kn, use_ws=False), what="the same without scratch")
        del kn
        lit = make_projs(col_layout="KN", col_mode=zr.DROP_K)
        by = {}
        base = None
        for r in cfg.ratios:
            run_step(r, ps=lit)
            ms = float(np.median(sample_steps(lambda: run_step(r, ps=lit), max(5, args.samples // 2))))
            base = base or ms
            fl = step_flops(r, lit)
            by[f"{r:.2f}"] = {"ms": ms, "tflops": fl / (ms * 1e-3) / 1e12, "speedup_vs_first": base / ms}
        secondary["paper_literal_drop_k_everywhere"] = {
            "what": "Sec. 3.1's worked example: the contraction (in-feature) axis is pruned on column-parallel shards "
                    "too (stored [K x N], scores = row norms), row-parallel shards as in the headline", "by_ratio": by}
        del lit
        pad = make_projs(pad=64)
        secondary["padded_leading_dimensions"] = dict(figure(pad), what="activations and their gradients with rows 64 elements "
                                                      "longer than the tensor (no 8 KB row stride), otherwise the headline path")
        del pad
        # the step as a captured graph, one graph per ratio (what is left of the host's launch cost)
        graphs = {}
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            for r in sorted(set(ratios)):
                run_step(r)
                side.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    run_step(r)
                graphs[r] = g
            side.synchronize()
            for r in ratios[:args.warmup]:
                graphs[r].replay()
            side.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            w0 = time.perf_counter()
            a.record(side)
            for r in ratios[args.warmup:]:
                graphs[r].replay()
            b.record(side)
            side.synchronize()
            gw = (time.perf_counter() - w0) * 1e3
        gms = max(a.elapsed_time(b), gw)
        secondary["hip_graph_replay"] = {"TFLOP/s": flops / (gms * 1e-3) / 1e12, "ms_per_step": gms / args.steps,
                                         "what": "the same seeded steps, each ratio's step captured once and replayed"}
        del graphs

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
    if not args.no_aux:
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
        # one long vector (2^24 scores, 64 MB): many workgroups with scratch against the single workgroup
        nl = 1 << 24
        sl = torch.randn(nl, dtype=torch.float32, device=dev)
        kl = torch.empty(nl, dtype=torch.int32, device=dev)
        dl = torch.empty(nl, dtype=torch.int32, device=dev)
        wsl = torch.empty(zr.select_workspace_bytes(nl), dtype=torch.uint8, device=dev)
        ms = timed(lambda: zr.resize_select_ws(sl, 0.25, wsl, keep_idx=kl, drop_idx=dl), n=10)
        ms1 = timed(lambda: zr.resize_select_ws(sl, 0.25, None, keep_idx=kl, drop_idx=dl), n=2)
        aux["select_large_n"] = {"n": nl, "ms": ms, "GB/s": 8.0 * nl / (ms * 1e-3) / 1e9,
                                 "frac_hbm_peak": 8.0 * nl / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                 "physical_GB/s": 28.0 * nl / (ms * 1e-3) / 1e9,
                                 "physical_frac_hbm_peak": 28.0 * nl / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                 "single_workgroup_ms": ms1,
                                 "bytes": "algorithmic: 4n read + 4n written; physical: the vector is read by six "
                                          "launches (four histograms, count, write) and the lists are written once"}
        del sl, kl, dl, wsl
        keep25, _ = zr.resize_select(p0["scores"], 0.25)
        buf = p0["Y"] if p0["mode"] == zr.DROP_N else p0["dX"]
        ncols = buf.shape[1]
        prev = torch.zeros_like(buf)
        esz = buf.element_size()
        dropped_bytes = esz * M * (ncols - keep25.numel())
        kept_bytes = esz * M * keep25.numel()
        whole = esz * M * ncols
        # physical bytes: the dropped columns are scattered 2-byte elements; at this ratio every
        # 32-byte sector of the tensor holds one, so the memory system moves the whole tensor
        for name, pol, nbytes, phys in (("zero", zr.ZERO, dropped_bytes, whole), ("same", zr.SAME, 2 * dropped_bytes, 2 * whole),
                                        ("average", zr.AVERAGE, kept_bytes + dropped_bytes, 2 * whole)):
            ms = timed(lambda pol=pol: zr.impute(buf, 1, keep25, pol, prev if pol == zr.SAME else None))
            aux[f"impute_{name}"] = {"shape": [M, ncols], "ratio": 0.25, "ms": ms, "GB/s": nbytes / (ms * 1e-3) / 1e9,
                                     "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                     "physical_GB/s": phys / (ms * 1e-3) / 1e9,
                                     "physical_frac_hbm_peak": phys / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
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

    # ---- CPU oracle on the host cores: bounded sample, and the check of the GPU's step ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle
        m_slice = min(M, 3072)          # about 15 s of float64 work on the 16 host threads of a GPU machine
        ratio = 0.25
        keeps = run_step(ratio)         # one more step of the timed path; its outputs are checked below
        torch.cuda.synchronize()
        work = 0.0
        secs = 0.0
        worst = {"Y": 0.0, "dX": 0.0}
        bad = 0
        for pi, (pr, p, keep) in enumerate(zip(cfg.projections, projs, keeps)):
            t = host[pi]["t"]
            Xs, dYs = t["X"][:m_slice], t["dY"][:m_slice]
            r = wl.ratio_for(cfg, pr, ratio)
            c0 = time.perf_counter()
            okeep, _ = oracle.resize_select(host[pi]["scores"], r)
            wantY = oracle.resized_linear_fwd(Xs, t["W"], okeep, pr.mode)
            wantdX, _ = oracle.resized_linear_bwd(Xs, t["W"], dYs, okeep, pr.mode)
            secs += time.perf_counter() - c0
            work += wl.kept_flops(m_slice, pr.K, pr.N, pr.n_axis, len(okeep))
            # the GPU's rows of the same tokens (dW sums over all tokens and is not comparable to a slice)
            bad += int(not np.array_equal(keep.cpu().numpy(), okeep))
            for name, got, want in (("Y", p["Y"], wantY), ("dX", p["dX"], wantdX)):
                g = got[:m_slice].float().cpu().numpy().astype(np.float64)
                err = float(np.linalg.norm(g - want) / np.linalg.norm(want))
                worst[name] = max(worst[name], err)
                # one rounding of the output type per element (+ a floor for results near zero)
                lim = 2.0 ** -8 * np.abs(want) * 1.001 + 2.0 ** -13 * float(np.sqrt(np.mean(want * want)))
                bad += int(np.count_nonzero(np.abs(g - want) > (lim if cfg.dtype == "bf16" else 1e-5 * np.max(np.abs(want)))))
        cpu = {"value": work / secs / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"{cfg.name}: all {len(cfg.projections)} projections, select+fwd+bwd at ratio {ratio}, "
                         f"the first {m_slice} tokens of the benchmark's own inputs, float64, {secs:.1f} s",
               "gpu_step_check": {"what": "kept lists bit-exact; Y and dX rows of those tokens from one more step of the timed "
                                          "path, element-wise within one output rounding of the oracle",
                                  "elements_out_of_bound": bad, "worst_rel_frobenius": worst, "ok": bad == 0}}
        if bad:
            print(f"bench.py: the GPU step does not match the oracle ({bad} elements / lists out of bound)", file=sys.stderr)

    step_bytes = sum(t.numel() * t.element_size() for p in projs for t in (p["X"], p["W"], p["dY"], p["Y"], p["dX"], p["dW"]))
    line = {
        "metric": "effective TFLOP/s (fwd+bwd) of resized TP shard GEMM vs resize ratio; % MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": total_ms / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: M={M} tokens, projections "
                               + ", ".join(f"{p.name}[{p.K}x{p.N}]{p.parallel}" for p in cfg.projections)
                               + "; per-step ratio drawn (seeded) from " + str(list(cfg.ratios)),
                   "path": f"resize_select_multi (one launch for the {len(cfg.projections)} projections) + resized_linear_fwd + resized_linear_bwd(dX,dW), Zero imputation, "
                           "with the optional scratch buffer for the extracted kept columns of activations (the backward call reuses "
                           "what the forward call of the same projection extracted); column-parallel shards "
                           "stored [N x K], row-parallel [K x N] (the kept list selects rows of the stored weight, no weight copy)",
                   "buffers": f"one step touches {step_bytes / 1e6:.0f} MB of distinct tensors, {step_bytes / 268.4e6:.1f}x the 256 MB "
                              "memory-side cache: " +
                              ("every tensor is evicted before its next use, so no buffer rotation is needed"
                               if step_bytes > 2 * 268.4e6 else
                               "about the size of that cache, so part of a step's inputs may still be resident from the step "
                               "before (buffers are not rotated; this workload is a parity case, not the headline)")},
        "frac_mfma_peak": value / peak,
        "gpu_ms_per_step": gpu_ms / args.steps, "wall_ms_per_step": wall_ms / args.steps,
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "extract": extract, "by_ratio": sweep,
        "secondary": secondary, "aux": aux,
    }
    print(json.dumps(line))
    return 0 if (cpu is None or cpu["gpu_step_check"]["ok"]) else 1


if __name__ == "__main__":
    sys.exit(main())
