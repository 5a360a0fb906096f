"""Parity at the full sizes of the workloads.  The oracle (float64 loops on the
host) computes sampled output rows / columns one by one; the whole tensors are
additionally checked, element by element at the kept positions, against the
masked-dense identity evaluated with an fp32 library GEMM on the GPU (a property
that holds at any size), and imputed positions bit-exactly.
test_full_size_projection: one projection at a time through zr_resize_select.
test_bench_path_*: exactly what bench.py times: one zr_resize_select_multi launch
for the shard's projections, forward, then backward with the scratch buffer still
holding what the forward extracted (ZR_WS_HOLDS_FORWARD), over every ratio of the
workload.  test_big_tile_*: the options that small shapes never take to the
256-wide tiles (Average / Same, no scratch, element-gather layout, accumulate)."""
import numpy as np
import pytest

from paper_2401_11469_amd import workloads as wl

pytestmark = pytest.mark.gpu

DROP_N, DROP_K = 0, 1
TOL = {"f32": 1e-5, "bf16": 2e-2}
N_SAMPLE = 96


@pytest.fixture(scope="module")
def zr():
    import torch
    assert torch.cuda.is_available()
    from paper_2401_11469_amd import zr as binding
    binding.debug_record_kernel_names(True)     # tests assert which kernel instantiation ran
    return binding


from parity_util import check_kept_np, check_kept_torch, relf  # noqa: E402


def _np64(t):
    return t.float().cpu().numpy().astype(np.float64)


def _check_projection(zr, oracle, cid, pi, ratio):
    import torch
    cfg = wl.CONFIGS[cid]
    pr = cfg.projections[pi]
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    tol = TOL[cfg.dtype]
    t = wl.make_tensors(cid, pi)
    Xh, Wh, dYh = t["X"], t["W"], t["dY"]
    M, K, N = Xh.shape[0], pr.K, pr.N
    scores = wl.make_scores(cid, pi, Wh)
    r = wl.ratio_for(cfg, pr, ratio)
    mode, n = pr.mode, pr.n_axis

    X, W, dY = (torch.from_numpy(a).to(tdt).cuda() for a in (Xh, Wh, dYh))
    # as bench.py stores the shards: column-parallel (DROP_N) ones [N x K], so that the
    # kept list selects rows of the stored weight in both modes
    nk = mode == DROP_N
    layout = 1 if nk else 0
    Wdev = W.t().contiguous() if nk else W
    keep, drop = zr.resize_select(torch.from_numpy(scores).cuda(), r)
    S, P = oracle.resize_select(scores, r)
    assert np.array_equal(keep.cpu().numpy(), S) and np.array_equal(drop.cpu().numpy(), P)   # bit-exact
    assert len(S) == oracle.keep_count(n, r)

    Y = torch.full((M, N), 3.0, dtype=tdt, device="cuda")
    dX = torch.full((M, K), 3.0, dtype=tdt, device="cuda")
    dW = torch.full((N, K) if nk else (K, N), 3.0, dtype=tdt, device="cuda")
    # as bench.py launches it: with the optional scratch buffer
    ws = torch.empty(max(16, zr.workspace_bytes(M, K, N, len(S), mode, tdt)), dtype=torch.uint8, device="cuda")
    zr.resized_linear_fwd(X, Wdev, keep, mode, Y=Y, workspace=ws, w_layout=layout)
    zr.resized_linear_bwd(X, Wdev, dY, keep, mode, dX=dX, dW=dW, workspace=ws, w_layout=layout)
    torch.cuda.synchronize()
    if nk:
        dW = dW.t()          # a [K x N] view for the checks below

    # (1) whole tensors: masked-dense identity with a library GEMM in fp32
    mask = torch.zeros(n, dtype=torch.float32, device="cuda")
    mask[keep.long()] = 1.0
    Xf, Wf, dYf = X.float(), W.float(), dY.float()
    torch.backends.cuda.matmul.allow_tf32 = False
    if mode == DROP_K:
        Xm, Wm = Xf * mask[None, :], Wf * mask[:, None]
        refs = (Xm @ Wm, (dYf @ Wm.T) * mask[None, :], (Xm.T @ dYf) * mask[:, None])
    else:
        Wm, dYm = Wf * mask[None, :], dYf * mask[None, :]
        refs = ((Xf @ Wm) * mask[None, :], dYm @ Wm.T, (Xf.T @ dYm) * mask[None, :])
    keptb = mask > 0
    if mode == DROP_K:
        where, terms = (None, keptb[None, :], keptb[:, None]), (len(S), N, M)
    else:
        where, terms = (keptb[None, :], None, keptb[None, :]), (K, len(S), M)
    for name, got, ref, wh, C in zip(("Y", "dX", "dW"), (Y, dX, dW), refs, where, terms):
        assert torch.isfinite(got).all(), name
        err = (torch.linalg.norm(got.float() - ref) / torch.linalg.norm(ref)).item()
        assert err <= tol, (cid, pr.name, ratio, name, err)
        # every kept element within one rounding of the output type (+ fp32 accumulation)
        e = check_kept_torch(f"config {cid} {pr.name} r={ratio} {name}", got, ref, cfg.dtype, C, wh)
        print(f"  {name}: relative Frobenius error {e:.2e}", flush=True)
    del Xf, Wf, dYf, refs

    # (2) imputed positions are exactly +0.0
    if len(P):
        Pi = drop.long()
        zs = (dX[:, Pi], dW[Pi, :]) if mode == DROP_K else (Y[:, Pi], dW[:, Pi])
        for z in zs:
            assert torch.all(z == 0) and not torch.any(torch.signbit(z))

    # (3) sampled rows / columns against the oracle
    g = np.random.Generator(np.random.PCG64(cid * 100 + pi))
    rows = np.sort(g.choice(M, size=min(N_SAMPLE, M), replace=False))
    wantY = oracle.resized_linear_fwd(Xh[rows], Wh, S, mode)
    wantdX, _ = oracle.resized_linear_bwd(Xh[rows], Wh, dYh[rows], S, mode)
    ridx = torch.from_numpy(rows).cuda()
    eY, edX = relf(_np64(Y[ridx]), wantY), relf(_np64(dX[ridx]), wantdX)
    assert eY <= tol and edX <= tol, (cid, pr.name, ratio, eY, edX)
    kept_np = np.zeros(n, dtype=bool)
    kept_np[S] = True
    check_kept_np("Y rows", _np64(Y[ridx]), wantY, cfg.dtype, terms[0], kept_np[None, :] if mode == DROP_N else None)
    check_kept_np("dX rows", _np64(dX[ridx]), wantdX, cfg.dtype, terms[1], kept_np[None, :] if mode == DROP_K else None)
    # dW contracts over all tokens: sample along the axis that is NOT pruned
    if mode == DROP_K:
        cols = np.sort(g.choice(N, size=min(N_SAMPLE, N), replace=False))
        _, want = oracle.resized_linear_bwd(Xh, Wh[:, cols], dYh[:, cols], S, mode)
        got = _np64(dW[:, torch.from_numpy(cols).cuda()])
    else:
        ks = np.sort(g.choice(K, size=min(N_SAMPLE, K), replace=False))
        _, want = oracle.resized_linear_bwd(Xh[:, ks], Wh[ks, :], dYh, S, mode)
        got = _np64(dW[torch.from_numpy(ks).cuda(), :])
    edW = relf(got, want)
    assert edW <= tol, (cid, pr.name, ratio, edW)
    check_kept_np("dW slice", got, want, cfg.dtype, M, kept_np[:, None] if mode == DROP_K else kept_np[None, :])


def _cases():
    out = []
    picks = {2: (0.0, 0.1, 0.5), 3: (0.0, 0.4), 4: (0.0, 0.15, 0.5), 5: (0.3,)}
    for cid, ratios in picks.items():
        for pi in range(len(wl.CONFIGS[cid].projections)):
            for r in ratios:
                out.append((cid, pi, r))
    return out


@pytest.mark.parametrize("cid,pi,ratio", _cases())
def test_full_size_projection(zr, oracle, cid, pi, ratio):
    print(f"config {cid} projection {wl.CONFIGS[cid].projections[pi].name} ratio {ratio}", flush=True)
    _check_projection(zr, oracle, cid, pi, ratio)


# ---------------------------------------------------------------------------
# The launch configuration bench.py times, ratio by ratio
# ---------------------------------------------------------------------------

class _Shard:
    """Device tensors of one workload's layer shard, laid out as bench.py lays them out."""

    def __init__(self, zr, cid, only=None, layouts=None):
        import torch
        self.torch, self.zr, self.cid = torch, zr, cid
        self.cfg = cfg = wl.CONFIGS[cid]
        self.tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        self.M = cfg.M
        self.projs = []
        for pi, pr in enumerate(cfg.projections):
            if only is not None and pr.name not in only:
                continue
            t = wl.make_tensors(cid, pi)
            nk = pr.mode == DROP_N
            if layouts and pr.name in layouts:
                nk = layouts[pr.name] == "NK"
            W = torch.from_numpy(t["W"]).to(self.tdt).cuda()
            self.projs.append(dict(
                pi=pi, pr=pr, n=pr.n_axis, nk=nk, layout=1 if nk else 0, host=t,
                scores_h=wl.make_scores(cid, pi, t["W"]),
                X=torch.from_numpy(t["X"]).to(self.tdt).cuda(), W=W,
                Wdev=W.t().contiguous() if nk else W,
                dY=torch.from_numpy(t["dY"]).to(self.tdt).cuda(),
                Y=torch.empty((self.M, pr.N), dtype=self.tdt, device="cuda"),
                dX=torch.empty((self.M, pr.K), dtype=self.tdt, device="cuda"),
                dW=torch.empty((pr.N, pr.K) if nk else (pr.K, pr.N), dtype=self.tdt, device="cuda")))
        for p in self.projs:
            p["scores"] = torch.from_numpy(p["scores_h"]).cuda()
        nbytes = max(zr.workspace_bytes(self.M, p["pr"].K, p["pr"].N, p["n"], p["pr"].mode, self.tdt) for p in self.projs)
        self.ws = torch.empty(max(16, nbytes), dtype=torch.uint8, device="cuda")

    def step(self, ratio, use_ws=True, holds_forward=True):
        """select (one launch for all projections) + forward + backward; returns the kept lists."""
        zr, cfg = self.zr, self.cfg
        for p in self.projs:
            for k in ("Y", "dX", "dW"):
                p[k].fill_(3.0)
        keeps, drops = zr.resize_select_multi([p["scores"] for p in self.projs],
                                              [wl.ratio_for(cfg, p["pr"], ratio) for p in self.projs])
        ws = self.ws if use_ws else None
        for p, keep in zip(self.projs, keeps):
            pr = p["pr"]
            zr.resized_linear_fwd(p["X"], p["Wdev"], keep, pr.mode, Y=p["Y"], workspace=ws, w_layout=p["layout"])
            p["kernels"] = [zr.debug_last_kernel()]
            zr.resized_linear_bwd(p["X"], p["Wdev"], p["dY"], keep, pr.mode, dX=p["dX"], dW=p["dW"], workspace=ws,
                                  w_layout=p["layout"], workspace_holds_forward=holds_forward and use_ws)
            p["kernels"].append(zr.debug_last_kernel())
        self.torch.cuda.synchronize()
        return keeps, drops

    def check(self, oracle, p, keep, drop, ratio, rows=48):
        """Whole tensors element by element against the masked-dense identity, imputed zeros,
        and sampled rows against the oracle."""
        torch, cfg = self.torch, self.cfg
        pr, n, mode, M = p["pr"], p["n"], p["pr"].mode, self.M
        K, N = pr.K, pr.N
        r = wl.ratio_for(cfg, pr, ratio)
        S, P = oracle.resize_select(p["scores_h"], r)
        assert np.array_equal(keep.cpu().numpy(), S) and np.array_equal(drop.cpu().numpy(), P)
        mask = torch.zeros(n, dtype=torch.float32, device="cuda")
        mask[keep.long()] = 1.0
        keptb = mask > 0
        Xf, Wf, dYf = p["X"].float(), p["W"].float(), p["dY"].float()
        torch.backends.cuda.matmul.allow_tf32 = False
        dW = p["dW"].t() if p["nk"] else p["dW"]
        tag = f"config {self.cid} {pr.name} r={ratio}"
        if mode == DROP_K:
            Xm, Wm = Xf * mask[None, :], Wf * mask[:, None]
            checks = (("Y", p["Y"], lambda: Xm @ Wm, None, len(S)),
                      ("dX", p["dX"], lambda: (dYf @ Wm.T) * mask[None, :], keptb[None, :], N),
                      ("dW", dW, lambda: (Xm.T @ dYf) * mask[:, None], keptb[:, None], M))
        else:
            Wm, dYm = Wf * mask[None, :], dYf * mask[None, :]
            checks = (("Y", p["Y"], lambda: (Xf @ Wm) * mask[None, :], keptb[None, :], K),
                      ("dX", p["dX"], lambda: dYm @ Wm.T, None, len(S)),
                      ("dW", dW, lambda: (Xf.T @ dYm) * mask[None, :], keptb[None, :], M))
        for name, got, ref_fn, wh, C in checks:
            ref = ref_fn()
            check_kept_torch(f"{tag} {name}", got, ref, cfg.dtype, C, wh)
            del ref
        if len(P):
            Pi = drop.long()
            zs = (p["dX"][:, Pi], dW[Pi, :]) if mode == DROP_K else (p["Y"][:, Pi], dW[:, Pi])
            for z in zs:
                assert torch.all(z == 0) and not torch.any(torch.signbit(z)), tag
        g = np.random.Generator(np.random.PCG64(self.cid * 1000 + p["pi"] * 10 + int(ratio * 100)))
        ridx = np.sort(g.choice(M, size=rows, replace=False))
        h = p["host"]
        wantY = oracle.resized_linear_fwd(h["X"][ridx], h["W"], S, mode)
        wantdX, _ = oracle.resized_linear_bwd(h["X"][ridx], h["W"], h["dY"][ridx], S, mode)
        rg = torch.from_numpy(ridx).cuda()
        kept_np = np.zeros(n, dtype=bool)
        kept_np[S] = True
        check_kept_np(f"{tag} Y rows", _np64(p["Y"][rg]), wantY, cfg.dtype, K if mode == DROP_N else len(S),
                      kept_np[None, :] if mode == DROP_N else None)
        check_kept_np(f"{tag} dX rows", _np64(p["dX"][rg]), wantdX, cfg.dtype, N if mode == DROP_K else len(S),
                      kept_np[None, :] if mode == DROP_K else None)


def test_bench_path_every_ratio_of_the_llama_7b_shard(zr, oracle):
    """Config 4 as bench.py runs it (select_multi for the 5 projections, scratch buffer reused by
    the backward call), every ratio of its list; one column-parallel (qkv) and one row-parallel
    (down) projection are checked in full at every ratio, the other three at three ratios."""
    sh = _Shard(zr, 4)
    cfg = sh.cfg
    for ratio in cfg.ratios:
        print(f"bench path, config 4, ratio {ratio}", flush=True)
        keeps, drops = sh.step(ratio)
        for p, keep, drop in zip(sh.projs, keeps, drops):
            full = p["pr"].name in ("qkv", "down") or ratio in (0.0, 0.05, 0.5)
            if full:
                sh.check(oracle, p, keep, drop, ratio)
            assert p["kernels"][0].startswith("fast_kernel") and p["kernels"][1].startswith("fast_kernel"), p["kernels"]


def test_bench_path_other_workloads(zr, oracle):
    """Configs 2, 3 and 5 through the same calls as bench.py, every ratio of their lists."""
    for cid in (2, 3, 5):
        sh = _Shard(zr, cid)
        for ratio in sh.cfg.ratios:
            print(f"bench path, config {cid}, ratio {ratio}", flush=True)
            keeps, drops = sh.step(ratio)
            for p, keep, drop in zip(sh.projs, keeps, drops):
                sh.check(oracle, p, keep, drop, ratio, rows=24)
        del sh


def test_full_size_element_gather_layout(zr, oracle):
    """The layout the workload descriptions write ([K x N] weight, output features pruned): the kept
    list selects single elements of every stored row, the in-flight gather loaders run on the big
    tiles; with and without the scratch buffer."""
    sh = _Shard(zr, 4, only=("qkv", "gate"), layouts={"qkv": "KN", "gate": "KN"})
    for ratio, use_ws in ((0.15, True), (0.35, False)):
        print(f"KN x DROP_N, ratio {ratio}, scratch {use_ws}", flush=True)
        keeps, drops = sh.step(ratio, use_ws=use_ws)
        for p, keep, drop in zip(sh.projs, keeps, drops):
            sh.check(oracle, p, keep, drop, ratio)
            print("   ", p["pr"].name, p["kernels"], flush=True)


def test_big_tile_no_scratch(zr, oracle):
    """Row-gather layouts without the scratch buffer: the activations are gathered in flight."""
    sh = _Shard(zr, 4, only=("qkv", "down"))
    keeps, drops = sh.step(0.15, use_ws=False)
    for p, keep, drop in zip(sh.projs, keeps, drops):
        sh.check(oracle, p, keep, drop, 0.15)
        print("   ", p["pr"].name, p["kernels"], flush=True)


@pytest.mark.parametrize("name", ["qkv", "down"])
@pytest.mark.parametrize("policy", ["average", "same", "same_in_place"])
def test_big_tile_other_policies(zr, oracle, name, policy):
    """Average and Same imputation through the epilogues of the 256-wide tiles (sums continued
    across the big panel and the remainder panel; previous tensor read by the scatter epilogue)."""
    import torch
    sh = _Shard(zr, 4, only=(name,))
    p = sh.projs[0]
    pr, mode, M, n = p["pr"], p["pr"].mode, sh.M, p["n"]
    K, N = pr.K, pr.N
    ratio = 0.15
    keep, drop = zr.resize_select(p["scores"], ratio)
    S, P = oracle.resize_select(p["scores_h"], ratio)
    assert np.array_equal(keep.cpu().numpy(), S)
    pol = zr.AVERAGE if policy == "average" else zr.SAME
    g = torch.Generator(device="cuda").manual_seed(5)
    outs = {k: p[k] for k in ("Y", "dX", "dW")}
    prevs = {}
    for k, t in outs.items():
        prev = torch.randn(t.shape, generator=g, device="cuda", dtype=torch.float32).to(sh.tdt)
        if policy == "same_in_place":
            t.copy_(prev)              # the output already holds the previous iteration's values
            prevs[k] = t
        else:
            t.fill_(3.0)
            prevs[k] = prev if policy == "same" else None
    keep_prev = {k: (v.clone() if v is not None else None) for k, v in prevs.items()}
    zr.resized_linear_fwd(p["X"], p["Wdev"], keep, mode, pol, prevs["Y"], Y=p["Y"], workspace=sh.ws, w_layout=p["layout"])
    k1 = zr.debug_last_kernel()
    zr.resized_linear_bwd(p["X"], p["Wdev"], p["dY"], keep, mode, pol, prevs["dX"], prevs["dW"], dX=p["dX"], dW=p["dW"],
                          workspace=sh.ws, w_layout=p["layout"], workspace_holds_forward=True)
    k2 = zr.debug_last_kernel()
    torch.cuda.synchronize()
    print("   ", name, policy, k1, "|", k2, flush=True)
    assert ("256" in k1 or "192" in k1) and ("256" in k2 or "192" in k2), (k1, k2)
    # kept positions: masked-dense identity; imputed positions: the policy's definition evaluated
    # on the stored kept values (Average) or the previous tensor's bits (Same)
    mask = torch.zeros(n, dtype=torch.float32, device="cuda")
    mask[keep.long()] = 1.0
    keptb = mask > 0
    Xf, Wf, dYf = p["X"].float(), p["W"].float(), p["dY"].float()
    dW = p["dW"].t() if p["nk"] else p["dW"]
    pdW = None if keep_prev["dW"] is None else (keep_prev["dW"].t() if p["nk"] else keep_prev["dW"])
    if mode == DROP_K:
        Xm, Wm = Xf * mask[None, :], Wf * mask[:, None]
        items = (("Y", p["Y"], Xm @ Wm, None, None, len(S), None),
                 ("dX", p["dX"], dYf @ Wm.T, keptb[None, :], 1, N, keep_prev["dX"]),
                 ("dW", dW, Xm.T @ dYf, keptb[:, None], 0, M, pdW))
    else:
        Wm, dYm = Wf * mask[None, :], dYf * mask[None, :]
        items = (("Y", p["Y"], Xf @ Wm, keptb[None, :], 1, K, keep_prev["Y"]),
                 ("dX", p["dX"], dYm @ Wm.T, None, None, len(S), None),
                 ("dW", dW, Xf.T @ dYm, keptb[None, :], 1, M, pdW))
    Pi, Si = drop.long(), keep.long()
    for nm, got, ref, wh, axis, C, prev in items:
        check_kept_torch(f"{name} {policy} {nm}", got, ref, sh.cfg.dtype, C, wh)
        if axis is None:
            continue
        gf = got.float()
        if policy == "average":
            if axis == 1:
                mean = gf[:, Si].mean(dim=1, keepdim=True)
                imp, whole = gf[:, Pi], mean.expand(-1, len(P))
            else:
                mean = gf[Si, :].mean(dim=0, keepdim=True)
                imp, whole = gf[Pi, :], mean.expand(len(P), -1)
            # one rounding of the fp32 mean of the stored kept values to the output type
            tol_abs = 2.0 ** -8 * float(gf.abs().max().item())
            assert float((imp - whole).abs().max().item()) <= tol_abs, (nm, "average")
        else:
            ip = got[:, Pi] if axis == 1 else got[Pi, :]
            pp = prev[:, Pi] if axis == 1 else prev[Pi, :]
            assert torch.equal(ip, pp), (nm, "same: dropped positions must hold the previous tensor's bits")
    # sampled rows against the oracle with the policy applied
    rows = np.sort(np.random.Generator(np.random.PCG64(77)).choice(M, size=32, replace=False))
    rg = torch.from_numpy(rows).cuda()
    h = p["host"]
    opol = {"average": 1, "same": 2, "same_in_place": 2}[policy]
    pY = None if keep_prev["Y"] is None else _np64(keep_prev["Y"][rg])
    pdX = None if keep_prev["dX"] is None else _np64(keep_prev["dX"][rg])
    wantY = oracle.resized_linear_fwd(h["X"][rows], h["W"], S, mode, opol, pY)
    kept_np = np.zeros(n, dtype=bool)
    kept_np[S] = True
    check_kept_np("Y rows", _np64(p["Y"][rg]), wantY, sh.cfg.dtype, K if mode == DROP_N else len(S),
                  kept_np[None, :] if mode == DROP_N else None)
    if mode == DROP_N and len(P):
        gotP, wantP = _np64(p["Y"][rg])[:, P], wantY[:, P]
        if opol == 2:
            assert np.array_equal(gotP, wantP)
        else:
            assert np.max(np.abs(gotP - wantP)) <= 2.0 ** -8 * np.max(np.abs(wantY))


def test_big_tile_migrated_accumulate(zr, oracle):
    """out += A B on the 256-wide tiles (M = 8192): accumulators seeded from the old output."""
    import torch
    g = np.random.Generator(np.random.PCG64(91))
    M, N, C = 8192, 4096, 688
    A = wl.round_to_bf16(g.standard_normal((M, C)).astype(np.float32))
    for transposed in (False, True):
        B = wl.round_to_bf16((g.standard_normal((N, C) if transposed else (C, N)) * 0.05).astype(np.float32))
        base = wl.round_to_bf16(g.standard_normal((M, N)).astype(np.float32))
        Ag, Bg = torch.from_numpy(A).bfloat16().cuda(), torch.from_numpy(B).bfloat16().cuda()
        out = torch.from_numpy(base).bfloat16().cuda()
        zr.migrated_accumulate(out, Ag, Bg, transposed)
        kn = zr.debug_last_kernel()
        torch.cuda.synchronize()
        print("   accumulate", transposed, kn, flush=True)
        assert "256" in kn, kn
        ref = torch.from_numpy(base).cuda() + Ag.float() @ (Bg.float().T if transposed else Bg.float())
        check_kept_torch(f"accumulate transposed={transposed}", out, ref, "bf16", C)
        rows = np.sort(g.choice(M, size=24, replace=False))
        want = oracle.migrated_accumulate(base[rows], A[rows], B, transposed)
        check_kept_np("accumulate rows", _np64(out[torch.from_numpy(rows).cuda()]), want, "bf16", C)


def test_big_tile_row_list_too_long_for_lds(zr):
    """A row list on the contraction axis with more entries than the ring loop keeps in LDS (6144):
    the product stays on 256 x 256 tiles but runs the 64-deep loop, which looks the list up as it goes."""
    import torch
    torch.manual_seed(11)
    M, K, N = 4096, 8192, 4096
    X = torch.randn(M, K, device="cuda", dtype=torch.bfloat16)
    W = (torch.randn(K, N, device="cuda") * 0.02).to(torch.bfloat16)
    keep = torch.sort(torch.randperm(K, device="cuda")[:zr.keep_count(K, 0.1)]).values.to(torch.int32)
    assert keep.numel() > 6144
    ws = torch.empty(zr.workspace_bytes(M, K, N, keep.numel(), DROP_K, torch.bfloat16), dtype=torch.uint8, device="cuda")
    Y = torch.full((M, N), 3.0, device="cuda", dtype=torch.bfloat16)
    zr.resized_linear_fwd(X, W, keep, DROP_K, Y=Y, workspace=ws, w_layout=0)
    torch.cuda.synchronize()
    assert zr.debug_last_kernel() == "fast_kernel<DmaP, DmaQM, 256, 256, 2, 4>", zr.debug_last_kernel()
    mask = torch.zeros(K, dtype=torch.float32, device="cuda")
    mask[keep.long()] = 1.0
    torch.backends.cuda.matmul.allow_tf32 = False
    ref = (X.float() * mask[None, :]) @ (W.float() * mask[:, None])
    check_kept_torch("long row list Y", Y, ref, "bf16", keep.numel(), None)
    # one more kept index than the ring loop's limit, and exactly the limit (which takes the ring loop)
    for nk, name in ((6145, "fast_kernel<DmaP, DmaQM, 256, 256, 2, 4>"), (6144, "fast_kernel<RingP, RingQM, 256, 256, 2, 4>")):
        kp = keep[:nk].contiguous()
        zr.resized_linear_fwd(X, W, kp, DROP_K, Y=Y, workspace=ws, w_layout=0)
        torch.cuda.synchronize()
        assert zr.debug_last_kernel() == name, (nk, zr.debug_last_kernel())
        mask.zero_()
        mask[kp.long()] = 1.0
        ref = (X.float() * mask[None, :]) @ (W.float() * mask[:, None])
        check_kept_torch(f"row list of {nk}", Y, ref, "bf16", nk, None)


def test_full_size_step_in_a_captured_graph(zr):
    """One layer step of the Llama-2-7B shard (big ring tiles, remainder panels, split contractions,
    extraction reuse) captured once and replayed with new priorities each time; every replay, with
    eager work and synchronisations in between, equals the same step run eagerly bit by bit."""
    import torch
    sh = _Shard(zr, 4, only=("qkv", "out", "down"))
    ratio = 0.25
    kb = [torch.empty(p["n"], dtype=torch.int32, device="cuda") for p in sh.projs]
    db = [torch.empty(p["n"], dtype=torch.int32, device="cuda") for p in sh.projs]

    def step():
        keeps, _ = zr.resize_select_multi([p["scores"] for p in sh.projs],
                                          [wl.ratio_for(sh.cfg, p["pr"], ratio) for p in sh.projs], keep_idx=kb, drop_idx=db)
        for p, keep in zip(sh.projs, keeps):
            pr = p["pr"]
            zr.resized_linear_fwd(p["X"], p["Wdev"], keep, pr.mode, Y=p["Y"], workspace=sh.ws, w_layout=p["layout"])
            zr.resized_linear_bwd(p["X"], p["Wdev"], p["dY"], keep, pr.mode, dX=p["dX"], dW=p["dW"], workspace=sh.ws,
                                  w_layout=p["layout"], workspace_holds_forward=True)
        return keeps

    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        keeps = step()
    g = np.random.Generator(np.random.PCG64(17))
    for rep in range(3):
        for p in sh.projs:
            p["scores"].copy_(torch.from_numpy(g.random(p["n"]).astype(np.float32)).cuda())
            for k in ("Y", "dX", "dW"):
                p[k].fill_(7.0)
        sh.ws.fill_(0x5a)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [[p[k].clone() for k in ("Y", "dX", "dW")] for p in sh.projs] + [[k.clone() for k in keeps]]
        for p in sh.projs:
            for k in ("Y", "dX", "dW"):
                p[k].fill_(9.0)
        sh.ws.fill_(0xa5)
        step()
        torch.cuda.synchronize()
        want = [[p[k] for k in ("Y", "dX", "dW")] for p in sh.projs] + [list(keeps)]
        for a, b in zip(got, want):
            for x, y in zip(a, b):
                assert torch.equal(x, y), rep
        for p in sh.projs:
            for k in ("Y", "dX", "dW"):
                assert torch.isfinite(p[k].float()).all()


@pytest.mark.parametrize("seed", range(10))
def test_random_large_ragged_shapes(zr, seed):
    """Shapes the workloads do not have: every extent ragged (multiples of 8 only), large enough for the
    schedule to cut big-tile panels and remainder panels along rows or columns; forward, dX and dW of both
    modes in the row-selecting layouts, with the scratch buffer; whole tensors element-wise against the
    masked-dense identity (fp32 library GEMM), imputed positions exact."""
    import torch
    g = np.random.Generator(np.random.PCG64(4000 + seed))
    M = int(g.integers(190, 800)) * 8
    K = int(g.integers(150, 560)) * 8
    N = int(g.integers(150, 560)) * 8
    mode = DROP_N if seed % 2 == 0 else DROP_K
    ratio = float(g.choice([0.05, 0.15, 0.25, 0.35, 0.5]))
    n = N if mode == DROP_N else K
    nk = mode == DROP_N                                   # column-parallel shards are stored [N x K]
    torch.manual_seed(seed)
    X = torch.randn(M, K, device="cuda", dtype=torch.bfloat16)
    W = (torch.randn(K, N, device="cuda") * 0.02).to(torch.bfloat16)
    dY = torch.randn(M, N, device="cuda", dtype=torch.bfloat16)
    Wdev = W.t().contiguous() if nk else W
    keep = torch.sort(torch.randperm(n, device="cuda")[:zr.keep_count(n, ratio)]).values.to(torch.int32)
    ws = torch.empty(zr.workspace_bytes(M, K, N, keep.numel(), mode, torch.bfloat16), dtype=torch.uint8, device="cuda")
    Y = torch.full((M, N), 3.0, device="cuda", dtype=torch.bfloat16)
    dX = torch.full((M, K), 3.0, device="cuda", dtype=torch.bfloat16)
    dW = torch.full((N, K) if nk else (K, N), 3.0, device="cuda", dtype=torch.bfloat16)
    kernels = []
    zr.resized_linear_fwd(X, Wdev, keep, mode, Y=Y, workspace=ws, w_layout=1 if nk else 0)
    kernels.append(zr.debug_last_kernel())
    zr.resized_linear_bwd(X, Wdev, dY, keep, mode, dX=dX, need_dW=False, workspace=ws, w_layout=1 if nk else 0,
                          workspace_holds_forward=True)
    kernels.append(zr.debug_last_kernel())
    zr.resized_linear_bwd(X, Wdev, dY, keep, mode, dW=dW, need_dX=False, workspace=ws, w_layout=1 if nk else 0,
                          workspace_holds_forward=mode == DROP_K)
    kernels.append(zr.debug_last_kernel())
    torch.cuda.synchronize()
    print(f"M={M} K={K} N={N} mode={mode} ratio={ratio}: {kernels}", flush=True)
    mask = torch.zeros(n, dtype=torch.float32, device="cuda")
    mask[keep.long()] = 1.0
    keptb = mask > 0
    Xf, Wf, dYf = X.float(), W.float(), dY.float()
    torch.backends.cuda.matmul.allow_tf32 = False
    dWkn = dW.t() if nk else dW
    tag = f"seed {seed}"
    if mode == DROP_K:
        Xm, Wm = Xf * mask[None, :], Wf * mask[:, None]
        checks = (("Y", Y, Xm @ Wm, None, keep.numel()),
                  ("dX", dX, (dYf @ Wm.T) * mask[None, :], keptb[None, :], N),
                  ("dW", dWkn, (Xm.T @ dYf) * mask[:, None], keptb[:, None], M))
        zs = (dX[:, ~keptb], dWkn[~keptb, :])
    else:
        Wm, dYm = Wf * mask[None, :], dYf * mask[None, :]
        checks = (("Y", Y, (Xf @ Wm) * mask[None, :], keptb[None, :], K),
                  ("dX", dX, dYm @ Wm.T, None, keep.numel()),
                  ("dW", dWkn, (Xf.T @ dYm) * mask[None, :], keptb[None, :], M))
        zs = (Y[:, ~keptb], dWkn[:, ~keptb])
    for name, got, ref, wh, C in checks:
        check_kept_torch(f"{tag} {name}", got, ref, "bf16", C, wh)
    for z in zs:
        assert torch.all(z == 0) and not torch.any(torch.signbit(z)), tag


def test_tensors_of_more_than_2_31_elements(zr):
    """Activations of 266240 x 8192 elements (2.18e9, 4.4 GB in bf16): every row offset of the loaders,
    the extraction and the epilogues has to be computed in 64 bits.  Rows from both ends of Y and dX and
    the whole dW against fp32 library products of the same (masked) operands."""
    import torch
    M, K, N = 266240, 8192, 256
    assert M * K > 2 ** 31
    torch.manual_seed(3)
    X = torch.empty(M, K, device="cuda", dtype=torch.bfloat16).normal_()
    W = (torch.randn(K, N, device="cuda") * 0.02).to(torch.bfloat16)
    dY = torch.randn(M, N, device="cuda", dtype=torch.bfloat16)
    keep = torch.sort(torch.randperm(K, device="cuda")[:zr.keep_count(K, 0.25)]).values.to(torch.int32)
    ws = torch.empty(zr.workspace_bytes(M, K, N, keep.numel(), DROP_K, torch.bfloat16), dtype=torch.uint8, device="cuda")
    Y = torch.full((M, N), 3.0, device="cuda", dtype=torch.bfloat16)
    dX = torch.full((M, K), 3.0, device="cuda", dtype=torch.bfloat16)
    dW = torch.full((K, N), 3.0, device="cuda", dtype=torch.bfloat16)
    zr.resized_linear_fwd(X, W, keep, DROP_K, Y=Y, workspace=ws, w_layout=0)
    k_fwd = zr.debug_last_kernel()
    zr.resized_linear_bwd(X, W, dY, keep, DROP_K, dX=dX, dW=dW, workspace=ws, w_layout=0, workspace_holds_forward=True)
    torch.cuda.synchronize()
    print(k_fwd, "|", zr.debug_last_kernel(), flush=True)
    kl = keep.long()
    mask = torch.zeros(K, dtype=torch.float32, device="cuda")
    mask[kl] = 1.0
    keptb = mask > 0
    torch.backends.cuda.matmul.allow_tf32 = False
    Wm = W.float() * mask[:, None]
    rows = torch.cat([torch.arange(0, 300, device="cuda"), torch.arange(M // 2 - 150, M // 2 + 150, device="cuda"),
                      torch.arange(M - 300, M, device="cuda")])
    Xr, dYr = X[rows].float(), dY[rows].float()
    check_kept_torch("Y rows", Y[rows], (Xr * mask[None, :]) @ Wm, "bf16", keep.numel(), None)
    check_kept_torch("dX rows", dX[rows], (dYr @ Wm.T) * mask[None, :], "bf16", N, keptb[None, :])
    assert torch.all(dX[rows][:, ~keptb] == 0)
    # dW = X[:,S]^T dY over all tokens, accumulated in fp32 in chunks of rows
    ref = torch.zeros(K, N, dtype=torch.float32, device="cuda")
    for r0 in range(0, M, 32768):
        ref += X[r0:r0 + 32768].float().T @ dY[r0:r0 + 32768].float()
    ref *= mask[:, None]
    check_kept_torch("dW", dW, ref, "bf16", M, keptb[:, None])
    assert torch.all(dW[~keptb, :] == 0)
