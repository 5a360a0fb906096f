"""Parity at the full sizes of the workloads, in the launch configuration
bench.py times.  The oracle (float64 loops on the host) computes sampled
output rows / columns one by one; the whole tensors are additionally checked
against the masked-dense identity evaluated with an fp32 library GEMM on the
GPU (a property that holds at any size), and imputed positions bit-exactly."""
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
    return binding


def relf(got, want):
    den = np.linalg.norm(want)
    return np.linalg.norm(got - want) / (den if den > 0 else 1.0)


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
    for name, got, ref in zip(("Y", "dX", "dW"), (Y, dX, dW), refs):
        assert torch.isfinite(got).all(), name
        err = (torch.linalg.norm(got.float() - ref) / torch.linalg.norm(ref)).item()
        assert err <= tol, (cid, pr.name, ratio, name, err)
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
