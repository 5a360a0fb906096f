"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Index work is bit-exact; floating point is
compared with the relative Frobenius error: <= 1e-5 for fp32, <= 2e-2 for bf16
inputs with fp32 accumulation; imputed positions are bit-exact."""
import numpy as np
import pytest

from paper_2401_11469_amd import workloads as wl

pytestmark = pytest.mark.gpu

DROP_N, DROP_K = 0, 1
ZERO, AVERAGE, SAME = 0, 1, 2
TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module")
def zr():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2401_11469_amd import zr as binding
    binding.debug_record_kernel_names(True)     # tests assert which kernel instantiation ran
    return binding


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    return torch


def _tdtype(torch, dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def to_gpu(torch, a, dtype, ld=None):
    """Upload an fp32 numpy array (already bf16-representable if dtype is bf16);
    ld > cols embeds it in a wider buffer filled with a canary."""
    t = torch.from_numpy(np.ascontiguousarray(a)).to(_tdtype(torch, dtype))
    if ld is None:
        return t.cuda()
    buf = torch.full((a.shape[0], ld), 777.0, dtype=t.dtype, device="cuda")
    buf[:, :a.shape[1]] = t.cuda()
    return buf[:, :a.shape[1]]


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


from parity_util import check_kept_np, relf  # noqa: E402  (tests/ is on sys.path under pytest)


def idx_gpu(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def subset(seed, n, n_keep):
    g = np.random.Generator(np.random.PCG64(seed))
    return np.sort(g.choice(n, size=n_keep, replace=False)).astype(np.int32)


# ------------------------------------------------------------------ select ---

@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 256, 640, 1000, 1024, 1025, 2752, 5120, 40000])
@pytest.mark.parametrize("kind", ["normal", "ties", "uniform"])
def test_select_bit_exact(zr, torch_mod, oracle, n, kind):
    torch = torch_mod
    s = wl.random_case(100 + n, 1, n, 1, score_kind=kind)["scores_K"]
    sg = torch.from_numpy(s).cuda()
    for ratio in (0.0, 0.05, 0.25, 0.5, 0.9):
        if oracle.keep_count(n, ratio) < 1:
            continue
        keep, drop = zr.resize_select(sg, ratio)
        ok, od = oracle.resize_select(s, ratio)
        assert keep.dtype == torch.int32
        assert np.array_equal(keep.cpu().numpy(), ok), (n, kind, ratio)
        assert np.array_equal(drop.cpu().numpy(), od), (n, kind, ratio)
        assert zr.keep_count(n, ratio) == oracle.keep_count(n, ratio)


@pytest.mark.parametrize("n,ratio", [(131072, 0.25), (131073, 0.5), (200000, 0.05), (1 << 20, 0.3),
                                     ((1 << 20) + 77, 0.0), (300001, 0.999), (1 << 22, 0.4)])
@pytest.mark.parametrize("kind", ["normal", "ties", "special"])
def test_select_on_many_workgroups_bit_exact(zr, torch_mod, oracle, n, ratio, kind):
    """One long vector cut into slices of 16384 scores (with scratch): bit-exact against the oracle and
    against the single-workgroup entry point; ties that straddle slices are resolved by index."""
    torch = torch_mod
    g = np.random.Generator(np.random.PCG64(n + int(ratio * 1000)))
    if kind == "normal":
        s = g.standard_normal(n).astype(np.float32)
    elif kind == "ties":
        s = g.integers(0, 5, size=n).astype(np.float32)           # a fifth of the vector ties with the threshold
    else:
        s = g.standard_normal(n).astype(np.float32)
        idx = g.choice(n, size=n // 7, replace=False)
        s[idx] = np.resize(np.array([np.nan, -0.0, 0.0, np.inf, -np.inf, 1.0, -1.0, 3e38, -3e38, 1e-45], np.float32), idx.size)
    assert zr.select_workspace_bytes(n) > 0 and zr.select_workspace_bytes(131071) == 0
    sg = torch.from_numpy(s).cuda()
    ws = torch.full((zr.select_workspace_bytes(n),), 0xab, dtype=torch.uint8, device="cuda")
    keep, drop = zr.resize_select_ws(sg, ratio, ws)
    ok, od = oracle.resize_select(s, ratio)
    assert np.array_equal(keep.cpu().numpy(), ok), (n, kind, ratio)
    assert np.array_equal(drop.cpu().numpy(), od), (n, kind, ratio)
    # again with the buffer as the first call left it, and without a drop list
    keep2, none = zr.resize_select_ws(sg, ratio, ws, want_drop=False)
    assert none is None and torch.equal(keep, keep2)
    # the single workgroup: without scratch, and through the plain entry point
    k1, d1 = zr.resize_select_ws(sg, ratio, None)
    assert torch.equal(k1, keep) and torch.equal(d1, drop)
    if n <= (1 << 20):
        k0, d0 = zr.resize_select(sg, ratio)
        assert torch.equal(k0, keep) and torch.equal(d0, drop)


def test_select_special_values_and_batch(zr, torch_mod, oracle):
    torch = torch_mod
    s = np.array([np.nan, -0.0, 0.0, np.inf, -np.inf, 1.0, np.nan, 0.0, -1.0, 1.0, -np.nan, 3e38],
                 dtype=np.float32)
    for ratio in (0.0, 0.1, 0.25, 0.4, 0.5, 0.75, 0.9):
        keep, drop = zr.resize_select(torch.from_numpy(s).cuda(), ratio)
        ok, od = oracle.resize_select(s, ratio)
        assert np.array_equal(keep.cpu().numpy(), ok) and np.array_equal(drop.cpu().numpy(), od)
    # batched: one workgroup per vector, the config-4 projections' axis lengths padded to one n
    g = np.random.Generator(np.random.PCG64(5))
    B, n = 37, 3072
    S = g.standard_normal((B, n)).astype(np.float32)
    S[3, :] = 1.0                     # all tied: the lowest indices are kept
    S[4, ::2] = np.nan
    keep, drop = zr.resize_select(torch.from_numpy(S).cuda(), 0.35)
    for b in range(B):
        ok, od = oracle.resize_select(S[b], 0.35)
        assert np.array_equal(keep[b].cpu().numpy(), ok) and np.array_equal(drop[b].cpu().numpy(), od)
    assert keep[3].cpu().numpy().tolist() == list(range(oracle.keep_count(n, 0.35)))


@pytest.mark.parametrize("n,ratio", [(1000, 0.3), (4096, 0.05), (12288, 0.5), (13000, 0.25)])
def test_select_many_vectors_in_one_launch(zr, torch_mod, oracle, n, ratio):
    """From 512 vectors on, a launch uses the small-workgroup variant (several vectors
    per compute unit); every vector must still match the oracle bit for bit."""
    torch = torch_mod
    g = np.random.Generator(np.random.PCG64(n))
    B = 600
    S = g.standard_normal((B, n)).astype(np.float32)
    S[:, ::7] = np.round(S[:, ::7], 1)          # plenty of ties
    S[5, :] = -2.0
    S[6, 1::3] = np.nan
    keep, drop = zr.resize_select(torch.from_numpy(S).cuda(), ratio)
    keep, drop = keep.cpu().numpy(), drop.cpu().numpy()
    for b in range(0, B, 7):
        ok, od = oracle.resize_select(S[b], ratio)
        assert np.array_equal(keep[b], ok) and np.array_equal(drop[b], od)


def test_select_on_config_scores(zr, torch_mod, oracle):
    torch = torch_mod
    for cid, cfg in wl.CONFIGS.items():
        for pi, pr in enumerate(cfg.projections):
            s = wl.make_scores(cid, pi)
            assert s.shape == (pr.n_axis,)
            for r in cfg.ratios:
                r = wl.ratio_for(cfg, pr, r)
                keep, drop = zr.resize_select(torch.from_numpy(s).cuda(), r)
                ok, od = oracle.resize_select(s, r)
                assert np.array_equal(keep.cpu().numpy(), ok) and np.array_equal(drop.cpu().numpy(), od)
                assert zr.validate_keep_idx(keep, pr.n_axis)


def test_validate_keep_idx(zr, torch_mod):
    torch = torch_mod
    assert zr.validate_keep_idx(idx_gpu(torch, [0, 3, 4]), 5)
    assert not zr.validate_keep_idx(idx_gpu(torch, [0, 3, 3]), 5)
    assert not zr.validate_keep_idx(idx_gpu(torch, [0, 3, 5]), 5)
    assert not zr.validate_keep_idx(idx_gpu(torch, [-1, 3, 4]), 5)


# ------------------------------------------- priority scores and ratios ---

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [DROP_N, DROP_K])
@pytest.mark.parametrize("use_ws", [False, True])
@pytest.mark.parametrize("K,N", [(1, 1), (7, 5), (130, 257), (512, 256), (1000, 772), (2048, 1024)])
def test_priority_scores_parity(zr, torch_mod, oracle, dtype, mode, K, N, use_ws):
    torch = torch_mod
    ws = None
    if use_ws:
        ws = torch.empty(max(16, zr.priority_workspace_bytes(K, N, mode)), dtype=torch.uint8, device="cuda")
    g = np.random.Generator(np.random.PCG64(K * 7 + N))
    cast = wl.round_to_bf16 if dtype == "bf16" else (lambda x: x)
    Wp = cast((g.standard_normal((K, N)) * 0.02).astype(np.float32))
    Wt = cast((Wp + g.standard_normal((K, N)).astype(np.float32) * 1e-3).astype(np.float32))
    n = N if mode == DROP_N else K
    prev_scores = g.random(n).astype(np.float32)
    ld = N + 3 if N % 2 else N + 8          # odd shapes take the scalar loads, even ones the vector loads
    Wtg, Wpg = to_gpu(torch, Wt, dtype, ld=ld), to_gpu(torch, Wp, dtype, ld=ld)
    got = zr.priority_scores(Wtg, Wpg, mode, workspace=ws).cpu().numpy().astype(np.float64)
    want = oracle.priority_scores(Wt, Wp, mode)
    assert got.shape == want.shape
    assert np.max(np.abs(got - want)) <= 1e-5 * max(np.max(np.abs(want)), 1e-30)
    # incremental rule: previously pruned indices keep their previous score, bit for bit
    keep = subset(3, n, max(1, (2 * n) // 3))
    got = zr.priority_scores(Wtg, Wpg, mode, torch.from_numpy(prev_scores).cuda(), idx_gpu(torch, keep), workspace=ws)
    got = got.cpu().numpy()
    want = oracle.priority_scores(Wt, Wp, mode, prev_scores, keep)
    dropped = np.setdiff1d(np.arange(n), keep)
    assert np.array_equal(got[dropped], prev_scores[dropped])
    assert np.max(np.abs(got[keep].astype(np.float64) - want[keep])) <= 1e-5 * max(np.max(np.abs(want)), 1e-30)
    # bitwise repeatable
    again = zr.priority_scores(Wtg, Wpg, mode, torch.from_numpy(prev_scores).cuda(), idx_gpu(torch, keep),
                               workspace=ws).cpu().numpy()
    assert np.array_equal(got, again)


def test_ratio_controller_parity(zr, torch_mod, oracle):
    torch = torch_mod
    g = np.random.Generator(np.random.PCG64(77))
    for n in (1, 63, 1000, 4096, 20000):
        s = g.random(n).astype(np.float32)
        for theta in (-1.0, 0.0, 0.25, float(s[0]), 2.0):
            cnt = int(zr.count_above(torch.from_numpy(s).cuda(), theta).item())
            assert cnt == int(np.count_nonzero(s > np.float32(theta)))
            for gamma in (0.0, 0.3):
                assert zr.layer_ratio(cnt, n, 0.8, gamma) == oracle.layer_ratio(s, np.float32(theta), 0.8, gamma)
    for T_i, T_avg, M_i in ((12.0, 10.0, 8.0), (9.0, 10.0, 8.0), (30.0, 10.0, 8.0), (10.5, 10.0, 3.0)):
        assert zr.pruning_ratio(T_i, T_avg, M_i) == oracle.pruning_ratio(T_i, T_avg, M_i)


# ------------------------------------------ migrated share, local reduce ---

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("transposed", [False, True])
@pytest.mark.parametrize("M,N,L,begin,end", [
    (64, 64, 64, 0, 64),          # whole, aligned
    (300, 264, 520, 128, 392),    # aligned slice spanning tiles (fast path for bf16)
    (300, 264, 520, 131, 390),    # unaligned slice
    (130, 77, 40, 3, 4),          # a single migrated column
    (513, 1030, 300, 0, 300),     # several tiles with ragged edges
])
def test_migrated_accumulate_parity(zr, torch_mod, oracle, dtype, transposed, M, N, L, begin, end):
    """out += A[:, range] @ W_rows[range, :] in both storage layouts of the weight."""
    torch = torch_mod
    g = np.random.Generator(np.random.PCG64(M + N + L + begin))
    cast = wl.round_to_bf16 if dtype == "bf16" else (lambda x: x)
    A = cast(g.standard_normal((M, L)).astype(np.float32))
    Wm = cast((g.standard_normal((N, L) if transposed else (L, N)) * 0.05).astype(np.float32))
    base = cast(g.standard_normal((M, N)).astype(np.float32))
    Ag, Wg, out = to_gpu(torch, A, dtype), to_gpu(torch, Wm, dtype), to_gpu(torch, base, dtype, ld=N + 8)
    As = Ag[:, begin:end]
    Bs = Wg[:, begin:end] if transposed else Wg[begin:end, :]
    zr.migrated_accumulate(out, As, Bs, transposed)
    torch.cuda.synchronize()
    assert torch.all(out._base[:, N:] == 777.0), "padding overwritten"
    want = oracle.migrated_accumulate(base, A[:, begin:end], Wm[:, begin:end] if transposed else Wm[begin:end, :],
                                      transposed)
    first = to_np(out)
    check_kept_np("out", first, want, dtype, end - begin)
    # a second share lands on top of the first (the receiver may serve several stragglers):
    # again one rounding, now of (what the first call stored) + the share
    zr.migrated_accumulate(out, As, Bs, transposed)
    want2 = oracle.migrated_accumulate(first, A[:, begin:end], Wm[:, begin:end] if transposed else Wm[begin:end, :],
                                       transposed)
    check_kept_np("out, second share", to_np(out), want2, dtype, end - begin)


def test_migrated_shares_sum_to_the_stragglers_product(zr, torch_mod, oracle):
    """fp32, integer-valued inputs (every sum exact): the receivers' shares, each
    over its zr_migration_range, add up to the straggler's own product."""
    torch = torch_mod
    g = np.random.Generator(np.random.PCG64(99))
    e, r_k, L_mig, M, N = 5, 3, 70, 96, 80
    A = g.integers(-3, 4, size=(M, L_mig)).astype(np.float32)
    W = g.integers(-3, 4, size=(L_mig, N)).astype(np.float32)
    total = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    Ag, Wg = torch.from_numpy(A).cuda(), torch.from_numpy(W).cuda()
    for r in range(e):
        b, en = zr.migration_range(r, r_k, e, L_mig)
        assert (b, en) == oracle.migration_range(r, r_k, e, L_mig)
        if en > b:
            zr.migrated_accumulate(total, Ag[:, b:en], Wg[b:en, :], False)
    assert np.array_equal(total.cpu().numpy().astype(np.float64), A.astype(np.float64) @ W.astype(np.float64))


# ------------------------------------------------------------------ impute ---

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("policy", [ZERO, AVERAGE, SAME])
@pytest.mark.parametrize("rows,cols", [(1, 1), (5, 7), (33, 300), (300, 33), (129, 1031)])
def test_impute_parity(zr, torch_mod, oracle, dtype, axis, policy, rows, cols):
    torch = torch_mod
    g = np.random.Generator(np.random.PCG64(rows * 131 + cols))
    cast = wl.round_to_bf16 if dtype == "bf16" else (lambda x: x)
    out = cast(g.standard_normal((rows, cols)).astype(np.float32))
    prev = cast(g.standard_normal((rows, cols)).astype(np.float32))
    n = rows if axis == 0 else cols
    for n_keep in sorted({1, max(1, n // 2), max(1, n - 1), n}):
        S = subset(n_keep + 17, n, n_keep)
        ld = cols + 5
        og = to_gpu(torch, out, dtype, ld=ld)
        pg = to_gpu(torch, prev, dtype, ld=ld)
        zr.impute(og, axis, idx_gpu(torch, S), policy, pg if policy == SAME else None)
        want = oracle.impute(out, axis, S, policy, prev)
        got = to_np(og)
        drop = np.setdiff1d(np.arange(n), S)
        kept_got = got[S, :] if axis == 0 else got[:, S]
        kept_in = out[S, :] if axis == 0 else out[:, S]
        assert np.array_equal(kept_got, kept_in.astype(np.float64))      # kept slices untouched
        dg = got[drop, :] if axis == 0 else got[:, drop]
        dw = want[drop, :] if axis == 0 else want[:, drop]
        if policy in (ZERO, SAME):
            assert np.array_equal(dg, dw)
            if policy == ZERO:
                assert not np.any(np.signbit(dg))
        elif drop.size:
            # mean of up to n values of size ~1 in fp32, then one rounding to the dtype
            atol = 1e-5 if dtype == "f32" else 2.0 ** -8
            assert np.max(np.abs(dg - dw)) <= atol * max(1.0, np.max(np.abs(dw)))
        # the padding between rows is never written
        base = og._base if og._base is not None else og
        assert torch.all(base[:, cols:] == 777.0)


@pytest.mark.parametrize("rows,n", [(1, 2), (9, 64), (37, 130), (130, 1000), (64, 4096)])
def test_extract_kept_columns_bit_exact(zr, torch_mod, oracle, rows, n):
    torch = torch_mod
    g = np.random.Generator(np.random.PCG64(rows + n))
    A = wl.round_to_bf16(g.standard_normal((rows, n)).astype(np.float32))
    Ag = to_gpu(torch, A, "bf16")
    for n_keep in sorted({1, 2, max(1, n // 2), max(1, n - 1), n}):
        S = subset(n_keep + 3, n, n_keep)
        width = (n_keep + 63) // 64 * 64
        out = torch.full((rows, width + 8), 777.0, dtype=torch.bfloat16, device="cuda")
        zr.extract_kept_columns(Ag, idx_gpu(torch, S), out=out[:, :width])
        want = oracle.extract_kept_columns(A, S, width)
        assert np.array_equal(to_np(out[:, :width]), want)
        assert not np.any(np.signbit(to_np(out[:, n_keep:width])))
        assert torch.all(out[:, width:] == 777.0)


def test_select_multi_matches_single_vector_calls(zr, torch_mod, oracle):
    """One launch over vectors of different lengths and ratios, including a
    vector too long for the LDS-staged variant."""
    torch = torch_mod
    g = np.random.Generator(np.random.PCG64(321))
    for ns, ratios in (([3072, 1024, 2752, 2752, 2752], [0.25] * 5),
                       ([1, 7, 64, 1000, 4097, 777], [0.0, 0.5, 0.3, 0.999, 0.05, 0.45]),
                       ([20000, 5], [0.1, 0.2])):
        hs = []
        for n in ns:
            v = g.standard_normal(n).astype(np.float32)
            v[g.integers(0, n, size=max(1, n // 10))] = 0.5          # ties
            hs.append(v)
        keeps, drops = zr.resize_select_multi([torch.from_numpy(v).cuda() for v in hs], ratios)
        torch.cuda.synchronize()
        for v, r, k, d in zip(hs, ratios, keeps, drops):
            S, P = oracle.resize_select(v, r)
            assert np.array_equal(k.cpu().numpy(), S) and np.array_equal(d.cpu().numpy(), P)


# ------------------------------------------------------------------- GEMMs ---

W_KN, W_NK = 0, 1


def run_layer(zr, torch, case, S, mode, dtype, policy=ZERO, pad=0, use_ws=False, w_layout=W_KN):
    """fwd + bwd through the C ABI; returns float64 numpy (Y, dX, dW).
    use_ws: hand the calls the optional scratch buffer (extracted-activation path)."""
    M, K = case["X"].shape
    N = case["W"].shape[1]
    ws = None
    if use_ws:
        nbytes = zr.workspace_bytes(M, K, N, len(S), mode, _tdtype(torch, dtype))
        ws = torch.full((max(nbytes, 16),), 0x7F, dtype=torch.uint8, device="cuda")   # NaN-pattern garbage
    ld = (lambda c: c + pad) if pad else (lambda c: None)
    # the weight, its gradient and the gradient's previous value live in the chosen layout
    nk = w_layout == W_NK
    wl_ = (lambda a: np.ascontiguousarray(a.T)) if nk else (lambda a: a)
    wcols = K if nk else N
    X = to_gpu(torch, case["X"], dtype, ld(K))
    W = to_gpu(torch, wl_(case["W"]), dtype, ld(wcols))
    dY = to_gpu(torch, case["dY"], dtype, ld(N))
    keep = idx_gpu(torch, S)
    pY = to_gpu(torch, case["prev_Y"], dtype, ld(N)) if policy == SAME else None
    pdX = to_gpu(torch, case["prev_dX"], dtype, ld(K)) if policy == SAME else None
    pdW = to_gpu(torch, wl_(case["prev_dW"]), dtype, ld(wcols)) if policy == SAME else None
    Y = to_gpu(torch, np.full((M, N), 555.0, np.float32), dtype, ld(N))
    dX = to_gpu(torch, np.full((M, K), 555.0, np.float32), dtype, ld(K))
    dW = to_gpu(torch, wl_(np.full((K, N), 555.0, np.float32)), dtype, ld(wcols))
    zr.resized_linear_fwd(X, W, keep, mode, policy, pY, Y=Y, workspace=ws, w_layout=w_layout)
    zr.resized_linear_bwd(X, W, dY, keep, mode, policy, pdX, pdW, dX=dX, dW=dW, workspace=ws, w_layout=w_layout)
    torch.cuda.synchronize()
    if pad:
        for t in (Y, dX, dW):
            assert torch.all(t._base[:, t.shape[1]:] == 777.0), "padding overwritten"
    return to_np(Y), to_np(dX), (to_np(dW).T if nk else to_np(dW))


def check_layer(oracle, case, S, mode, dtype, policy, got, tol=None):
    tol = TOL[dtype] if tol is None else tol
    M, K = case["X"].shape
    N = case["W"].shape[1]
    wantY = oracle.resized_linear_fwd(case["X"], case["W"], S, mode, policy, case.get("prev_Y"))
    wantdX, wantdW = oracle.resized_linear_bwd(case["X"], case["W"], case["dY"], S, mode, policy,
                                               case.get("prev_dX"), case.get("prev_dW"))
    names = ("Y", "dX", "dW")
    n = N if mode == DROP_N else K
    P = np.setdiff1d(np.arange(n), S)
    kept = np.zeros(n, dtype=bool)
    kept[S] = True
    # which positions of each output are products (the rest is imputed), and the length of
    # the sums behind them
    if mode == DROP_K:
        where = (None, kept[None, :], kept[:, None])
        terms = (len(S), N, M)
    else:
        where = (kept[None, :], None, kept[None, :])
        terms = (K, len(S), M)
    for name, g, w, wh, C in zip(names, got, (wantY, wantdX, wantdW), where, terms):
        assert g.shape == w.shape
        assert np.all(np.isfinite(g)), name
        e = relf(g, w)
        assert e <= tol, (name, e)
        check_kept_np(name, g, w, dtype, C, wh)       # element by element at the kept positions
    # imputed positions: bit-exact for Zero / Same
    if P.size and policy in (ZERO, SAME):
        Y, dX, dW = got
        if mode == DROP_K:
            pairs = [(dX[:, P], wantdX[:, P]), (dW[P, :], wantdW[P, :])]
        else:
            pairs = [(Y[:, P], wantY[:, P]), (dW[:, P], wantdW[:, P])]
        for g, w in pairs:
            assert np.array_equal(g, w)
            if policy == ZERO:
                assert not np.any(np.signbit(g))
    if P.size and policy == AVERAGE:
        # imputed means, element by element: one rounding of the mean to the output type on
        # top of the (averaged-out) roundings of the kept values it is taken over
        Y, dX, dW = got
        if mode == DROP_K:
            pairs = [(dX[:, P], wantdX[:, P], wantdX), (dW[P, :], wantdW[P, :], wantdW)]
        else:
            pairs = [(Y[:, P], wantY[:, P], wantY), (dW[:, P], wantdW[:, P], wantdW)]
        eps = 2.0 ** -8 if dtype == "bf16" else 1e-5
        for g, w, whole in pairs:
            assert np.max(np.abs(g - w)) <= eps * np.max(np.abs(whole))
    return wantY, wantdX, wantdW


SMALL_SHAPES = [(1, 1, 1), (3, 5, 7), (64, 64, 64), (130, 200, 136), (257, 130, 300), (96, 520, 264)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [DROP_N, DROP_K])
@pytest.mark.parametrize("M,K,N", SMALL_SHAPES)
def test_layer_parity_small_and_ragged(zr, torch_mod, oracle, dtype, mode, M, K, N):
    torch = torch_mod
    case = wl.random_case(1000 + M + 7 * K + 13 * N, M, K, N, dtype)
    n = N if mode == DROP_N else K
    for n_keep in sorted({1, max(1, n // 2), max(1, (3 * n) // 4), max(1, n - 1), n}):
        S = subset(n_keep * 31 + n, n, n_keep)
        got = run_layer(zr, torch, case, S, mode, dtype)
        check_layer(oracle, case, S, mode, dtype, ZERO, got)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [DROP_N, DROP_K])
def test_layer_parity_unaligned_leading_dimensions(zr, torch_mod, oracle, dtype, mode):
    """ld not a multiple of the vector width: element-wise paths; the padding
    columns between rows must stay untouched."""
    torch = torch_mod
    M, K, N = 150, 139, 203
    case = wl.random_case(4242, M, K, N, dtype)
    n = N if mode == DROP_N else K
    for n_keep in (n, (2 * n) // 3):
        S = subset(n_keep, n, n_keep)
        got = run_layer(zr, torch, case, S, mode, dtype, pad=3)
        check_layer(oracle, case, S, mode, dtype, ZERO, got)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [DROP_N, DROP_K])
@pytest.mark.parametrize("policy", [AVERAGE, SAME])
def test_layer_parity_other_policies(zr, torch_mod, oracle, dtype, mode, policy):
    torch = torch_mod
    M, K, N = 140, 264, 200
    case = wl.random_case(777, M, K, N, dtype)
    n = N if mode == DROP_N else K
    S = subset(9, n, (3 * n) // 5)
    got = run_layer(zr, torch, case, S, mode, dtype, policy)
    check_layer(oracle, case, S, mode, dtype, policy, got)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [DROP_N, DROP_K])
@pytest.mark.parametrize("policy", [ZERO, AVERAGE, SAME])
@pytest.mark.parametrize("M,K,N,pad,use_ws", [(140, 264, 200, 0, False), (300, 520, 392, 0, True),
                                              (130, 77, 51, 3, False), (257, 512, 320, 8, True)])
def test_layer_parity_weight_stored_out_by_in(zr, torch_mod, oracle, dtype, mode, policy, M, K, N, pad, use_ws):
    """The shard, its gradient and the gradient's previous value stored [N x K]:
    same mathematics, the kept list now selects rows of the stored weight in DROP_N."""
    torch = torch_mod
    case = wl.random_case(1000 + M + K + N, M, K, N, dtype)
    n = N if mode == DROP_N else K
    for n_keep in sorted({1, (3 * n) // 5, n - 1, n}):
        S = subset(n_keep + 3, n, n_keep)
        got = run_layer(zr, torch, case, S, mode, dtype, policy, pad=pad, use_ws=use_ws, w_layout=W_NK)
        check_layer(oracle, case, S, mode, dtype, policy, got)
        if dtype == "bf16" and policy == ZERO and not pad:
            # both layouts contract in the same order: bitwise equal results
            ref = run_layer(zr, torch, case, S, mode, dtype, policy, w_layout=W_KN)
            for x, y in zip(got, ref):
                assert np.array_equal(x, y)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [DROP_N, DROP_K])
@pytest.mark.parametrize("M,K,N", [(64, 64, 64), (300, 520, 392), (700, 1100, 900)])
def test_average_through_the_epilogue_sums(zr, torch_mod, oracle, dtype, mode, M, K, N):
    """With scratch the Average policy takes its means from sums the product's tiles
    write; without it from a second pass over the stored output.  Both follow the
    oracle; shapes span one tile, several tiles, and the two-panel schedule."""
    torch = torch_mod
    case = wl.random_case(55 + M, M, K, N, dtype)
    n = N if mode == DROP_N else K
    for n_keep in sorted({1, n // 2, n - 1}):
        S = subset(n_keep, n, n_keep)
        for layout in (W_KN, W_NK):
            a = run_layer(zr, torch, case, S, mode, dtype, AVERAGE, use_ws=True, w_layout=layout)
            check_layer(oracle, case, S, mode, dtype, AVERAGE, a)
        b = run_layer(zr, torch, case, S, mode, dtype, AVERAGE, use_ws=False)
        check_layer(oracle, case, S, mode, dtype, AVERAGE, b)


@pytest.mark.parametrize("policy", [ZERO, SAME, AVERAGE])
def test_fast_kernels_with_an_output_width_that_is_not_a_chunk_multiple(zr, torch_mod, oracle, policy):
    """Column-parallel shard stored [N x K] with N = 300: every leading dimension is a multiple
    of 8 (the fast kernels apply) but the scattered width is not, so the column-scatter
    epilogue must not touch whole 16-byte chunks at the row ends."""
    torch = torch_mod
    M, K, N = 270, 520, 300
    case = wl.random_case(9090, M, K, N, "bf16")
    X = to_gpu(torch, case["X"], "bf16")
    Wt = to_gpu(torch, np.ascontiguousarray(case["W"].T), "bf16")
    dY = to_gpu(torch, case["dY"], "bf16", ld=304)
    for n_keep in (N - 1, 200, 3):
        S = subset(n_keep + 11, N, n_keep)
        keep = idx_gpu(torch, S)
        pY = to_gpu(torch, case["prev_Y"], "bf16", ld=304) if policy == SAME else None
        pdW = to_gpu(torch, np.ascontiguousarray(case["prev_dW"].T), "bf16") if policy == SAME else None
        Y = to_gpu(torch, np.full((M, N), 555.0, np.float32), "bf16", ld=304)
        dX = to_gpu(torch, np.full((M, K), 555.0, np.float32), "bf16")
        dWt = to_gpu(torch, np.full((N, K), 555.0, np.float32), "bf16")
        ws = torch.empty(zr.workspace_bytes(M, K, N, n_keep, DROP_N, torch.bfloat16), dtype=torch.uint8, device="cuda")
        zr.resized_linear_fwd(X, Wt, keep, DROP_N, policy, pY, Y=Y, workspace=ws, w_layout=W_NK)
        assert zr.debug_last_kernel().startswith("fast_kernel")
        zr.resized_linear_bwd(X, Wt, dY, keep, DROP_N, policy, None, pdW, dX=dX, dW=dWt, workspace=ws, w_layout=W_NK)
        torch.cuda.synchronize()
        assert torch.all(Y._base[:, N:] == 777.0), "padding overwritten"
        check_layer(oracle, case, S, DROP_N, "bf16", policy, (to_np(Y), to_np(dX), to_np(dWt).T))


def test_contiguous_and_extreme_kept_sets(zr, torch_mod, oracle):
    """Kept sets that are a prefix, a suffix, every other index, or one far
    index: the scatter epilogue's ownership ranges degenerate in each."""
    torch = torch_mod
    M, K, N = 200, 300, 280
    case = wl.random_case(99, M, K, N, "bf16")
    for mode in (DROP_N, DROP_K):
        n = N if mode == DROP_N else K
        sets = [np.arange(0, n // 2), np.arange(n // 2, n), np.arange(0, n, 2), np.arange(1, n, 2),
                np.array([n - 1]), np.array([0]), np.array([0, n - 1]),
                np.concatenate([np.arange(0, 5), np.arange(n - 130, n)])]
        for S in sets:
            S = S.astype(np.int32)
            got = run_layer(zr, torch, case, S, mode, "bf16")
            check_layer(oracle, case, S, mode, "bf16", ZERO, got)
            # Same: the scatter epilogue copies the previous tensor at the same positions
            got = run_layer(zr, torch, case, S, mode, "bf16", SAME)
            check_layer(oracle, case, S, mode, "bf16", SAME, got)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("pad", [0, 3])
def test_same_imputation_in_place(zr, torch_mod, oracle, dtype, pad):
    """The previous tensor may be the output buffer itself: dropped positions
    then keep what they held, kept positions receive the new results."""
    torch = torch_mod
    M, K, N = 300, 264, 392
    case = wl.random_case(4242, M, K, N, dtype)
    for mode in (DROP_N, DROP_K):
        n = N if mode == DROP_N else K
        S = subset(17, n, (2 * n) // 3)
        keep = idx_gpu(torch, S)
        ld = (lambda c: c + pad) if pad else (lambda c: None)
        X, W, dY = (to_gpu(torch, case[k], dtype, ld(c)) for k, c in (("X", K), ("W", N), ("dY", N)))
        Y, dX, dW = (to_gpu(torch, case[k], dtype, ld(c)) for k, c in (("prev_Y", N), ("prev_dX", K), ("prev_dW", N)))
        zr.resized_linear_fwd(X, W, keep, mode, SAME, Y, Y=Y)
        zr.resized_linear_bwd(X, W, dY, keep, mode, SAME, dX, dW, dX=dX, dW=dW)
        torch.cuda.synchronize()
        check_layer(oracle, case, S, mode, dtype, SAME, (to_np(Y), to_np(dX), to_np(dW)))


@pytest.mark.parametrize("mode", [DROP_N, DROP_K])
@pytest.mark.parametrize("M,K,N", [(130, 200, 136), (257, 130, 300), (320, 520, 392), (64, 64, 64)])
def test_workspace_path_matches_oracle_and_in_flight_path(zr, torch_mod, oracle, mode, M, K, N):
    """With the optional scratch buffer the activations' kept columns are
    extracted first; results must match the oracle and the in-flight path."""
    torch = torch_mod
    case = wl.random_case(31 + M + K + N, M, K, N, "bf16")
    n = N if mode == DROP_N else K
    for n_keep in sorted({1, 2, max(1, n // 2), max(1, (3 * n) // 4), n - 1}):
        S = subset(n_keep * 7 + n, n, n_keep)
        a = run_layer(zr, torch, case, S, mode, "bf16", use_ws=True)
        check_layer(oracle, case, S, mode, "bf16", ZERO, a)
        b = run_layer(zr, torch, case, S, mode, "bf16", use_ws=False)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    # other policies go through the same extraction
    S = subset(5, n, (2 * n) // 3)
    for policy in (AVERAGE, SAME):
        got = run_layer(zr, torch, case, S, mode, "bf16", policy, use_ws=True)
        check_layer(oracle, case, S, mode, "bf16", policy, got)


@pytest.mark.parametrize("mode", [DROP_N, DROP_K])
@pytest.mark.parametrize("M,K,N", [(200, 2048, 328), (264, 1536, 2056), (2100, 1100, 136)])
def test_split_contraction_parity(zr, torch_mod, oracle, mode, M, K, N):
    """Few output tiles and a long contraction: with the scratch buffer the contraction is cut into
    slices that a second launch adds up (fp32, fixed order).  Against the oracle element by element,
    all three policies; repeatable bit by bit; and the path without scratch (never split) agrees to
    one rounding of the output."""
    torch = torch_mod
    case = wl.random_case(77 + M + K + N, M, K, N, "bf16")
    n = N if mode == DROP_N else K
    # the forward product in the row-gather layout is one that splits: check that it does
    nk = mode == DROP_N
    Sx = subset(9, n, (3 * n) // 4)
    Xg = to_gpu(torch, case["X"], "bf16")
    Wg = to_gpu(torch, np.ascontiguousarray(case["W"].T) if nk else case["W"], "bf16")
    wsx = torch.empty(zr.workspace_bytes(M, K, N, len(Sx), mode, torch.bfloat16), dtype=torch.uint8, device="cuda")
    zr.resized_linear_fwd(Xg, Wg, idx_gpu(torch, Sx), mode, workspace=wsx, w_layout=W_NK if nk else W_KN)
    torch.cuda.synchronize()
    if (K if mode == DROP_N else len(Sx)) >= 1024 and M <= 512:
        assert "split" in zr.debug_last_kernel(), zr.debug_last_kernel()
    for layout in (W_KN, W_NK):
        S = subset(3 * n + layout, n, (3 * n) // 4)
        for policy in (ZERO, SAME, AVERAGE):
            a = run_layer(zr, torch, case, S, mode, "bf16", policy, use_ws=True, w_layout=layout)
            check_layer(oracle, case, S, mode, "bf16", policy, a)
        a = run_layer(zr, torch, case, S, mode, "bf16", use_ws=True, w_layout=layout)
        a2 = run_layer(zr, torch, case, S, mode, "bf16", use_ws=True, w_layout=layout)
        b = run_layer(zr, torch, case, S, mode, "bf16", use_ws=False, w_layout=layout)
        for x, x2, y in zip(a, a2, b):
            assert np.array_equal(x, x2)
            assert np.max(np.abs(x - y)) <= 2.0 ** -7 * np.max(np.abs(y))


@pytest.mark.parametrize("policy", [ZERO, AVERAGE])
def test_backward_reuses_what_the_forward_extracted(zr, torch_mod, oracle, policy):
    """DROP_K: the forward leaves X[:,S] in the scratch buffer; a backward call that is told
    so must give the results of one that extracts again, bit for bit."""
    torch = torch_mod
    M, K, N = 300, 520, 392
    case = wl.random_case(4711, M, K, N, "bf16")
    S = subset(8, K, (2 * K) // 3)
    keep = idx_gpu(torch, S)
    X, W, dY = (to_gpu(torch, case[k], "bf16") for k in ("X", "W", "dY"))
    ws = torch.full((zr.workspace_bytes(M, K, N, len(S), DROP_K, torch.bfloat16),), 0x7F, dtype=torch.uint8, device="cuda")
    outs = []
    for reuse in (False, True):
        ws.fill_(0x7F)
        Y = zr.resized_linear_fwd(X, W, keep, DROP_K, policy, workspace=ws)
        dX, dW = zr.resized_linear_bwd(X, W, dY, keep, DROP_K, policy, workspace=ws, workspace_holds_forward=reuse)
        torch.cuda.synchronize()
        outs.append((to_np(Y), to_np(dX), to_np(dW)))
    check_layer(oracle, case, S, DROP_K, "bf16", policy, outs[1])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


def test_mfma_rate_probe_runs(zr, torch_mod):
    """The register-only MFMA loop used as a measuring aid: runs, and reports the FLOPs it does."""
    flops = zr.debug_mfma_rate(8, 4)
    torch_mod.cuda.synchronize()
    assert flops == 8 * 4 * 4 * 8 * 2.0 * 32 * 32 * 16
    with pytest.raises(zr.ZrError):
        zr.debug_mfma_rate(0, 4)


def test_bitwise_repeatable(zr, torch_mod):
    torch = torch_mod
    case = wl.random_case(5, 300, 520, 390, "bf16")
    for mode in (DROP_N, DROP_K):
        n = 390 if mode == DROP_N else 520
        S = subset(3, n, (2 * n) // 3)
        a = run_layer(zr, torch, case, S, mode, "bf16")
        b = run_layer(zr, torch, case, S, mode, "bf16")
        for x, y in zip(a, b):
            assert np.array_equal(x, y)


def test_config1_full(zr, torch_mod, oracle):
    """Tiny column-parallel fp32 layer: select by column L2 norm at ratio 0.25,
    then forward and backward, everything against the oracle."""
    torch = torch_mod
    cfg = wl.CONFIGS[1]
    t = wl.make_tensors(1, 0)
    scores = wl.make_scores(1, 0, t["W"])
    keep, drop = zr.resize_select(torch.from_numpy(scores).cuda(), 0.25)
    ok, od = oracle.resize_select(scores, 0.25)
    assert len(ok) == 192 and np.array_equal(keep.cpu().numpy(), ok) and np.array_equal(drop.cpu().numpy(), od)
    got = run_layer(zr, torch, t, ok, DROP_N, "f32")
    check_layer(oracle, t, ok, DROP_N, "f32", ZERO, got)
    # ratio 0 reproduces the full shard GEMM
    full = np.arange(256, dtype=np.int32)
    got = run_layer(zr, torch, t, full, DROP_N, "f32")
    X, W, dY = (t[k].astype(np.float64) for k in ("X", "W", "dY"))
    for name, g, w, C in zip(("Y", "dX", "dW"), got, (X @ W, dY @ W.T, X.T @ dY), (512, 256, 256)):
        assert relf(g, w) <= 1e-5
        check_kept_np(name, g, w, "f32", C)


# ------------------------------------------------------ streams and graphs ---

def _layer_step(zr, torch, t, ratio, ws):
    """select + forward + backward of one shard into the buffers of `t` (current stream)."""
    keeps, _ = zr.resize_select_multi([t["scores"]], [ratio], keep_idx=[t["keep"]], drop_idx=[t["drop"]])
    keep = keeps[0]
    zr.resized_linear_fwd(t["X"], t["W"], keep, t["mode"], Y=t["Y"], workspace=ws, w_layout=t["layout"])
    zr.resized_linear_bwd(t["X"], t["W"], t["dY"], keep, t["mode"], dX=t["dX"], dW=t["dW"], workspace=ws,
                          w_layout=t["layout"])


def _shard(torch, zr, mode, M, K, N, seed):
    case = wl.random_case(seed, M, K, N, "bf16")
    n = N if mode == DROP_N else K
    nk = mode == DROP_N
    g = np.random.Generator(np.random.PCG64(seed))
    t = dict(mode=mode, layout=W_NK if nk else W_KN, n=n, case=case,
             X=to_gpu(torch, case["X"], "bf16"), dY=to_gpu(torch, case["dY"], "bf16"),
             W=to_gpu(torch, np.ascontiguousarray(case["W"].T) if nk else case["W"], "bf16"),
             scores=torch.from_numpy(g.random(n).astype(np.float32)).cuda(),
             keep=torch.empty(n, dtype=torch.int32, device="cuda"), drop=torch.empty(n, dtype=torch.int32, device="cuda"),
             Y=torch.empty((M, N), dtype=torch.bfloat16, device="cuda"),
             dX=torch.empty((M, K), dtype=torch.bfloat16, device="cuda"),
             dW=torch.empty((N, K) if nk else (K, N), dtype=torch.bfloat16, device="cuda"))
    return t


def _check_shard(oracle, t, ratio):
    scores = t["scores"].cpu().numpy()
    S, _ = oracle.resize_select(scores, ratio)
    got = (to_np(t["Y"]), to_np(t["dX"]), to_np(t["dW"]).T if t["layout"] == W_NK else to_np(t["dW"]))
    check_layer(oracle, t["case"], S, t["mode"], "bf16", ZERO, got)


@pytest.mark.parametrize("mode", [DROP_N, DROP_K])
def test_whole_path_on_a_side_stream(zr, torch_mod, oracle, mode):
    """Every call takes the caller's stream; nothing runs on, or waits for, the default stream."""
    torch = torch_mod
    M, K, N = 300, 520, 392
    t = _shard(torch, zr, mode, M, K, N, 2024)
    ws = torch.empty(zr.workspace_bytes(M, K, N, t["n"], mode, torch.bfloat16), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()                      # default priority
    with torch.cuda.stream(side):
        _layer_step(zr, torch, t, 0.3, ws)
    side.synchronize()
    _check_shard(oracle, t, 0.3)


@pytest.mark.parametrize("mode", [DROP_N, DROP_K])
def test_whole_path_in_a_captured_graph(zr, torch_mod, oracle, mode):
    """No call allocates or synchronises, so select + forward + backward can be captured
    once and replayed: the kept COUNT is fixed by the ratio, the kept SET follows the
    scores present at replay time.  Every replay is checked, with eager work and
    synchronisations between the replays."""
    torch = torch_mod
    M, K, N = 300, 520, 392
    t = _shard(torch, zr, mode, M, K, N, 777)
    ws = torch.empty(zr.workspace_bytes(M, K, N, t["n"], mode, torch.bfloat16), dtype=torch.uint8, device="cuda")
    ratio = 0.25
    _layer_step(zr, torch, t, ratio, ws)            # warm-up: every kernel has run once
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _layer_step(zr, torch, t, ratio, ws)
    g = np.random.Generator(np.random.PCG64(5))
    for rep in range(3):
        t["scores"].copy_(torch.from_numpy(g.random(t["n"]).astype(np.float32)).cuda())   # new priorities
        for buf in (t["Y"], t["dX"], t["dW"]):
            buf.fill_(7.0)                                                               # eager work in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _check_shard(oracle, t, ratio)
        replayed = [x.clone() for x in (t["Y"], t["dX"], t["dW"], t["keep"])]
        _layer_step(zr, torch, t, ratio, ws)                                             # the same step, eagerly
        torch.cuda.synchronize()
        for a, b in zip(replayed, (t["Y"], t["dX"], t["dW"], t["keep"])):
            assert torch.equal(a, b)
