"""zr_priority_scores_static (the entry point for callers that cannot allocate) against
zr_priority_scores with a caller workspace: same bits, on two calls in a row, the second
with a smaller input, so that what the first call left in the library's scratch would show."""
import numpy as np
import pytest

from paper_2401_11469_amd import workloads as wl

pytestmark = pytest.mark.gpu

DROP_N, DROP_K = 0, 1


def _snapshots(torch, K, N, dtype, seed):
    g = np.random.Generator(np.random.PCG64(seed))
    cast = wl.round_to_bf16 if dtype == "bf16" else (lambda x: x)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Wp = cast((g.standard_normal((K, N)) * 0.02).astype(np.float32))
    Wt = cast((Wp + g.standard_normal((K, N)).astype(np.float32) * 1e-3).astype(np.float32))
    return Wt, Wp, torch.from_numpy(Wt).to(tdt).cuda(), torch.from_numpy(Wp).to(tdt).cuda()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_entry_point_matches_the_workspace_one(oracle, dtype):
    import torch
    from paper_2401_11469_amd import zr
    assert torch.cuda.is_available()
    assert zr.priority_static_scratch_bytes() == 1 << 20
    # first call: wide and tall (many row ranges); second: smaller in both directions
    for call, (K, N) in enumerate(((4096, 3072), (1000, 520))):
        Wt, Wp, Wtd, Wpd = _snapshots(torch, K, N, dtype, 31 + call)
        for mode in (DROP_N, DROP_K):
            n = N if mode == DROP_N else K
            nbytes = zr.priority_workspace_bytes(K, N, mode)
            assert nbytes <= zr.priority_static_scratch_bytes()
            ws = torch.empty(max(16, nbytes), dtype=torch.uint8, device="cuda")
            want = zr.priority_scores(Wtd, Wpd, mode, workspace=ws)
            got = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
            zr.priority_scores_static(Wtd, Wpd, mode, got)
            torch.cuda.synchronize()
            assert torch.equal(got, want), (call, mode, "bits differ from the workspace entry point")
            ref = oracle.priority_scores(Wt, Wp, mode)
            assert np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref)) <= 1e-5 * np.max(np.abs(ref))
            # the incremental rule through the same entry point
            keep = np.sort(np.random.Generator(np.random.PCG64(5)).choice(n, size=(2 * n) // 3, replace=False)).astype(np.int32)
            prev = np.random.Generator(np.random.PCG64(6)).random(n).astype(np.float32)
            kd, pd = torch.from_numpy(keep).cuda(), torch.from_numpy(prev).cuda()
            want2 = zr.priority_scores(Wtd, Wpd, mode, pd, kd, workspace=ws)
            got2 = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
            zr.priority_scores_static(Wtd, Wpd, mode, got2, pd, kd)
            torch.cuda.synchronize()
            assert torch.equal(got2, want2), (call, mode, "incremental")


def test_static_scratch_rejects_sizes_beyond_its_limit():
    import torch
    from paper_2401_11469_amd import zr
    K, N = 512, 400000          # needs more row-range sums than 1 MiB holds
    assert zr.priority_workspace_bytes(K, N, DROP_N) > zr.priority_static_scratch_bytes()
    Wt = torch.zeros((K, N), dtype=torch.bfloat16, device="cuda")
    out = torch.full((N,), -1.0, dtype=torch.float32, device="cuda")
    with pytest.raises(Exception) as e:
        zr.priority_scores_static(Wt, Wt, DROP_N, out)
    assert "limit" in str(e.value).lower()
    torch.cuda.synchronize()
    assert torch.all(out == -1.0)            # nothing was enqueued
