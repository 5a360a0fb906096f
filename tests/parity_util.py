"""Element-wise parity bounds shared by the GPU parity tests.

A kept result of the HIP path is g = round_to_output_type(s), where s is the
fp32-accumulated sum of exact products of the inputs; the oracle's value w is the
same sum in float64.  So for every kept element

    |g - w| <= u * |w| * (1 + 2^-10)  +  acc(C) * rms(w)

with u the unit roundoff of the OUTPUT type (bf16: 8 significant bits, u = 2^-8;
one rounding to nearest) and acc(C) the fp32 accumulation error of a C-term sum
relative to the typical result size: a random-walk estimate sqrt(C) * 2^-24 with a
safety factor of 8 (the worst-case bound C * 2^-24 * sum|a b| is never approached
by rounding errors of mixed sign).  fp32 outputs have no output rounding beyond
the accumulation itself and are held to 1e-5 * max|w| per element.
The whole-tensor figure that goes with it: relative Frobenius error, expected
about 1.6e-3 for bf16 outputs (rms of one rounding to 8 bits), failed above 5e-3;
fp32: failed above 1e-5.
"""
import numpy as np

U_BF16 = 2.0 ** -8
REL_F_LIMIT = {"f32": 1e-5, "bf16": 5e-3}


def acc_term(C: int) -> float:
    return 8.0 * float(np.sqrt(max(C, 1))) * 2.0 ** -24


def relf(got, want):
    den = np.linalg.norm(want)
    return np.linalg.norm(got - want) / (den if den > 0 else 1.0)


def check_kept_np(name, got, want, dtype, C, where=None):
    """got / want: float64 arrays of the same shape; `where`: boolean mask (broadcastable)
    of the kept positions, None = all.  Returns the relative Frobenius error over them."""
    if where is not None:
        sel = np.broadcast_to(where, want.shape)
        g, w = got[sel], want[sel]
    else:
        g, w = got.ravel(), want.ravel()
    if w.size == 0:
        return 0.0
    assert np.all(np.isfinite(g)), name
    rms = float(np.sqrt(np.mean(w * w)))
    if dtype == "bf16":
        bound = U_BF16 * np.abs(w) * (1.0 + 2.0 ** -10) + acc_term(C) * rms
    else:
        bound = np.full(w.shape, 1e-5 * float(np.max(np.abs(w))) if w.size else 0.0)
    diff = np.abs(g - w)
    bad = diff > bound
    if np.any(bad):
        i = int(np.argmax(diff - bound))
        raise AssertionError(f"{name}: {int(bad.sum())} of {w.size} kept elements beyond the element-wise bound; "
                             f"worst: got {g[i]!r} want {w[i]!r} bound {bound[i]!r}")
    e = relf(g, w)
    assert e <= REL_F_LIMIT[dtype], (name, "relative Frobenius error", e)
    return e


def check_kept_torch(name, got, ref, dtype, C, where=None):
    """The same check on the GPU for whole tensors: `ref` is an fp32 tensor (library GEMM of
    the masked-dense identity, itself an fp32 accumulation, which the accumulation term
    covers); `where`: boolean tensor (broadcastable) of kept positions."""
    import torch
    g = got.float()
    assert torch.isfinite(g).all(), name
    if where is not None:
        sel = where.expand_as(ref)
        n = int(sel.sum().item())
        if n == 0:
            return 0.0
        rms = float(torch.sqrt((ref * ref * sel).sum() / n).item())
    else:
        sel = None
        rms = float(torch.sqrt((ref * ref).mean()).item())
    if dtype == "bf16":
        bound = U_BF16 * (1.0 + 2.0 ** -10) * ref.abs() + acc_term(C) * rms
    else:
        mx = float((ref.abs() * sel).max().item()) if sel is not None else float(ref.abs().max().item())
        bound = torch.full_like(ref, 1e-5 * mx)
    over = (g - ref).abs() - bound
    if sel is not None:
        over = torch.where(sel, over, torch.full_like(over, -1.0))
    nbad = int((over > 0).sum().item())
    if nbad:
        i = int(torch.argmax(over).item())
        r, c = divmod(i, ref.shape[1])
        raise AssertionError(f"{name}: {nbad} kept elements beyond the element-wise bound; worst at ({r}, {c}): "
                             f"got {g[r, c].item()!r} ref {ref[r, c].item()!r} bound {bound[r, c].item()!r}")
    d = (g - ref)
    if sel is not None:
        d, rr = d * sel, ref * sel
    else:
        rr = ref
    e = float((torch.linalg.norm(d) / torch.linalg.norm(rr)).item())
    assert e <= REL_F_LIMIT[dtype], (name, "relative Frobenius error", e)
    return e
