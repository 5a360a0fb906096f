"""ctypes binding of libzr.so (argument marshalling only).

Functions carry the names of the C ABI in include/zr.h.  Tensors are torch
tensors living on the GPU; only their data pointers, shapes and strides cross
the boundary.  There is no CPU fallback: if the library is not built the
import raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

DROP_N, DROP_K = 0, 1
W_KN, W_NK = 0, 1
WS_FRESH, WS_HOLDS_FORWARD = 0, 1
ZERO, AVERAGE, SAME = 0, 1, 2
F32, BF16 = 0, 1

_LIB_PATH = os.environ.get("ZR_LIBZR_PATH") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libzr.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it first (python -m paper_2401_11469_amd.build); "
        "there is no fallback path")
_lib = ctypes.CDLL(_LIB_PATH)

_vp, _i32, _i64, _f64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double

_lib.zr_status_string.argtypes = [ctypes.c_int]
_lib.zr_status_string.restype = ctypes.c_char_p
_lib.zr_keep_count.argtypes = [_i64, _f64]
_lib.zr_keep_count.restype = _i64
_lib.zr_resize_select.argtypes = [_vp, _i32, _i32, _f64, _vp, _vp, _i64, _vp]
_lib.zr_resize_select.restype = ctypes.c_int
_lib.zr_workspace_bytes.argtypes = [_i32, _i32, _i32, _i32, ctypes.c_int, ctypes.c_int]
_lib.zr_workspace_bytes.restype = ctypes.c_size_t
_lib.zr_resized_linear_fwd.argtypes = [_vp, _i64, _vp, _i64, _vp, _i64, _i32, _i32, _i32,
                                       _vp, _i32, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, _vp,
                                       _vp, ctypes.c_size_t, _vp]
_lib.zr_resized_linear_fwd.restype = ctypes.c_int
_lib.zr_resized_linear_bwd.argtypes = [_vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64,
                                       _i32, _i32, _i32, _vp, _i32,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, _vp, _vp,
                                       _vp, ctypes.c_size_t, ctypes.c_int, _vp]
_lib.zr_resized_linear_bwd.restype = ctypes.c_int
_lib.zr_impute.argtypes = [_vp, _i64, _i32, _i32, _i32, _vp, _i32, ctypes.c_int, _vp, ctypes.c_int, _vp]
_lib.zr_impute.restype = ctypes.c_int
_lib.zr_extract_kept_columns.argtypes = [_vp, _i64, _i32, _i32, _vp, _i32, _vp, _i64, ctypes.c_int, _vp]
_lib.zr_extract_kept_columns.restype = ctypes.c_int
_lib.zr_debug_record_kernel_names.argtypes = [ctypes.c_int]
_lib.zr_debug_record_kernel_names.restype = None
_lib.zr_debug_last_kernel.argtypes = []
_lib.zr_debug_last_kernel.restype = ctypes.c_char_p
_lib.zr_priority_scores.argtypes = [_vp, _vp, _i64, _i32, _i32, ctypes.c_int, _vp, _vp, _i32, _vp, ctypes.c_int,
                                    _vp, ctypes.c_size_t, _vp]
_lib.zr_priority_workspace_bytes.argtypes = [_i32, _i32, ctypes.c_int]
_lib.zr_priority_workspace_bytes.restype = ctypes.c_size_t
_lib.zr_priority_scores.restype = ctypes.c_int
_lib.zr_priority_scores_static.argtypes = [_vp, _vp, _i64, _i32, _i32, ctypes.c_int, _vp, _vp, _i32, _vp, ctypes.c_int, _vp]
_lib.zr_priority_scores_static.restype = ctypes.c_int
_lib.zr_priority_static_scratch_bytes.argtypes = []
_lib.zr_priority_static_scratch_bytes.restype = ctypes.c_size_t
_lib.zr_pruning_ratio.argtypes = [_f64, _f64, _f64, _f64]
_lib.zr_pruning_ratio.restype = _f64
_lib.zr_count_above.argtypes = [_vp, _i32, ctypes.c_float, _vp, _vp]
_lib.zr_count_above.restype = ctypes.c_int
_lib.zr_layer_ratio.argtypes = [_i64, _i64, _f64, _f64]
_lib.zr_layer_ratio.restype = _f64
_lib.zr_migration_range.argtypes = [_i32, _i32, _i32, _i64, ctypes.POINTER(_i64), ctypes.POINTER(_i64)]
_lib.zr_migration_range.restype = ctypes.c_int
_lib.zr_migrated_accumulate.argtypes = [_vp, _i64, _vp, _i64, ctypes.c_int, _vp, _i64, _i32, _i32, _i32, ctypes.c_int, _vp]
_lib.zr_migrated_accumulate.restype = ctypes.c_int
_lib.zr_select_workspace_bytes.argtypes = [_i32]
_lib.zr_select_workspace_bytes.restype = ctypes.c_size_t
_lib.zr_resize_select_ws.argtypes = [_vp, _i32, _f64, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.zr_resize_select_ws.restype = ctypes.c_int
_lib.zr_resize_select_multi.argtypes = [_i32, ctypes.POINTER(_vp), ctypes.POINTER(_i32), ctypes.POINTER(_f64),
                                        ctypes.POINTER(_vp), ctypes.POINTER(_vp), _vp]
_lib.zr_resize_select_multi.restype = ctypes.c_int
_lib.zr_debug_time_next_product.argtypes = [_vp, _vp]
_lib.zr_debug_time_next_product.restype = ctypes.c_int
_lib.zr_debug_mfma_rate.argtypes = [_i32, _i32, _vp, ctypes.POINTER(_f64), _vp]
_lib.zr_debug_mfma_rate.restype = ctypes.c_int
_lib.zr_validate_keep_idx.argtypes = [_vp, _i32, _i32, _vp, _vp]
_lib.zr_validate_keep_idx.restype = ctypes.c_int


class ZrError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"libzr status {status}: {_lib.zr_status_string(status).decode()}")


def _check(status: int) -> None:
    if status != 0:
        raise ZrError(status)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _mat(t: Optional[torch.Tensor], name: str):
    """(pointer, leading dimension) of a 2-D row-major CUDA tensor."""
    if t is None:
        return None, 0
    if not t.is_cuda or t.dim() != 2 or t.stride(1) != 1:
        raise ValueError(f"{name}: need a 2-D GPU tensor with unit column stride")
    return t.data_ptr(), t.stride(0)


def _stream(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def workspace_bytes(M: int, K: int, N: int, n_keep: int, mode: int, dtype) -> int:
    code = dtype if isinstance(dtype, int) else (BF16 if dtype == torch.bfloat16 else F32)
    return int(_lib.zr_workspace_bytes(M, K, N, n_keep, mode, code))


def _ws(workspace: Optional[torch.Tensor]):
    if workspace is None:
        return None, 0
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace: need a contiguous GPU tensor")
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def keep_count(n: int, ratio: float) -> int:
    return int(_lib.zr_keep_count(n, ratio))


def status_string(status: int) -> str:
    return _lib.zr_status_string(status).decode()


def resize_select(scores: torch.Tensor, ratio: float, keep_idx: Optional[torch.Tensor] = None,
                  drop_idx: Optional[torch.Tensor] = None, want_drop: bool = True,
                  stream=None) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """scores: fp32 [n] or [batch, n] on the GPU.  Returns (keep_idx, drop_idx) as int32
    tensors of row length n' and n - n' (views of buffers with a common pitch)."""
    if scores.dtype != torch.float32 or not scores.is_cuda or not scores.is_contiguous():
        raise ValueError("scores: need a contiguous fp32 GPU tensor")
    batched = scores.dim() == 2
    n = scores.shape[-1]
    batch = scores.shape[0] if batched else 1
    n_keep = keep_count(n, ratio)
    if n_keep < 1:
        raise ZrError(3)
    ld = max(n_keep, n - n_keep, 1)
    if keep_idx is None:
        keep_idx = torch.empty((batch, ld), dtype=torch.int32, device=scores.device)
    if drop_idx is None and want_drop:
        drop_idx = torch.empty((batch, ld), dtype=torch.int32, device=scores.device)
    for t in (keep_idx, drop_idx):
        if t is not None and (t.dtype != torch.int32 or t.dim() != 2 or t.stride(1) != 1
                              or t.stride(0) != keep_idx.stride(0) or t.shape[0] < batch):
            raise ValueError("index buffers: int32 [batch, ld] with a common pitch")
    _check(_lib.zr_resize_select(scores.data_ptr(), n, batch, float(ratio), keep_idx.data_ptr(),
                                 None if drop_idx is None else drop_idx.data_ptr(),
                                 keep_idx.stride(0), _stream(stream)))
    k = keep_idx[:batch, :n_keep]
    d = None if drop_idx is None else drop_idx[:batch, :n - n_keep]
    if not batched:
        k = k[0]
        d = None if d is None else d[0]
    return k, d


def select_workspace_bytes(n: int) -> int:
    return int(_lib.zr_select_workspace_bytes(n))


def resize_select_ws(scores: torch.Tensor, ratio: float, workspace: Optional[torch.Tensor],
                     keep_idx: Optional[torch.Tensor] = None, drop_idx: Optional[torch.Tensor] = None,
                     want_drop: bool = True, stream=None) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """One fp32 vector [n] on the GPU, with a scratch buffer (select_workspace_bytes(n) bytes) that lets a
    long vector be selected by many workgroups.  Returns (keep_idx[n'], drop_idx[n - n'])."""
    if scores.dtype != torch.float32 or not scores.is_cuda or not scores.is_contiguous() or scores.dim() != 1:
        raise ValueError("scores: need a contiguous 1-D fp32 GPU tensor")
    n = scores.shape[0]
    n_keep = keep_count(n, ratio)
    if n_keep < 1:
        raise ZrError(3)
    if keep_idx is None:
        keep_idx = torch.empty(n_keep, dtype=torch.int32, device=scores.device)
    if drop_idx is None and want_drop:
        drop_idx = torch.empty(max(n - n_keep, 1), dtype=torch.int32, device=scores.device)
    for t, need in ((keep_idx, n_keep), (drop_idx, n - n_keep)):
        if t is not None and (t.dtype != torch.int32 or t.dim() != 1 or not t.is_contiguous() or t.numel() < need):
            raise ValueError("index buffers: contiguous int32 vectors of at least n' and n - n' entries")
    _check(_lib.zr_resize_select_ws(scores.data_ptr(), n, float(ratio), keep_idx.data_ptr(),
                                    None if drop_idx is None else drop_idx.data_ptr(), *_ws(workspace), _stream(stream)))
    return keep_idx[:n_keep], None if drop_idx is None else drop_idx[:n - n_keep]


def resize_select_multi(scores, ratios, keep_idx=None, drop_idx=None, stream=None):
    """One launch for several score vectors (lists of 1-D fp32 GPU tensors and ratios).
    Returns lists of kept / dropped index tensors (views of the given buffers, or new ones)."""
    cnt = len(scores)
    ns = [int(s.numel()) for s in scores]
    nk = [keep_count(n, r) for n, r in zip(ns, ratios)]
    if keep_idx is None:
        keep_idx = [torch.empty(n, dtype=torch.int32, device=s.device) for n, s in zip(ns, scores)]
    if drop_idx is None:
        drop_idx = [torch.empty(n, dtype=torch.int32, device=s.device) for n, s in zip(ns, scores)]
    for s in scores:
        if s.dtype != torch.float32 or not s.is_cuda or not s.is_contiguous():
            raise ValueError("scores: contiguous fp32 GPU tensors")
    PV, PI, PD = _vp * cnt, _i32 * cnt, _f64 * cnt
    _check(_lib.zr_resize_select_multi(cnt, PV(*[s.data_ptr() for s in scores]), PI(*ns), PD(*[float(r) for r in ratios]),
                                       PV(*[k.data_ptr() for k in keep_idx]), PV(*[d.data_ptr() for d in drop_idx]),
                                       _stream(stream)))
    return ([k.view(-1)[:c] for k, c in zip(keep_idx, nk)],
            [d.view(-1)[:n - c] for d, n, c in zip(drop_idx, ns, nk)])


def resized_linear_fwd(X: torch.Tensor, W: torch.Tensor, keep_idx: torch.Tensor, mode: int,
                       policy: int = ZERO, prev_Y: Optional[torch.Tensor] = None,
                       Y: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                       stream=None, w_layout: int = W_KN) -> torch.Tensor:
    """W is [K, N] (w_layout=W_KN) or [N, K] (W_NK)."""
    M, K = X.shape
    N = W.shape[1] if w_layout == W_KN else W.shape[0]
    if tuple(W.shape) != ((K, N) if w_layout == W_KN else (N, K)) or W.dtype != X.dtype:
        raise ValueError("W must be [K, N] (W_KN) or [N, K] (W_NK) with X's dtype")
    if Y is None:
        Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    (xp, ldx), (wp, ldw), (yp, ldy) = _mat(X, "X"), _mat(W, "W"), _mat(Y, "Y")
    pp, ldp = _mat(prev_Y, "prev_Y")
    if prev_Y is not None and ldp != ldy:
        raise ValueError("prev_Y must share Y's leading dimension")
    _check(_lib.zr_resized_linear_fwd(xp, ldx, wp, ldw, yp, ldy, M, K, N,
                                      keep_idx.data_ptr(), keep_idx.numel(), mode, w_layout, _dtype_code(X),
                                      policy, pp, *_ws(workspace), _stream(stream)))
    return Y


def resized_linear_bwd(X: torch.Tensor, W: torch.Tensor, dY: torch.Tensor, keep_idx: torch.Tensor,
                       mode: int, policy: int = ZERO, prev_dX: Optional[torch.Tensor] = None,
                       prev_dW: Optional[torch.Tensor] = None, dX: Optional[torch.Tensor] = None,
                       dW: Optional[torch.Tensor] = None, need_dX: bool = True, need_dW: bool = True,
                       workspace: Optional[torch.Tensor] = None, stream=None,
                       w_layout: int = W_KN,
                       workspace_holds_forward: bool = False) -> Tuple[Optional[torch.Tensor], Optional[torch.Tensor]]:
    """W and dW are [K, N] (w_layout=W_KN) or [N, K] (W_NK).  workspace_holds_forward: the
    workspace is the one the forward call of this layer step used and is untouched since."""
    M, K = X.shape
    N = dY.shape[1]
    wshape = (K, N) if w_layout == W_KN else (N, K)
    if dY.shape[0] != M or tuple(W.shape) != wshape:
        raise ValueError("dY must be [M, N] and W [K, N] (W_KN) or [N, K] (W_NK)")
    if need_dX and dX is None:
        dX = torch.empty((M, K), dtype=X.dtype, device=X.device)
    if need_dW and dW is None:
        dW = torch.empty(wshape, dtype=X.dtype, device=X.device)
    (xp, ldx), (wp, ldw), (gp, ldg) = _mat(X, "X"), _mat(W, "W"), _mat(dY, "dY")
    (dxp, lddx), (dwp, lddw) = _mat(dX if need_dX else None, "dX"), _mat(dW if need_dW else None, "dW")
    (pxp, ldpx), (pwp, ldpw) = _mat(prev_dX, "prev_dX"), _mat(prev_dW, "prev_dW")
    if (prev_dX is not None and need_dX and ldpx != lddx) or (prev_dW is not None and need_dW and ldpw != lddw):
        raise ValueError("previous tensors must share the outputs' leading dimensions")
    _check(_lib.zr_resized_linear_bwd(xp, ldx, wp, ldw, gp, ldg, dxp, lddx, dwp, lddw, M, K, N,
                                      keep_idx.data_ptr(), keep_idx.numel(), mode, w_layout, _dtype_code(X),
                                      policy, pxp, pwp, *_ws(workspace), 1 if workspace_holds_forward else 0,
                                      _stream(stream)))
    return (dX if need_dX else None), (dW if need_dW else None)


def impute(out: torch.Tensor, axis: int, keep_idx: torch.Tensor, policy: int = ZERO,
           prev: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """In place: fills the slices of ``out`` not listed in keep_idx along ``axis``."""
    op, ld = _mat(out, "out")
    pp, ldp = _mat(prev, "prev")
    if prev is not None and ldp != ld:
        raise ValueError("prev must share out's leading dimension")
    _check(_lib.zr_impute(op, ld, out.shape[0], out.shape[1], axis, keep_idx.data_ptr(),
                          keep_idx.numel(), policy, pp, _dtype_code(out), _stream(stream)))
    return out


def extract_kept_columns(inp: torch.Tensor, keep_idx: torch.Tensor, out: Optional[torch.Tensor] = None,
                         stream=None) -> torch.Tensor:
    """out[r, q] = inp[r, keep_idx[q]], zero padded to a multiple of 64 columns (bf16)."""
    rows, n = inp.shape
    width = (keep_idx.numel() + 63) // 64 * 64
    if out is None:
        out = torch.empty((rows, width), dtype=inp.dtype, device=inp.device)
    (ip, ld), (op, ldo) = _mat(inp, "inp"), _mat(out, "out")
    _check(_lib.zr_extract_kept_columns(ip, ld, rows, n, keep_idx.data_ptr(), keep_idx.numel(), op, ldo,
                                        _dtype_code(inp), _stream(stream)))
    return out


def priority_scores(W_t: torch.Tensor, W_prev: torch.Tensor, mode: int,
                    prev_scores: Optional[torch.Tensor] = None, prev_keep_idx: Optional[torch.Tensor] = None,
                    scores: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                    stream=None) -> torch.Tensor:
    K, N = W_t.shape
    (tp, ld), (pp, ldp) = _mat(W_t, "W_t"), _mat(W_prev, "W_prev")
    if W_prev.shape != W_t.shape or ldp != ld or W_prev.dtype != W_t.dtype:
        raise ValueError("W_prev must match W_t in shape, leading dimension and dtype")
    n = N if mode == DROP_N else K
    if scores is None:
        scores = torch.empty(n, dtype=torch.float32, device=W_t.device)
    _check(_lib.zr_priority_scores(tp, pp, ld, K, N, mode,
                                   None if prev_scores is None else prev_scores.data_ptr(),
                                   None if prev_keep_idx is None else prev_keep_idx.data_ptr(),
                                   0 if prev_keep_idx is None else prev_keep_idx.numel(),
                                   scores.data_ptr(), _dtype_code(W_t), *_ws(workspace), _stream(stream)))
    return scores


def priority_scores_static(W_t: torch.Tensor, W_prev: torch.Tensor, mode: int, scores: torch.Tensor,
                           prev_scores: Optional[torch.Tensor] = None, prev_keep_idx: Optional[torch.Tensor] = None,
                           stream=None) -> torch.Tensor:
    """zr_priority_scores_static: the library's own scratch, nothing allocated (the caller brings `scores`)."""
    K, N = W_t.shape
    (tp, ld), (pp, ldp) = _mat(W_t, "W_t"), _mat(W_prev, "W_prev")
    if W_prev.shape != W_t.shape or ldp != ld or W_prev.dtype != W_t.dtype:
        raise ValueError("W_prev must match W_t in shape, leading dimension and dtype")
    _check(_lib.zr_priority_scores_static(tp, pp, ld, K, N, mode,
                                          None if prev_scores is None else prev_scores.data_ptr(),
                                          None if prev_keep_idx is None else prev_keep_idx.data_ptr(),
                                          0 if prev_keep_idx is None else prev_keep_idx.numel(),
                                          scores.data_ptr(), _dtype_code(W_t), _stream(stream)))
    return scores


def priority_static_scratch_bytes() -> int:
    return int(_lib.zr_priority_static_scratch_bytes())


def priority_workspace_bytes(K: int, N: int, mode: int) -> int:
    return int(_lib.zr_priority_workspace_bytes(K, N, mode))


def pruning_ratio(T_i: float, T_avg: float, M_i: float, gamma_max: float = 0.9) -> float:
    return float(_lib.zr_pruning_ratio(T_i, T_avg, M_i, gamma_max))


def count_above(scores: torch.Tensor, theta: float, count: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if count is None:
        count = torch.empty(1, dtype=torch.int32, device=scores.device)
    _check(_lib.zr_count_above(scores.data_ptr(), scores.numel(), float(theta), count.data_ptr(), _stream(stream)))
    return count


def layer_ratio(count_above_: int, L: int, alpha: float, gamma: float) -> float:
    return float(_lib.zr_layer_ratio(int(count_above_), int(L), alpha, gamma))


def migration_range(r_i: int, r_k: int, e: int, L_mig: int):
    b, en = _i64(0), _i64(0)
    _check(_lib.zr_migration_range(r_i, r_k, e, L_mig, ctypes.byref(b), ctypes.byref(en)))
    return int(b.value), int(en.value)


def migrated_accumulate(out: torch.Tensor, A: torch.Tensor, B: torch.Tensor, b_transposed: bool, stream=None) -> torch.Tensor:
    """out += A @ B (or A @ B.T); A, B, out may be column/row slices of larger matrices."""
    M, C = A.shape
    N = out.shape[1]
    if out.shape[0] != M or tuple(B.shape) != ((N, C) if b_transposed else (C, N)):
        raise ValueError("shape mismatch")
    if not (A.dtype == B.dtype == out.dtype):
        raise ValueError("dtype mismatch")
    (ap, lda), (bp, ldb), (op, ldo) = _mat(A, "A"), _mat(B, "B"), _mat(out, "out")
    _check(_lib.zr_migrated_accumulate(ap, lda, bp, ldb, 1 if b_transposed else 0, op, ldo, M, N, C,
                                       _dtype_code(out), _stream(stream)))
    return out


def debug_time_next_product(start: "torch.cuda.Event", stop: "torch.cuda.Event") -> None:
    """The next product records the two events right around its GEMM launch(es).
    The events must have been created with enable_timing=True and recorded once
    before (torch creates the HIP event lazily)."""
    _check(_lib.zr_debug_time_next_product(start.cuda_event, stop.cuda_event))


def debug_mfma_rate(blocks: int, iters: int, stream=None) -> float:
    """Launches the register-only MFMA loop (time it with events); returns the FLOPs it performs."""
    sink = torch.empty(blocks, dtype=torch.float32, device="cuda")
    flops = ctypes.c_double(0.0)
    _check(_lib.zr_debug_mfma_rate(blocks, iters, sink.data_ptr(), ctypes.byref(flops), _stream(stream)))
    return float(flops.value)


def debug_record_kernel_names(on: bool = True) -> None:
    """Switches the recording of GEMM kernel names on or off for this thread (off by default)."""
    _lib.zr_debug_record_kernel_names(1 if on else 0)


def debug_last_kernel() -> str:
    return _lib.zr_debug_last_kernel().decode()


def validate_keep_idx(keep_idx: torch.Tensor, n: int, stream=None) -> bool:
    flag = torch.zeros(1, dtype=torch.int32, device=keep_idx.device)
    st = _lib.zr_validate_keep_idx(keep_idx.data_ptr(), keep_idx.numel(), n, flag.data_ptr(), _stream(stream))
    if st == 0:
        return True
    if st == 4:
        return False
    raise ZrError(st)
