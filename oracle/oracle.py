"""CPU oracle for the resized tensor-parallel shard GEMMs (ZERO-resizing).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  It shares no code with the HIP library and the
HIP library never calls it.

Everything is float64 and written in the paper's own order of steps
(Sec. 3.1): prune the operands (extract the kept slices, concatenated in
ascending index order), multiply the pruned matrices with an ordinary matrix
product, then recover the normal shape of every output that lost slices and
impute the missing ones (Zero / Same / Average).  The index set that was
pruned is shared by the input and the weight (Sec. 3.2, "Priority Pruning")
and carried from forward to backward (the lineage tuple of Sec. 3.1); here it
is simply the ``keep_idx`` argument.

Notation: tokens M = bs*sql, X[M x K], W[K x N] (in x out), Y = X W,
dX = dY W^T, dW = X^T dY.  ``mode`` says which axis of W ``keep_idx`` indexes:
DROP_K = the contraction axis (the paper's worked example: columns of its
[out,in] weight and of the input), DROP_N = the output-feature axis (the dual
case of the "dual-pruning" scheme).

Readings of the paper taken here (the paper is silent or ambiguous):
  * kept set = the L*(1-gamma) indices with the LARGEST scores (Algorithm 1:
    top-L_pri select, then ascending sort); small variation is pruned first.
  * kept count = floor((1-gamma)*L + 0.5) in IEEE double.
  * order key of a score: NaN ranks lowest, -0.0 equals +0.0, ties keep the
    lower index first.
  * no rescaling of kept contributions: outputs simply miss the pruned
    partial products (Sec. 3.2, first paragraph).
  * Zero imputes +0.0; Same copies the caller's previous-iteration tensor at
    the same positions; Average imputes, for every missing slice, the
    element-wise mean of the kept slices of the current result.
    Average: parity unpinned against the paper (it prints no value for it);
    pinned only against this stated definition.
  * lightweight migration (Sec. 4.1-4.2): the renumbering r' = (r_i + e - r_k) % e
    and the range [m (r'-1), m r' - 1] are the paper's; when e - 1 does not
    divide L_mig (the paper assumes it does), m = floor(L_mig / (e-1)) and the
    first L_mig mod (e-1) renumbered receivers take one column more, so that
    the ranges still tile [0, L_mig).  The straggler itself (r' = 0) computes
    none of its migrated columns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

DROP_N = 0
DROP_K = 1
ZERO, AVERAGE, SAME = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zr_oracle.c")
_LIB = os.path.join(_HERE, "libzr_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C part with gcc (float64 loops, OpenMP, FP contraction off)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.zro_matmul_f64.argtypes = [dp, dp, dp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
        lib.zro_matmul_f64.restype = None
        lib.zro_num_threads.restype = ctypes.c_int
        lib.zro_keep_count.argtypes = [ctypes.c_int64, ctypes.c_double]
        lib.zro_keep_count.restype = ctypes.c_int64
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().zro_num_threads())


def matmul(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """Ordinary matrix product A[I x C] @ B[C x J] in float64 (plain C loops)."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    assert A.ndim == 2 and B.ndim == 2 and A.shape[1] == B.shape[0]
    I, C = A.shape
    J = B.shape[1]
    out = np.empty((I, J), dtype=np.float64)
    if I == 0 or J == 0:
        return out
    dp = ctypes.POINTER(ctypes.c_double)
    _load().zro_matmul_f64(A.ctypes.data_as(dp), B.ctypes.data_as(dp), out.ctypes.data_as(dp), I, C, J)
    return out


# --------------------------------------------------------------------------
# Selection (Algorithm 1: L_pri = L*(1-gamma); top-L_pri select; ascending sort)
# --------------------------------------------------------------------------

def keep_count(n: int, ratio: float) -> int:
    """Kept count for a pruned axis of length n at pruning ratio gamma."""
    if not (0.0 <= ratio < 1.0):
        raise ValueError("ratio must satisfy 0 <= ratio < 1")
    return int(_load().zro_keep_count(int(n), float(ratio)))


def resize_select(scores: np.ndarray, ratio: float) -> Tuple[np.ndarray, np.ndarray]:
    """Kept and pruned index sets, both ascending.

    A full sort of all indices by (score descending, index ascending) with the
    order key described in the module header; the first n' are kept.
    """
    s = np.asarray(scores, dtype=np.float32)
    assert s.ndim == 1
    n = s.shape[0]
    n_keep = keep_count(n, ratio)
    if n_keep < 1:
        raise ValueError("ratio leaves no kept index")
    is_nan = np.isnan(s)
    val = np.where(is_nan, np.float32(0), s).astype(np.float64) + 0.0  # -0.0 + 0.0 == +0.0
    idx = np.arange(n)
    # lexsort: last key is the primary one.  NaN last, then larger value first,
    # then lower index first.
    order = np.lexsort((idx, -val, is_nan))
    keep = np.sort(order[:n_keep]).astype(np.int32)
    drop = np.sort(order[n_keep:]).astype(np.int32)
    return keep, drop


# --------------------------------------------------------------------------
# Priority bookkeeping and ratios (Sec. 3.1 Eq. 1; Sec. 3.2; Algorithm 1, the
# per-layer block before the top-L_pri select)
# --------------------------------------------------------------------------

def priority_scores(W_t, W_prev, mode: int, prev_scores=None, prev_keep_idx=None) -> np.ndarray:
    """Weight-variation score of every index of the pruned axis:
    delta_i = (1/R) * sum_j |w_ji^t - w_ji^(t-1)|, the mean absolute change of
    slice i over its R elements (columns of W for DROP_N, rows for DROP_K).

    Incremental update: an index that was pruned in the previous epoch (it is
    not in ``prev_keep_idx``) keeps its previous score instead, because its
    zero-imputed gradient made its change artificially small.
    Reading: the algorithm's "sorted" variation list is addressed by original
    index; sorting is part of the later top-L_pri select."""
    Wt = np.asarray(W_t, dtype=np.float64)
    Wp = np.asarray(W_prev, dtype=np.float64)
    assert Wt.shape == Wp.shape
    diff = np.abs(Wt - Wp)
    if mode == DROP_N:
        delta = diff.sum(axis=0) / float(Wt.shape[0])
    elif mode == DROP_K:
        delta = diff.sum(axis=1) / float(Wt.shape[1])
    else:
        raise ValueError("mode")
    if prev_keep_idx is not None:
        assert prev_scores is not None
        was_kept = np.zeros(delta.shape[0], dtype=bool)
        was_kept[np.asarray(prev_keep_idx, dtype=np.int64)] = True
        delta = np.where(was_kept, delta, np.asarray(prev_scores, dtype=np.float64))
    return delta


def pruning_ratio(T_i: float, T_avg: float, M_i: float, gamma_max: float = 0.9) -> float:
    """Eq. 1: gamma = (T_i - T_avg) / M_i, the share of the matrix-multiplication
    time M_i a straggler must shed to close its gap to the average iteration
    time.  Reading: a task that is not slower than the average prunes nothing
    (0), and the ratio is capped at ``gamma_max`` (the paper evaluates up to 9/10)."""
    if not (M_i > 0.0):
        raise ValueError("M_i must be positive")
    g = (T_i - T_avg) / M_i
    return float(min(max(g, 0.0), gamma_max))


def layer_ratio(scores, theta: float, alpha: float, gamma: float) -> float:
    """Differentiated per-layer ratio (Algorithm 1): L_uni = number of indices
    whose variation exceeds theta (= N_iter * theta_iter); gamma_k = 1 - L_uni / L;
    the ratio actually used is max(gamma_k, alpha * gamma).
    Reading: the algorithm's "sum of (delta > theta)" is a count."""
    s = np.asarray(scores, dtype=np.float64)
    L = s.shape[0]
    L_uni = int(np.count_nonzero(s > theta))
    return float(max(1.0 - L_uni / float(L), alpha * gamma))


# --------------------------------------------------------------------------
# Recovery + imputation (Sec. 3.1, "Consistency Constraint" and the policies)
# --------------------------------------------------------------------------

def _dropped(n: int, keep_idx: np.ndarray) -> np.ndarray:
    mask = np.ones(n, dtype=bool)
    mask[keep_idx] = False
    return np.nonzero(mask)[0]


def impute(out: np.ndarray, axis: int, keep_idx: np.ndarray, policy: int = ZERO,
           prev: Optional[np.ndarray] = None) -> np.ndarray:
    """Fill the slices of ``out`` that are missing along ``axis`` (0 = rows,
    1 = columns); kept slices are returned unchanged.  Returns a new array."""
    res = np.array(out, dtype=np.float64, copy=True)
    keep_idx = np.asarray(keep_idx, dtype=np.int64)
    drop = _dropped(res.shape[axis], keep_idx)
    if drop.size == 0:
        return res
    if policy == ZERO:
        fill = 0.0
        if axis == 0:
            res[drop, :] = fill
        else:
            res[:, drop] = fill
    elif policy == SAME:
        assert prev is not None and prev.shape == res.shape
        p = np.asarray(prev, dtype=np.float64)
        if axis == 0:
            res[drop, :] = p[drop, :]
        else:
            res[:, drop] = p[:, drop]
    elif policy == AVERAGE:
        if axis == 0:
            mean = res[keep_idx, :].sum(axis=0) / float(keep_idx.size)   # one mean row
            res[drop, :] = mean[None, :]
        else:
            mean = res[:, keep_idx].sum(axis=1) / float(keep_idx.size)   # one mean column
            res[:, drop] = mean[:, None]
    else:
        raise ValueError("policy")
    return res


def _recover(pruned: np.ndarray, full_shape, axis: int, keep_idx: np.ndarray) -> np.ndarray:
    """Put the slices of a pruned result back at their original positions
    (the i-th kept slice returns to index keep_idx[i]); missing slices are
    left as NaN until impute() fills them."""
    full = np.full(full_shape, np.nan, dtype=np.float64)
    if axis == 0:
        full[keep_idx, :] = pruned
    else:
        full[:, keep_idx] = pruned
    return full


def extract_kept_columns(A, keep_idx, width: Optional[int] = None) -> np.ndarray:
    """The pruning step on its own (Sec. 3.1): the kept columns of A concatenated
    in ascending index order; optionally zero-padded on the right to ``width``."""
    A = np.asarray(A, dtype=np.float64)
    S = np.asarray(keep_idx, dtype=np.int64)
    out = A[:, S]
    if width is not None and width > out.shape[1]:
        out = np.concatenate([out, np.zeros((A.shape[0], width - out.shape[1]))], axis=1)
    return out


# --------------------------------------------------------------------------
# Resized linear layer
# --------------------------------------------------------------------------

def resized_linear_fwd(X, W, keep_idx, mode: int, policy: int = ZERO, prev_Y=None) -> np.ndarray:
    """Forward of the resized layer; result has the normal shape [M x N]."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    S = np.asarray(keep_idx, dtype=np.int64)
    M, K = X.shape
    N = W.shape[1]
    assert W.shape[0] == K
    if mode == DROP_K:
        # prune the same index list from input and weight; the output keeps its
        # normal shape and simply misses the pruned partial products
        pruned_input = X[:, S]
        pruned_weight = W[S, :]
        return matmul(pruned_input, pruned_weight)
    if mode == DROP_N:
        pruned_weight = W[:, S]
        pruned_output = matmul(X, pruned_weight)                 # [M x n']
        Y = _recover(pruned_output, (M, N), 1, S)
        return impute(Y, 1, S, policy, prev_Y)
    raise ValueError("mode")


def resized_linear_bwd(X, W, dY, keep_idx, mode: int, policy: int = ZERO,
                       prev_dX=None, prev_dW=None) -> Tuple[np.ndarray, np.ndarray]:
    """Backward of the resized layer: (dX [M x K], dW [K x N]), normal shapes."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    S = np.asarray(keep_idx, dtype=np.int64)
    M, K = X.shape
    N = W.shape[1]
    assert W.shape[0] == K and dY.shape == (M, N)
    if mode == DROP_K:
        # the upstream gradient stays normal-sized; input and weight are pruned
        pruned_input = X[:, S]                                   # [M x n']
        pruned_weight = W[S, :]                                  # [n' x N]
        pruned_dX = matmul(dY, pruned_weight.T)                  # [M x n']
        pruned_dW = matmul(pruned_input.T, dY)                   # [n' x N]
        dX = impute(_recover(pruned_dX, (M, K), 1, S), 1, S, policy, prev_dX)
        dW = impute(_recover(pruned_dW, (K, N), 0, S), 0, S, policy, prev_dW)
        return dX, dW
    if mode == DROP_N:
        # dual case: the pruned index list lives on the output-feature axis, so
        # it is the weight's and the upstream gradient's columns that are pruned
        pruned_weight = W[:, S]                                  # [K x n']
        pruned_dY = dY[:, S]                                     # [M x n']
        dX = matmul(pruned_dY, pruned_weight.T)                  # [M x K], normal shape
        pruned_dW = matmul(X.T, pruned_dY)                       # [K x n']
        dW = impute(_recover(pruned_dW, (K, N), 1, S), 1, S, policy, prev_dW)
        return dX, dW
    raise ValueError("mode")


# ---------------------------------------------------------------------------
# Lightweight migration, one receiver's share (Sec. 4.1, Sec. 4.2 renumbering)
# ---------------------------------------------------------------------------

def migration_range(r_i: int, r_k: int, e: int, L_mig: int) -> Tuple[int, int]:
    """Columns of the straggler's L_mig migrated columns that task r_i computes,
    as (begin, end) with end exclusive.  The straggler has rank r_k among e
    tasks; the normal tasks are renumbered r' = (r_i + e - r_k) % e = 1..e-1
    and task r' takes [m (r'-1), m r' - 1], m = L_mig / (e-1)."""
    assert e >= 2 and L_mig >= 0
    r_new = (r_i + e - r_k) % e
    if r_new == 0:
        return 0, 0
    m, rem = divmod(L_mig, e - 1)
    begin = m * (r_new - 1) + min(r_new - 1, rem)
    count = m + (1 if r_new - 1 < rem else 0)
    return begin, begin + count


def migrated_accumulate(out, A, B, b_transposed: bool) -> np.ndarray:
    """Local reduce of a migrated sub-matrix (Sec. 4.1): the receiver adds the
    product of the slices it was assigned to its own partial-sum output,
    out + A B (row-parallel forward: A = X_mig[:, range], B = W_mig[range, :])
    or out + A B^T (column-parallel backward: A = dY_mig[:, range],
    B = W_mig[:, range]), so that the ordinary all-reduce that follows also
    carries the migrated results."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    return np.asarray(out, dtype=np.float64) + matmul(A, B.T if b_transposed else B)
