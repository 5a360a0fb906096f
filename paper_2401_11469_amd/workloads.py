"""Seeded synthetic workloads for the resized tensor-parallel shard GEMMs.

This module only *generates inputs*: shapes, seeds, random draws and the
bf16 rounding of those draws.  It holds none of the method's arithmetic
(no selection, no GEMM, no imputation), so both the CPU oracle's tests and
the HIP path's tests/bench may draw their inputs from it.

The shapes stand in for the transformer layers the method is applied to
(one tensor-parallel task's shard of each linear projection, Sec. 2.2 of
the paper): column-parallel projections split W on its output axis N,
row-parallel ones on its input axis K.  Weights are stored W[K x N]
(in-features x out-features), activations X[M x K] with M = batch*seq
tokens, upstream gradient dY[M x N].
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

DROP_N = 0  # keep_idx indexes W's columns / output features (column-parallel shard)
DROP_K = 1  # keep_idx indexes W's rows / contraction axis (row-parallel shard)

BASE_SEED = 20240111
TENSOR_X, TENSOR_W, TENSOR_DY, TENSOR_SCORES, TENSOR_RATIOS, TENSOR_PREV = 0, 1, 2, 3, 4, 5
W_SIGMA = 0.02  # N(0, 0.02): 0.02 is the standard deviation (GPT-2 init convention)


@dataclass(frozen=True)
class Projection:
    name: str
    parallel: str  # "col" or "row"
    K: int
    N: int

    @property
    def mode(self) -> int:
        return DROP_N if self.parallel == "col" else DROP_K

    @property
    def n_axis(self) -> int:
        """Length of the pruned axis."""
        return self.N if self.parallel == "col" else self.K


@dataclass(frozen=True)
class Config:
    cid: int
    name: str
    dtype: str  # "f32" or "bf16"
    M: int
    projections: Tuple[Projection, ...]
    ratios: Tuple[float, ...]
    scores: str  # "l2" | "lognormal" | "uniform"
    # per-parallel-kind ratio override (config 5): {"col": r, "row": r}
    mixed: Tuple[Tuple[str, float], ...] = ()


def _p(name, parallel, K, N):
    return Projection(name, parallel, K, N)


CONFIGS: Dict[int, Config] = {
    1: Config(1, "tiny-col-linear-tp2", "f32", 256,
              (_p("lin", "col", 512, 256),), (0.25,), "l2"),
    2: Config(2, "gpt2-medium-tp4", "bf16", 8 * 1024,
              (_p("qkv", "col", 1024, 768), _p("out", "row", 256, 1024),
               _p("fc1", "col", 1024, 1024), _p("fc2", "row", 1024, 1024)),
              (0.0, 0.1, 0.25, 0.5), "l2"),
    3: Config(3, "vit-large-tp2", "bf16", 64 * 197,
              (_p("fc1", "col", 1024, 2048), _p("fc2", "row", 2048, 1024)),
              (0.0, 0.2, 0.4), "lognormal"),
    4: Config(4, "llama2-7b-tp4", "bf16", 4 * 2048,
              (_p("qkv", "col", 4096, 3072), _p("out", "row", 1024, 4096),
               _p("gate", "col", 4096, 2752), _p("up", "col", 4096, 2752),
               _p("down", "row", 2752, 4096)),
              tuple(j / 20 for j in range(11)), "l2"),
    5: Config(5, "llama2-13b-tp8", "bf16", 2 * 4096,
              (_p("qkv", "col", 5120, 1920), _p("out", "row", 640, 5120),
               _p("gate", "col", 5120, 1728), _p("up", "col", 5120, 1728),
               _p("down", "row", 1728, 5120)),
              (0.3, 0.15), "uniform", (("col", 0.3), ("row", 0.15))),
}


def seed_for(cid: int, proj_index: int, tensor_id: int) -> int:
    return BASE_SEED + 1000 * cid + 10 * proj_index + tensor_id


def _rng(cid: int, proj_index: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed_for(cid, proj_index, tensor_id)))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32.

    Input preparation only: the draws are made representable in bf16 so that
    the oracle and the GPU consume identical bits.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def _cast(x: np.ndarray, dtype: str) -> np.ndarray:
    x = x.astype(np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


def make_tensors(cid: int, proj_index: int, M: int | None = None,
                 want=("X", "W", "dY")) -> Dict[str, np.ndarray]:
    """fp32 arrays (bf16-representable when the config is bf16) for one projection.

    ``M`` overrides the token count (a leading slice of the same stream is NOT
    implied: a different M gives a fresh draw of that size).
    """
    cfg = CONFIGS[cid]
    pr = cfg.projections[proj_index]
    M = cfg.M if M is None else M
    out = {}
    if "X" in want:
        out["X"] = _cast(_rng(cid, proj_index, TENSOR_X).standard_normal((M, pr.K), dtype=np.float32), cfg.dtype)
    if "W" in want:
        w = _rng(cid, proj_index, TENSOR_W).standard_normal((pr.K, pr.N), dtype=np.float32) * np.float32(W_SIGMA)
        out["W"] = _cast(w, cfg.dtype)
    if "dY" in want:
        out["dY"] = _cast(_rng(cid, proj_index, TENSOR_DY).standard_normal((M, pr.N), dtype=np.float32), cfg.dtype)
    return out


def make_scores(cid: int, proj_index: int, W: np.ndarray | None = None) -> np.ndarray:
    """Per-index fp32 importance scores along the pruned axis.

    "l2": L2 norm of each W column (column-parallel) or row (row-parallel);
    it stands in for the paper's weight-variation score, which needs two
    weight snapshots from real training.  "lognormal": exp(N(0,1)).
    "uniform": U[0,1).
    """
    cfg = CONFIGS[cid]
    pr = cfg.projections[proj_index]
    n = pr.n_axis
    if cfg.scores == "l2":
        if W is None:
            W = make_tensors(cid, proj_index, M=1, want=("W",))["W"]
        axis = 0 if pr.parallel == "col" else 1
        return np.sqrt((W.astype(np.float64) ** 2).sum(axis=axis)).astype(np.float32)
    g = _rng(cid, proj_index, TENSOR_SCORES)
    if cfg.scores == "lognormal":
        return np.exp(g.standard_normal(n)).astype(np.float32)
    if cfg.scores == "uniform":
        return g.random(n, dtype=np.float32)
    raise ValueError(cfg.scores)


def ratio_for(cfg: Config, pr: Projection, ratio: float) -> float:
    """Config 5 fixes one ratio per parallel kind; other configs use ``ratio``."""
    for kind, r in cfg.mixed:
        if kind == pr.parallel:
            return r
    return ratio


def ratio_sequence(cid: int, steps: int) -> List[float]:
    """Seeded per-step ratios drawn uniformly from the config's ratio list
    (mimics time-varying straggler contention)."""
    cfg = CONFIGS[cid]
    g = _rng(cid, 0, TENSOR_RATIOS)
    pick = g.integers(0, len(cfg.ratios), size=steps)
    return [cfg.ratios[int(i)] for i in pick]


def random_case(seed: int, M: int, K: int, N: int, dtype: str = "f32",
                score_kind: str = "normal") -> Dict[str, np.ndarray]:
    """Free-form seeded case for parity tests over odd shapes."""
    g = np.random.Generator(np.random.PCG64(seed))
    X = _cast(g.standard_normal((M, K), dtype=np.float32), dtype)
    W = _cast(g.standard_normal((K, N), dtype=np.float32) * np.float32(W_SIGMA), dtype)
    dY = _cast(g.standard_normal((M, N), dtype=np.float32), dtype)
    out = {"X": X, "W": W, "dY": dY}
    for tag, n in (("scores_K", K), ("scores_N", N)):
        if score_kind == "normal":
            s = g.standard_normal(n).astype(np.float32)
        elif score_kind == "ties":  # few distinct values: many exact ties
            s = g.integers(0, 4, size=n).astype(np.float32)
        else:
            s = g.random(n, dtype=np.float32)
        out[tag] = s
    out["prev_Y"] = _cast(g.standard_normal((M, N), dtype=np.float32), dtype)
    out["prev_dX"] = _cast(g.standard_normal((M, K), dtype=np.float32), dtype)
    out["prev_dW"] = _cast(g.standard_normal((K, N), dtype=np.float32), dtype)
    return out


def kept_flops(M: int, K: int, N: int, n: int, n_keep: int) -> float:
    """Kept work of one projection, forward + dX + dW: 6*M*K*N*(n_keep/n)."""
    return 6.0 * M * K * N * (n_keep / n)
