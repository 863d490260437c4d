"""Seeded synthetic workloads: banks, queries, Q tables, update batches.

This module only draws random inputs (NumPy, CPU).  It contains none of the retrieval method's
arithmetic, so both the GPU library's tests and the CPU oracle can consume it.  The paper
(Sec. 3.2) never states bank sizes, embedding model or dimension; the shapes below are the
synthetic workloads this repository measures, and stand in for an agent's memory bank only in shape.

Every bank is generated in independent 65,536-row chunks, chunk j of workload c being seeded by
(SEED + c, j), so that any chunk can be regenerated alone.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

SEED = 260310846
CHUNK_ROWS = 65536

DRAFT, REFINE = 0, 1


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # seed offset
    N: int                     # bank size (entries)
    d: int                     # embedding dimension
    dtype: str                 # "f32" | "bf16" | "f16"  (storage type; accumulation is fp32 or wider)
    B: int                     # queries per retrieval call
    k1: int                    # candidate pool size (the paper's K)
    k2: int                    # final context size (the paper's N)
    lam: float                 # mixing weight between z(sim) and z(Q)
    alpha: float               # step size of the value update
    clustered: bool = False
    n_clusters: int = 256
    extra: dict = field(default_factory=dict)


TINY = Workload("tiny", 1, 4096, 768, "f32", 1, 32, 4, 0.5, 0.1)
MID = Workload("mid", 2, 65536, 1024, "f32", 64, 64, 8, 0.5, 0.1)
CLUSTERED = Workload("clustered", 3, 1048576, 1024, "bf16", 256, 128, 16, 0.5, 0.1, clustered=True)
LARGE = Workload("large", 4, 4194304, 1536, "bf16", 1024, 128, 16, 0.5, 0.05)
STREAM = Workload("stream", 5, 8388608, 4096, "f16", 128, 256, 32, 0.7, 0.1,
                  extra={"N0": 1048576, "steps": 112})
WORKLOADS = {w.name: w for w in (TINY, MID, CLUSTERED, LARGE, STREAM)}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (used for reduced-size parity cases)."""
    d = dict(w.__dict__)
    d.update(kw)
    return Workload(**d)


def _rng(w: Workload, *stream) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([SEED + w.index, *stream]))


def _normalise(x: np.ndarray) -> np.ndarray:
    n = np.sqrt((x.astype(np.float64) ** 2).sum(axis=1, keepdims=True))
    return (x / n).astype(np.float32)


def _centres(w: Workload) -> np.ndarray:
    # unnormalised N(0, I_d) centres: |c| ~ sqrt(d), so 0.3*N(0,1) noise keeps clusters tight
    return _rng(w, 1000).standard_normal((w.n_clusters, w.d), dtype=np.float32)


def bank_chunk(w: Workload, j: int, rows: int | None = None) -> np.ndarray:
    """fp32 rows [rows, d] of chunk j (ids j*CHUNK_ROWS ...), each L2-normalised."""
    rows = min(CHUNK_ROWS, w.N - j * CHUNK_ROWS) if rows is None else rows
    g = _rng(w, 1, j)
    x = g.standard_normal((rows, w.d), dtype=np.float32)
    if w.clustered:
        which = g.integers(0, w.n_clusters, size=rows)
        x = _centres(w)[which] + np.float32(0.3) * x
    return _normalise(x)


def n_chunks(w: Workload, N: int | None = None) -> int:
    N = w.N if N is None else N
    return (N + CHUNK_ROWS - 1) // CHUNK_ROWS


def bank(w: Workload) -> np.ndarray:
    """Whole bank as one fp32 array (only for sizes that fit host memory comfortably)."""
    return np.concatenate([bank_chunk(w, j) for j in range(n_chunks(w))], axis=0)


def queries(w: Workload, step: int = 0, B: int | None = None) -> np.ndarray:
    """fp32 queries [B, d], L2-normalised; near cluster centres for the clustered workload."""
    B = w.B if B is None else B
    g = _rng(w, 2, step)
    x = g.standard_normal((B, w.d), dtype=np.float32)
    if w.clustered:
        which = g.integers(0, w.n_clusters, size=B)
        x = _centres(w)[which] + np.float32(0.1) * x
    return _normalise(x)


def q_tables(w: Workload, N: int | None = None) -> np.ndarray:
    """Initial Q tables [2, N] fp32 (row 0 drafting, row 1 refining)."""
    N = w.N if N is None else N
    g = _rng(w, 3)
    if w.name in ("mid", "stream"):
        return np.zeros((2, N), np.float32)        # built up by update batches / start cold
    if w.clustered:
        return np.clip(g.normal(0.0, 0.5, size=(2, N)), -1.0, 1.0).astype(np.float32)
    return g.uniform(-1.0, 1.0, size=(2, N)).astype(np.float32)


def ema_rounds(w: Workload, rounds: int = 20, per_round: int = 8192, p: float = 0.3,
               N: int | None = None):
    """Update batches that build the `mid` workload's Q tables: for each round and each stage,
    ids drawn uniformly with replacement and Bernoulli(p) rewards.  Yields (stage, ids, rewards)."""
    N = w.N if N is None else N
    for r in range(rounds):
        for stage in (DRAFT, REFINE):
            g = _rng(w, 4, r, stage)
            ids = g.integers(0, N, size=per_round).astype(np.int32)
            rewards = (g.random(per_round) < p).astype(np.float32)
            yield stage, ids, rewards


def zipf_update(w: Workload, M: int = 16384, s: float = 1.1, N: int | None = None):
    """Heavily duplicated update batch: Zipf(s) ranks over N mapped through a fixed random
    permutation, rewards uniform in [0,1]."""
    N = w.N if N is None else N
    g = _rng(w, 5)
    weights = 1.0 / np.power(np.arange(1, N + 1, dtype=np.float64), s)
    cdf = np.cumsum(weights)
    cdf /= cdf[-1]
    ranks = np.searchsorted(cdf, g.random(M), side="left")
    perm_seed = _rng(w, 6)
    # a fixed pseudo-random bijection of [0,N): affine map with an odd multiplier modulo a power of
    # two when N is one, else an explicit permutation
    if N & (N - 1) == 0:
        a = int(perm_seed.integers(0, N // 2)) * 2 + 1
        b = int(perm_seed.integers(0, N))
        ids = (ranks.astype(np.int64) * a + b) % N
    else:
        ids = perm_seed.permutation(N)[ranks]
    return ids.astype(np.int32), g.random(M).astype(np.float32)


def bernoulli_rewards(w: Workload, step: int, count: int, p: float = 0.2) -> np.ndarray:
    return (_rng(w, 7, step).random(count) < p).astype(np.float32)
