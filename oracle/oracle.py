"""NumPy-facing wrapper of the CPU oracle (oracle/evomem_oracle.c) -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module.  It holds
no arithmetic of its own beyond argument marshalling and the trivial merge of per-chunk candidate
lists; every step of the method (Sec. 3.2 of the paper: dense recall, value filter, unified value
update) is computed by the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

F32, BF16, F16 = 0, 1, 2
_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "evomem_oracle.c")
# EVOMEM_ORACLE_LIB selects another build of the same source (the sanitizer build of the CPU tests)
_LIB = os.environ.get("EVOMEM_ORACLE_LIB") or os.path.join(_HERE, "libevomem_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, contraction off, OpenMP over queries)."""
    if os.environ.get("EVOMEM_ORACLE_LIB"):
        return _LIB                                   # built by whoever named it
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i32p, f32p, f64p = (C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_double))
        L.orc_round_to_store.argtypes = [f32p, C.c_int64, C.c_int, f32p]
        L.orc_round_to_store.restype = C.c_int
        L.orc_recall.argtypes = [f32p, C.c_int64, C.c_int, C.c_int32, f32p, C.c_int, C.c_int,
                                 i32p, f64p, C.c_int]
        L.orc_recall.restype = C.c_int
        L.orc_sims_of.argtypes = [f32p, C.c_int64, C.c_int, f32p, i32p, C.c_int, f64p]
        L.orc_sims_of.restype = C.c_int
        L.orc_rerank.argtypes = [i32p, f64p, C.c_int, f32p, C.c_double, C.c_int, i32p, f32p, f64p]
        L.orc_rerank.restype = C.c_int
        u32p, u8p = C.POINTER(C.c_uint32), C.POINTER(C.c_ubyte)
        L.orc_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.orc_philox4x32_10.restype = None
        L.orc_rerank_eps.argtypes = [i32p, f64p, C.c_int, f32p, C.c_double, C.c_int, C.c_float, C.c_uint64, C.c_uint64,
                                     C.c_uint32, i32p, f32p, f64p, u8p]
        L.orc_rerank_eps.restype = C.c_int
        L.orc_recall_masked.argtypes = [f32p, C.c_int64, C.c_int, u32p, f32p, C.c_int, u32p, u32p, C.c_int, i32p, f64p]
        L.orc_recall_masked.restype = C.c_int
        L.orc_shape_rewards.argtypes = [C.c_int, u8p, f32p, f32p, C.c_int64, C.c_int, C.c_double, C.c_double, f64p, f32p]
        L.orc_shape_rewards.restype = C.c_int
        L.orc_select_by_q.argtypes = [i32p, C.c_int64, f32p, C.c_int64, C.c_float, C.c_uint64, C.c_uint64, C.c_uint32,
                                      i32p, f32p, u8p]
        L.orc_select_by_q.restype = C.c_int64
        L.orc_update_q64.argtypes = [f32p, C.c_int64, i32p, f32p, C.c_int64, C.c_double]
        L.orc_update_q64.restype = C.c_int64
        L.orc_update_q32.argtypes = [f32p, C.c_int64, i32p, f32p, C.c_int64, C.c_float]
        L.orc_update_q32.restype = C.c_int64
        L.orc_max_threads.restype = C.c_int
        _lib = L
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def max_threads() -> int:
    return int(_load().orc_max_threads())


def round_to_store(x, dtype: int) -> np.ndarray:
    """Values the bank holds for x (round-to-nearest-even to the element type), widened to fp32."""
    x = _f32(x)
    out = np.empty_like(x)
    rc = _load().orc_round_to_store(_p(x, C.c_float), x.size, dtype, _p(out, C.c_float))
    if rc:
        raise ValueError("bad dtype")
    return out


def recall(store, queries, k1: int, id_base: int = 0, threads: int = 1):
    """Top-k1 per query by (cosine desc, id asc) over rounded bank rows `store` [N,d] and rounded
    `queries` [B,d].  Returns (ids int32 [B,k1], sims float64 [B,k1])."""
    store, queries = _f32(store), _f32(queries)
    N, d = store.shape
    B = queries.shape[0]
    assert queries.shape[1] == d
    ids = np.empty((B, k1), np.int32)
    sims = np.empty((B, k1), np.float64)
    rc = _load().orc_recall(_p(store, C.c_float), N, d, id_base, _p(queries, C.c_float), B, k1,
                            _p(ids, C.c_int32), _p(sims, C.c_double), threads)
    if rc:
        raise RuntimeError(f"orc_recall failed rc={rc}")
    return ids, sims


def merge_recall(parts, k1: int):
    """Combine per-chunk recall results [(ids, sims), ...] of the same queries into the top-k1 of
    the union, same order rule.  (A selection of already-computed pairs; no new arithmetic.)"""
    ids = np.concatenate([p[0] for p in parts], axis=1)
    sims = np.concatenate([p[1] for p in parts], axis=1)
    out_i = np.full((ids.shape[0], k1), -1, np.int32)
    out_s = np.full((ids.shape[0], k1), -np.inf, np.float64)
    for b in range(ids.shape[0]):
        keep = ids[b] >= 0
        i, s = ids[b][keep], sims[b][keep]
        order = np.lexsort((i, -s))[:k1]
        out_i[b, :order.size] = i[order]
        out_s[b, :order.size] = s[order]
    return out_i, out_s


def sims_of(store, query, ids) -> np.ndarray:
    store, query = _f32(store), _f32(query)
    ids = np.ascontiguousarray(ids, np.int32)
    out = np.empty(ids.size, np.float64)
    _load().orc_sims_of(_p(store, C.c_float), store.shape[0], store.shape[1], _p(query, C.c_float),
                        _p(ids, C.c_int32), ids.size, _p(out, C.c_double))
    return out


def rerank(cand_ids, cand_sims, qtable, lam: float, k2: int):
    """Value filter for ONE query: returns (ids int32 [k2], scores float32 [k2], scores float64 [k2])."""
    cand_ids = np.ascontiguousarray(cand_ids, np.int32)
    cand_sims = np.ascontiguousarray(cand_sims, np.float64)
    keep = cand_ids >= 0
    cand_ids, cand_sims = np.ascontiguousarray(cand_ids[keep]), np.ascontiguousarray(cand_sims[keep])
    qtable = _f32(qtable)
    ids = np.empty(k2, np.int32)
    s32 = np.empty(k2, np.float32)
    s64 = np.empty(k2, np.float64)
    rc = _load().orc_rerank(_p(cand_ids, C.c_int32), _p(cand_sims, C.c_double), cand_ids.size,
                            _p(qtable, C.c_float), lam, k2, _p(ids, C.c_int32), _p(s32, C.c_float),
                            _p(s64, C.c_double))
    if rc:
        raise RuntimeError("orc_rerank failed")
    return ids, s32, s64


def recall_masked(store, tags, queries, allow, exclude, k1: int):
    """Top-k1 among the entries each query accepts (type bit set in allow[b], group != exclude[b])."""
    store, queries = _f32(store), _f32(queries)
    tags, allow, exclude = (np.ascontiguousarray(a, np.uint32) for a in (tags, allow, exclude))
    B = queries.shape[0]
    ids = np.empty((B, k1), np.int32)
    sims = np.empty((B, k1), np.float64)
    rc = _load().orc_recall_masked(_p(store, C.c_float), store.shape[0], store.shape[1], _p(tags, C.c_uint32),
                                   _p(queries, C.c_float), B, _p(allow, C.c_uint32), _p(exclude, C.c_uint32), k1,
                                   _p(ids, C.c_int32), _p(sims, C.c_double))
    if rc:
        raise RuntimeError("orc_recall_masked failed")
    return ids, sims


def philox4x32_10(ctr, key):
    """Philox-4x32-10 block: ctr 4 and key 2 uint32 words -> 4 uint32 words."""
    ctr = np.ascontiguousarray(ctr, np.uint32)
    key = np.ascontiguousarray(key, np.uint32)
    out = np.empty(4, np.uint32)
    _load().orc_philox4x32_10(_p(ctr, C.c_uint32), _p(key, C.c_uint32), _p(out, C.c_uint32))
    return out


def rerank_eps(cand_ids, cand_sims, qtable, lam: float, k2: int, eps: float, seed: int, step: int, query_index: int):
    """Epsilon-greedy slot filling for ONE query (Sec. 3.3): returns (ids, scores f32, scores f64, explored u8)."""
    cand_ids = np.ascontiguousarray(cand_ids, np.int32)
    cand_sims = np.ascontiguousarray(cand_sims, np.float64)
    keep = cand_ids >= 0
    cand_ids, cand_sims = np.ascontiguousarray(cand_ids[keep]), np.ascontiguousarray(cand_sims[keep])
    qtable = _f32(qtable)
    ids = np.empty(k2, np.int32)
    s32 = np.empty(k2, np.float32)
    s64 = np.empty(k2, np.float64)
    ex = np.empty(k2, np.uint8)
    rc = _load().orc_rerank_eps(_p(cand_ids, C.c_int32), _p(cand_sims, C.c_double), cand_ids.size,
                                _p(qtable, C.c_float), lam, k2, float(np.float32(eps)), seed, step, query_index,
                                _p(ids, C.c_int32), _p(s32, C.c_float), _p(s64, C.c_double), _p(ex, C.c_ubyte))
    if rc:
        raise RuntimeError("orc_rerank_eps failed")
    return ids, s32, s64, ex


def shape_rewards(stage: int, feasible, latency, best_latency, normalise: bool, sigma_min: float = 0.1,
                  clip: float = 0.0, state=None):
    """Stage rewards (Sec. 3.3 / 3.4) with optional online normalisation (App. A).  Returns (rewards f32,
    new state [count, sum, sum of squares])."""
    feasible = np.ascontiguousarray(feasible, np.uint8)
    latency, best_latency = _f32(latency), _f32(best_latency)
    st = np.zeros(3, np.float64) if state is None else np.ascontiguousarray(state, np.float64).copy()
    out = np.empty(feasible.size, np.float32)
    rc = _load().orc_shape_rewards(stage, _p(feasible, C.c_ubyte), _p(latency, C.c_float), _p(best_latency, C.c_float),
                                   feasible.size, int(normalise), sigma_min, clip, _p(st, C.c_double), _p(out, C.c_float))
    if rc:
        raise RuntimeError("orc_shape_rewards failed")
    return out, st


def select_by_q(set_ids, set_offsets, qtable, eps: float = 0.0, seed: int = 0, step: int = 0):
    """Start-point selection (Sec. 3.4) for G sets given as one id array and G + 1 offsets into it.
    Returns (ids int32[G], values f32[G], explored u8[G], number of ids that are no members)."""
    set_ids = np.ascontiguousarray(set_ids, np.int32)
    off = np.ascontiguousarray(set_offsets, np.int64)
    qtable = _f32(qtable)
    G = off.size - 1
    out_id, out_q, ex = np.empty(G, np.int32), np.empty(G, np.float32), np.empty(G, np.uint8)
    skipped = 0
    for g in range(G):
        part = np.ascontiguousarray(set_ids[off[g]:off[g + 1]])
        one_id, one_q, one_ex = np.empty(1, np.int32), np.empty(1, np.float32), np.empty(1, np.uint8)
        skipped += _load().orc_select_by_q(_p(part, C.c_int32), part.size, _p(qtable, C.c_float), qtable.size,
                                           float(np.float32(eps)), seed, step, g,
                                           _p(one_id, C.c_int32), _p(one_q, C.c_float), _p(one_ex, C.c_ubyte))
        out_id[g], out_q[g], ex[g] = one_id[0], one_q[0], one_ex[0]
    return out_id, out_q, ex, int(skipped)


def update_q64(qtable, ids, rewards, alpha: float):
    """Sequential value update, fp64 state; returns (new table fp32, number of skipped ids)."""
    q = _f32(qtable).copy()
    ids = np.ascontiguousarray(ids, np.int32)
    rewards = _f32(rewards)
    skipped = _load().orc_update_q64(_p(q, C.c_float), q.size, _p(ids, C.c_int32),
                                     _p(rewards, C.c_float), ids.size, alpha)
    return q, int(skipped)


def update_q32(qtable, ids, rewards, alpha: float):
    """Sequential value update carried in fp32 (bit-exact target of a sequential fp32 fold)."""
    q = _f32(qtable).copy()
    ids = np.ascontiguousarray(ids, np.int32)
    rewards = _f32(rewards)
    skipped = _load().orc_update_q32(_p(q, C.c_float), q.size, _p(ids, C.c_int32),
                                     _p(rewards, C.c_float), ids.size, np.float32(alpha))
    return q, int(skipped)


def retrieve(store, queries, qtable, k1: int, k2: int, lam: float, threads: int = 1):
    """Whole retrieval for a batch: recall then value filter.  Returns dict of arrays."""
    cid, csim = recall(store, queries, k1, threads=threads)
    B = cid.shape[0]
    ids = np.empty((B, k2), np.int32)
    sc = np.empty((B, k2), np.float32)
    sc64 = np.empty((B, k2), np.float64)
    for b in range(B):
        ids[b], sc[b], sc64[b] = rerank(cid[b], csim[b], qtable, lam, k2)
    return {"ids": ids, "scores": sc, "scores64": sc64, "cand_ids": cid, "cand_sims": csim}
