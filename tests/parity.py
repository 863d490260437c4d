"""Stage-wise comparison of the GPU library with the CPU oracle (used by the GPU tests and smoke).

Stage A  candidate pool: the GPU's pool must be the oracle's top-k1 by (similarity desc, id asc).
         An id present on one side only is accepted only if its oracle similarity is within 1e-5 of
         the oracle's k1-th best (near-tie at the boundary); positions may differ only between
         entries whose oracle similarities differ by < 1e-5.
Stage B  value filter: the oracle re-ranks the GPU's OWN pool (a legal boundary swap changes the
         pool's mean and deviation and with it every score), then final ids must agree except
         between entries whose oracle scores differ by < 1e-5, and scores must agree within
         1e-5 * max(1, |score|)  (z-scores are O(1) and cross zero, so a purely relative bound
         is ill-posed).
"""
from __future__ import annotations

import numpy as np

TOL = 1e-5


def check_retrieve(orc, store_rounded, queries_rounded, qtable, k1, k2, lam, gpu, ora_recall=None,
                   sample=None, threads=8):
    """gpu: dict ids, scores, cand_ids, cand_sims (numpy).  Returns a dict of counts."""
    B = queries_rounded.shape[0]
    qs = range(B) if sample is None else sample
    lam = float(np.float32(lam))
    N = store_rounded.shape[0]
    k1e, k2e = min(k1, N), min(k2, min(k1, N))
    if ora_recall is None:
        sel = np.ascontiguousarray(queries_rounded[list(qs)])
        oi, os_ = orc.recall(store_rounded, sel, k1, threads=threads)
    else:
        oi, os_ = ora_recall
    stats = {"boundary_swaps": 0, "order_swaps": 0, "final_swaps": 0, "queries": 0}
    for row, b in enumerate(qs):
        gi = gpu["cand_ids"][b]
        assert np.all(gi[:k1e] >= 0) and np.all(gi[k1e:] == -1), f"query {b}: pool padding wrong"
        assert np.all(np.isneginf(gpu["cand_sims"][b][k1e:]))
        gi = gi[:k1e]
        assert len(set(gi.tolist())) == k1e, f"query {b}: duplicate ids in pool"
        o_ids, o_sims = oi[row][:k1e], os_[row][:k1e]
        g_true = orc.sims_of(store_rounded, queries_rounded[b], gi)      # oracle sims of the GPU's ids
        kth = o_sims[-1]
        only_g = set(gi.tolist()) - set(o_ids.tolist())
        only_o = set(o_ids.tolist()) - set(gi.tolist())
        assert len(only_g) == len(only_o)
        for i in only_g:
            s = g_true[gi.tolist().index(i)]
            assert abs(s - kth) < TOL, f"query {b}: id {i} in GPU pool has sim {s}, k1-th best is {kth}"
        for i in only_o:
            s = o_sims[o_ids.tolist().index(i)]
            assert abs(s - kth) < TOL, f"query {b}: oracle id {i} (sim {s}) missing from GPU pool, k1-th {kth}"
        stats["boundary_swaps"] += len(only_g)
        # order inside the GPU pool must follow the oracle's sims (desc) / id (asc) up to near-ties
        for j in range(k1e - 1):
            a, c = g_true[j], g_true[j + 1]
            if a > c:
                continue
            if a == c:      # exact tie (e.g. duplicate rows): the lower id must come first
                assert gi[j] < gi[j + 1], f"query {b}: tie at {j} not broken towards the lower id"
                continue
            assert c - a < TOL, f"query {b}: pool order violated at {j}: {a} < {c}"
            stats["order_swaps"] += 1
        # reported similarities
        gs = gpu["cand_sims"][b][:k1e].astype(np.float64)
        assert np.all(np.abs(gs - g_true) <= TOL * np.maximum(1.0, np.abs(g_true))), f"query {b}: pool sims off"
        # stage B on the GPU's own pool
        r_ids, r_s32, r_s64 = orc.rerank(gi, g_true, qtable, lam, k2)
        f_ids, f_sc = gpu["ids"][b], gpu["scores"][b]
        assert np.all(f_ids[k2e:] == -1) and np.all(np.isneginf(f_sc[k2e:]))
        if not np.array_equal(f_ids[:k2e], r_ids[:k2e]):
            full_ids, _, full_sc = orc.rerank(gi, g_true, qtable, lam, k1e)
            score_of = dict(zip(full_ids.tolist(), full_sc.tolist()))
            for j in range(k2e):
                if f_ids[j] != r_ids[j]:
                    assert int(f_ids[j]) in score_of, f"query {b}: final id {f_ids[j]} not in pool"
                    assert abs(score_of[int(f_ids[j])] - r_s64[j]) < TOL, (
                        f"query {b}: final slot {j}: gpu id {f_ids[j]} score {score_of[int(f_ids[j])]} vs "
                        f"oracle id {r_ids[j]} score {r_s64[j]}")
                    stats["final_swaps"] += 1
        ref = r_s64[:k2e]
        assert np.all(np.abs(f_sc[:k2e].astype(np.float64) - ref) <= TOL * np.maximum(1.0, np.abs(ref))), (
            f"query {b}: final scores off: {f_sc[:k2e]} vs {ref}")
        stats["queries"] += 1
    return stats


def gpu_retrieve(bank, torch, queries_np, stage, k1, k2, lam):
    q = torch.from_numpy(np.ascontiguousarray(queries_np)).to(bank.device)
    ids, sc, cid, csim = bank.retrieve(q, stage, k1, k2, float(lam), want_candidates=True)
    torch.cuda.synchronize()
    return {"ids": ids.cpu().numpy(), "scores": sc.cpu().numpy(),
            "cand_ids": cid.cpu().numpy(), "cand_sims": csim.cpu().numpy()}
