"""The stage-wise checker that judges every GPU result (tests/parity.py) is itself checked here, on
the CPU: the oracle's own output must pass with no swap counted, results that differ only inside
the allowed near-tie band must pass and be counted, and every planted fault must be rejected."""
import copy

import numpy as np
import pytest

from tests import parity

K1, K2, LAM = 16, 4, 0.5


def _unit(rng, n, d):
    x = rng.standard_normal((n, d)).astype(np.float32)
    return (x / np.linalg.norm(x, axis=1, keepdims=True)).astype(np.float32)


def _as_gpu(orc, store, q, qtab, k1=K1, k2=K2, lam=LAM):
    """What a correct library would return: the oracle's result in the library's output types."""
    r = orc.retrieve(store, q, qtab, k1, k2, float(np.float32(lam)))
    return {"ids": r["ids"].copy(), "scores": r["scores"].copy(),
            "cand_ids": r["cand_ids"].copy(), "cand_sims": r["cand_sims"].astype(np.float32)}


@pytest.fixture(scope="module")
def case(orc):
    rng = np.random.default_rng(77)
    store = _unit(rng, 1500, 24)
    q = _unit(rng, 3, 24)
    # query 1's best row exists twice more (exact ties inside the pool, ids 40 < 900 < 1400)
    store[900] = store[40]
    store[1400] = store[40]
    q[1] = store[40]
    qtab = rng.uniform(-1, 1, 1500).astype(np.float32)
    good = _as_gpu(orc, store, q, qtab)
    # the planted faults below rely on clear gaps: no neighbours within 3e-5 in the pools or just beyond them
    _, sims = orc.recall(store, q, K1 + 8)
    gaps = -np.diff(sims, axis=1)
    assert np.all((gaps > 3e-5) | (gaps == 0))
    return store, q, qtab, good


def _check(orc, case, gpu, **kw):
    store, q, qtab, _ = case
    return parity.check_retrieve(orc, store, q, qtab, kw.pop("k1", K1), kw.pop("k2", K2), LAM, gpu, **kw)


def test_oracle_output_passes_with_no_swaps(orc, case):
    stats = _check(orc, case, case[3])
    assert stats == {"boundary_swaps": 0, "order_swaps": 0, "final_swaps": 0, "queries": 3}
    assert _check(orc, case, case[3], sample=[2])["queries"] == 1


def test_pool_member_replaced_by_a_worse_row_is_rejected(orc, case):
    store, q, qtab, good = case
    ids, sims = orc.recall(store, q, K1 + 6)
    bad = copy.deepcopy(good)
    bad["cand_ids"][0, K1 - 1] = ids[0, K1 + 5]               # clearly (> 3e-5) below the k1-th best
    bad["cand_sims"][0, K1 - 1] = sims[0, K1 + 5]
    with pytest.raises(AssertionError, match="k1-th"):
        _check(orc, case, bad)


def test_exact_tie_towards_the_higher_id_is_rejected(orc, case):
    _, _, _, good = case
    assert good["cand_ids"][1, :3].tolist() == [40, 900, 1400]
    bad = copy.deepcopy(good)
    bad["cand_ids"][1, [1, 2]] = bad["cand_ids"][1, [2, 1]]
    with pytest.raises(AssertionError, match="lower id"):
        _check(orc, case, bad)


def test_pool_order_violation_is_rejected(orc, case):
    bad = copy.deepcopy(case[3])
    for key in ("cand_ids", "cand_sims"):
        bad[key][2, [5, 6]] = bad[key][2, [6, 5]]
    with pytest.raises(AssertionError, match="pool order"):
        _check(orc, case, bad)


def test_similarity_or_score_off_by_two_tolerances_is_rejected(orc, case):
    bad = copy.deepcopy(case[3])
    bad["cand_sims"][0, 3] += np.float32(2e-5)
    with pytest.raises(AssertionError, match="pool sims"):
        _check(orc, case, bad)
    bad = copy.deepcopy(case[3])
    bad["scores"][2, 1] -= np.float32(2e-5) * max(1.0, abs(float(bad["scores"][2, 1])))
    with pytest.raises(AssertionError, match="final scores"):
        _check(orc, case, bad)
    ok = copy.deepcopy(case[3])                                # half a tolerance is accepted
    ok["scores"][2, 1] -= np.float32(4e-6)
    ok["cand_sims"][0, 3] += np.float32(4e-6)
    _check(orc, case, ok)


def test_duplicate_and_foreign_ids_are_rejected(orc, case):
    bad = copy.deepcopy(case[3])
    bad["cand_ids"][0, 7] = bad["cand_ids"][0, 6]
    with pytest.raises(AssertionError, match="duplicate"):
        _check(orc, case, bad)
    bad = copy.deepcopy(case[3])                               # a final item that is not in the pool
    outside = next(i for i in range(1500) if i not in set(bad["cand_ids"][0].tolist()))
    bad["ids"][0, 2] = outside
    with pytest.raises(AssertionError, match="not in pool"):
        _check(orc, case, bad)


def test_final_items_in_the_wrong_order_or_wrongly_chosen_are_rejected(orc, case):
    store, q, qtab, good = case
    bad = copy.deepcopy(good)
    bad["ids"][0, [0, 1]] = bad["ids"][0, [1, 0]]              # scores left in place: ids disagree
    with pytest.raises(AssertionError, match="final slot"):
        _check(orc, case, bad)
    bad = copy.deepcopy(good)                                  # last slot takes the pool's worst-scored member
    full_ids, s32, _ = orc.rerank(good["cand_ids"][0], orc.sims_of(store, q[0], good["cand_ids"][0]), qtab,
                                  float(np.float32(LAM)), K1)
    bad["ids"][0, K2 - 1], bad["scores"][0, K2 - 1] = full_ids[-1], s32[-1]
    with pytest.raises(AssertionError):
        _check(orc, case, bad)


def test_wrong_padding_is_rejected(orc):
    rng = np.random.default_rng(78)
    store, q = _unit(rng, 10, 8), _unit(rng, 2, 8)
    qtab = rng.uniform(-1, 1, 10).astype(np.float32)
    good = _as_gpu(orc, store, q, qtab, k1=16, k2=12)          # k1 > N: six empty pool slots, two empty final slots
    assert np.all(good["cand_ids"][:, 10:] == -1) and np.all(good["ids"][:, 10:] == -1)
    chk = lambda g: parity.check_retrieve(orc, store, q, qtab, 16, 12, LAM, g)
    assert chk(good)["queries"] == 2
    for key, col, val in (("cand_ids", 12, 3), ("cand_sims", 11, 0.0), ("ids", 11, 3), ("scores", 10, 0.0)):
        bad = copy.deepcopy(good)
        bad[key][1, col] = val
        with pytest.raises(AssertionError):
            chk(bad)
    bad = copy.deepcopy(good)                                  # a -1 inside the used part of the pool
    bad["cand_ids"][0, 4] = -1
    with pytest.raises(AssertionError):
        chk(bad)


def test_near_ties_inside_the_allowance_pass_and_are_counted(orc):
    """Two rows about 2e-6 apart at the pool boundary, two more inside the pool: taking either of the
    first pair and listing the second pair in either order is allowed (ids may differ where the
    oracle's values differ by < 1e-5), each is counted, and the final items are judged on the pool
    that was actually taken."""
    rng = np.random.default_rng(79)
    store, q = _unit(rng, 800, 24), _unit(rng, 1, 24)
    qtab = rng.uniform(-1, 1, 800).astype(np.float32)
    ids, _ = orc.recall(store, q, K1)
    twin_of = {int(ids[0, K1 - 2]): 790, int(ids[0, 4]): 795}      # the inner twin shifts the outer pair to the boundary
    for src, dst in twin_of.items():
        row = store[src].astype(np.float64)
        step = q[0].astype(np.float64) - row * float(row @ q[0])      # towards the query: raises the cosine
        store[dst] = (row + 2e-6 * step / np.linalg.norm(step)).astype(np.float32)
    ids, sims = orc.recall(store, q, K1 + 1)
    assert 0 < sims[0, K1 - 1] - sims[0, K1] < 5e-6 and {int(ids[0, K1 - 1]), int(ids[0, K1])} == {int(list(twin_of)[0]), 790}
    j = ids[0].tolist().index(795) if 795 in ids[0].tolist() else None
    assert j is not None and 0 < sims[0, j] - sims[0, j + 1] < 5e-6
    chk = lambda g: parity.check_retrieve(orc, store, q, qtab, K1, K2, LAM, g)
    good = _as_gpu(orc, store, q, qtab)
    assert chk(good) == {"boundary_swaps": 0, "order_swaps": 0, "final_swaps": 0, "queries": 1}
    # the other member of the boundary pair in the pool, the inner pair the other way round
    pool = ids[0, :K1].copy()
    pool[K1 - 1] = ids[0, K1]
    pool[[j, j + 1]] = pool[[j + 1, j]]
    true = orc.sims_of(store, q[0], pool)
    f_ids, f_s32, _ = orc.rerank(pool, true, qtab, float(np.float32(LAM)), K2)
    alt = {"ids": f_ids[None], "scores": f_s32[None], "cand_ids": pool[None], "cand_sims": true.astype(np.float32)[None]}
    stats = chk(alt)
    assert stats["boundary_swaps"] == 1 and stats["order_swaps"] == 1 and stats["queries"] == 1
    # the same pool with the final items of the ORACLE's pool: a different pool has different
    # z-scores, so those scores are off by far more than the tolerance
    stale = dict(alt, ids=good["ids"], scores=good["scores"])
    if not np.allclose(good["scores"], alt["scores"], atol=2e-5, rtol=0):
        with pytest.raises(AssertionError):
            chk(stale)


def test_near_tie_in_the_final_scores_is_counted_as_a_swap(orc):
    """Two pool members whose scores differ by < 1e-5 may come out in either order (lambda = 1: the
    score is the z-score of the value alone, so two values ten fp32 steps apart give such a pair)."""
    rng = np.random.default_rng(80)
    store, q = _unit(rng, 600, 16), _unit(rng, 1, 16)
    qtab = rng.uniform(-1, 1, 600).astype(np.float32)
    ids, sims = orc.recall(store, q, K1)
    a, b = int(ids[0, 3]), int(ids[0, 9])
    qtab[a] = np.float32(2.0)
    qtab[b] = np.nextafter(np.float32(2.0), np.float32(0), dtype=np.float32)
    for _ in range(9):
        qtab[b] = np.nextafter(qtab[b], np.float32(0), dtype=np.float32)
    full, _, s64 = orc.rerank(ids[0], sims[0], qtab, 1.0, K1)
    assert full[0] == a and full[1] == b and 0 < s64[0] - s64[1] < 1e-5 and s64[1] - s64[2] > 1e-3
    chk = lambda g: parity.check_retrieve(orc, store, q, qtab, K1, K2, 1.0, g)
    good = _as_gpu(orc, store, q, qtab, lam=1.0)
    assert chk(good)["final_swaps"] == 0
    swapped = copy.deepcopy(good)
    swapped["ids"][0, [0, 1]] = swapped["ids"][0, [1, 0]]
    stats = chk(swapped)
    assert stats["final_swaps"] == 2 and stats["boundary_swaps"] == 0
    # the same exchange between items whose scores are clearly apart is a fault
    bad = copy.deepcopy(good)
    bad["ids"][0, [1, 2]] = bad["ids"][0, [2, 1]]
    with pytest.raises(AssertionError, match="final slot"):
        chk(bad)
