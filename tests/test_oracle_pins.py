"""Pins for the CPU oracle: every function is checked against something other than itself --
hand calculations (tests/golden), brute force written out in Python, closed forms from App. A of
the paper, invariants, and library routines (NumPy fp64 matmul + sort, NumPy/PyTorch rounding)."""
import json
import math
import os

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")
F32, BF16, F16 = 0, 1, 2


def _unit(rng, n, d):
    x = rng.standard_normal((n, d)).astype(np.float32)
    return (x / np.linalg.norm(x, axis=1, keepdims=True)).astype(np.float32)


# ----------------------------------------------------------------------------- rounding

def test_round_bf16_matches_torch_and_ties(orc):
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * s for s in (1e-30, 1e-3, 1, 1e5, 1e30)])
    x = np.concatenate([x, np.array([0.0, -0.0, np.inf, -np.inf, 3.3895e38, 1e-45], np.float32)])
    got = orc.round_to_store(x, BF16)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # hand-made halfway cases: bf16 has 8 significant bits, so 1+2^-8 is a tie
    ties = np.array([1 + 2.0**-8, 1 + 3 * 2.0**-8, 1 + 2.0**-8 + 2.0**-20, 1 + 2.0**-8 - 2.0**-20], np.float32)
    exp = np.array([1.0, 1 + 2.0**-6, 1 + 2.0**-7, 1.0], np.float32)
    assert np.array_equal(orc.round_to_store(ties, BF16), exp)


def test_round_f16_matches_numpy_and_ties(orc):
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * s
                        for s in (1e-9, 6e-8, 1e-5, 1e-3, 1, 300, 7e4)])
    x = np.concatenate([x, np.array([0.0, -0.0, np.inf, -np.inf, 65504, 65519.99, 65520, 2.0**-24,
                                     2.0**-25, 2.0**-25 * 1.0001, 3 * 2.0**-25], np.float32)])
    got = orc.round_to_store(x, F16)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).astype(np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    ties = np.array([1 + 2.0**-11, 1 + 3 * 2.0**-11, 2048 + 1, 2048 + 3], np.float32)
    exp = np.array([1.0, 1 + 2.0**-9, 2048, 2052], np.float32)
    assert np.array_equal(orc.round_to_store(ties, F16), exp)


def test_round_f32_is_identity(orc):
    x = np.random.default_rng(3).standard_normal(1000).astype(np.float32)
    assert np.array_equal(orc.round_to_store(x, F32), x)


# ----------------------------------------------------------------------------- recall

def _brute_recall(store, q, k1):
    """Definition written out with Python floats (fp64): cosine against every row, full sort."""
    out = []
    for b in range(q.shape[0]):
        nq = math.sqrt(sum(float(v) * float(v) for v in q[b]))
        pairs = []
        for n in range(store.shape[0]):
            ne = math.sqrt(sum(float(v) * float(v) for v in store[n]))
            dot = sum(float(a) * float(c) for a, c in zip(q[b], store[n]))
            pairs.append((-(dot / (nq * ne)), n))
        pairs.sort()
        out.append(pairs[:k1])
    return out


def test_recall_brute_force_tiny_with_ties(orc):
    rng = np.random.default_rng(4)
    store = rng.integers(-3, 4, size=(48, 6)).astype(np.float32)
    store[np.abs(store).sum(1) == 0, 0] = 1
    store[17] = store[5]          # exact duplicates: identical sims, lower id must come first
    store[40] = store[5]
    store[9] = store[33]
    q = np.stack([store[5], store[33] * 2.5, rng.integers(-3, 4, 6).astype(np.float32) + 0.5])
    ids, sims = orc.recall(store, q, 12)
    brute = _brute_recall(store, q, 12)
    for b in range(3):
        assert [p[1] for p in brute[b]] == ids[b].tolist()
        assert np.allclose([-p[0] for p in brute[b]], sims[b], rtol=0, atol=1e-14)
    assert ids[0, :3].tolist() == [5, 17, 40] and abs(sims[0, 0] - 1.0) < 1e-14
    assert ids[1, :2].tolist() == [9, 33]


def test_recall_one_hot_bank_and_self_query(orc):
    d = 16
    store = np.eye(d, dtype=np.float32) * np.arange(1, d + 1, dtype=np.float32)[:, None]   # scaled one-hots
    q = np.zeros((2, d), np.float32)
    q[0, 3] = 5.0
    q[1, 7], q[1, 2] = 3.0, 4.0
    ids, sims = orc.recall(store, q, d)
    assert ids[0, 0] == 3 and sims[0, 0] == 1.0 and np.all(sims[0, 1:] == 0.0)
    assert ids[0, 1:].tolist() == [i for i in range(d) if i != 3]        # all tied at 0: id ascending
    assert ids[1, :2].tolist() == [2, 7] and np.allclose(sims[1, :2], [0.8, 0.6], atol=1e-15)


def test_recall_matches_numpy_gemm_and_sort(orc):
    rng = np.random.default_rng(5)
    store = rng.standard_normal((3000, 96)).astype(np.float32) * rng.uniform(0.1, 10, (3000, 1)).astype(np.float32)
    q = rng.standard_normal((7, 96)).astype(np.float32)
    ids, sims = orc.recall(store, q, 50, threads=2)
    S = (q.astype(np.float64) @ store.astype(np.float64).T)
    S /= np.linalg.norm(q.astype(np.float64), axis=1)[:, None]
    S /= np.linalg.norm(store.astype(np.float64), axis=1)[None, :]
    for b in range(7):
        order = np.lexsort((np.arange(3000), -S[b]))[:50]
        assert np.array_equal(order, ids[b])
        assert np.allclose(S[b][order], sims[b], rtol=0, atol=1e-13)


def test_recall_scale_and_permutation_invariance(orc):
    rng = np.random.default_rng(6)
    store = rng.standard_normal((500, 32)).astype(np.float32)
    q = rng.standard_normal((4, 32)).astype(np.float32)
    ids, sims = orc.recall(store, q, 20)
    # power-of-two scalings are exact in floating point: sims must not move at all beyond 1 ulp
    ids2, sims2 = orc.recall(store * np.float32(4.0), q * np.float32(0.125), 20)
    assert np.array_equal(ids, ids2) and np.allclose(sims, sims2, rtol=0, atol=1e-15)
    perm = rng.permutation(500)
    ids3, sims3 = orc.recall(store[perm], q, 20)
    assert np.array_equal(perm[ids3], ids) and np.allclose(sims3, sims, rtol=0, atol=1e-15)


def test_recall_padding_and_chunk_merge(orc):
    rng = np.random.default_rng(7)
    store = rng.standard_normal((10, 8)).astype(np.float32)
    q = rng.standard_normal((2, 8)).astype(np.float32)
    ids, sims = orc.recall(store, q, 16)
    assert np.all(ids[:, 10:] == -1) and np.all(np.isneginf(sims[:, 10:])) and np.all(ids[:, :10] >= 0)
    big = rng.standard_normal((300, 8)).astype(np.float32)
    whole = orc.recall(big, q, 16)
    parts = [orc.recall(big[a:a + 100], q, 16, id_base=a) for a in (0, 100, 200)]
    merged = orc.merge_recall(parts, 16)
    assert np.array_equal(whole[0], merged[0]) and np.array_equal(whole[1], merged[1])


def test_recall_uses_stored_representation(orc):
    """The cosine is taken between the rounded vectors: rounding first, then an fp64 library GEMM."""
    rng = np.random.default_rng(8)
    raw = _unit(rng, 400, 64)
    q = _unit(rng, 3, 64)
    for dt, tdt in ((BF16, torch.bfloat16), (F16, torch.float16)):
        st = torch.from_numpy(raw).to(tdt).to(torch.float64).numpy()
        qq = torch.from_numpy(q).to(tdt).to(torch.float64).numpy()
        S = (qq @ st.T) / np.linalg.norm(qq, axis=1)[:, None] / np.linalg.norm(st, axis=1)[None, :]
        ids, sims = orc.recall(orc.round_to_store(raw, dt), orc.round_to_store(q, dt), 10)
        for b in range(3):
            order = np.lexsort((np.arange(400), -S[b]))[:10]
            assert np.array_equal(order, ids[b]) and np.allclose(S[b][order], sims[b], atol=1e-13, rtol=0)


# ----------------------------------------------------------------------------- similarities of given ids

def test_sims_of_brute_force_on_integer_vectors(orc):
    """Cosines of named ids against the definition written out with Python floats; ids outside the
    bank (negative, N, far beyond) read -inf; the order of the id list is the order of the output."""
    rng = np.random.default_rng(41)
    store = rng.integers(-4, 5, size=(37, 7)).astype(np.float32)
    store[np.abs(store).sum(1) == 0, 2] = 1
    q = (rng.integers(-4, 5, size=7) + 0.25).astype(np.float32)
    ids = np.array([36, 0, 5, 5, -1, 37, 12, 1000000, 20, -7], np.int32)
    got = orc.sims_of(store, q, ids)
    nq = math.sqrt(sum(float(v) * float(v) for v in q))
    for j, i in enumerate(ids):
        if i < 0 or i >= 37:
            assert got[j] == -np.inf
            continue
        ne = math.sqrt(sum(float(v) * float(v) for v in store[i]))
        dot = sum(float(a) * float(c) for a, c in zip(q, store[i]))
        assert abs(got[j] - dot / (nq * ne)) < 1e-15
    assert got[2] == got[3]                                    # the same id twice: the same value twice
    # special cases with closed forms: a row against itself, its negative, an orthogonal one-hot row
    eye = np.eye(5, dtype=np.float32) * np.array([1, 2, 3, 4, 5], np.float32)[:, None]
    s = orc.sims_of(eye, eye[2] * 7, np.arange(5, dtype=np.int32))
    assert np.array_equal(s, np.array([0, 0, 1, 0, 0], np.float64))
    assert orc.sims_of(eye, -eye[3], np.array([3], np.int32))[0] == -1.0


def test_sims_of_matches_numpy_on_rounded_rows_and_recall(orc):
    """On rows rounded to the 16-bit types: an fp64 library product on the rounded values, and the
    similarities `recall` reports for the ids it returns (the same arithmetic reached another way)."""
    rng = np.random.default_rng(42)
    raw, q = _unit(rng, 900, 96), _unit(rng, 4, 96)
    for dt in (F32, BF16, F16):
        st, qq = orc.round_to_store(raw, dt), orc.round_to_store(q, dt)
        s64, q64 = st.astype(np.float64), qq.astype(np.float64)
        S = (q64 @ s64.T) / np.linalg.norm(q64, axis=1)[:, None] / np.linalg.norm(s64, axis=1)[None, :]
        r_ids, r_sims = orc.recall(st, qq, 25)
        for b in range(4):
            pick = rng.permutation(900)[:60].astype(np.int32)
            assert np.allclose(orc.sims_of(st, qq[b], pick), S[b][pick], atol=1e-13, rtol=0)
            assert np.array_equal(orc.sims_of(st, qq[b], r_ids[b]), r_sims[b])
    # the norm of the ROW must enter (a dropped row norm leaves unnormalised rows wrong)
    scaled = (raw * rng.uniform(0.5, 3.0, size=(900, 1))).astype(np.float32)
    pick = np.arange(0, 900, 7, dtype=np.int32)
    assert np.allclose(orc.sims_of(scaled, q[0], pick), orc.sims_of(raw, q[0], pick), atol=1e-6, rtol=0)
    # ... and that of the query
    assert np.allclose(orc.sims_of(raw, q[0] * 5, pick), orc.sims_of(raw, q[0], pick), atol=1e-7, rtol=0)


# ----------------------------------------------------------------------------- value filter

def test_rerank_hand_example(orc):
    g = json.load(open(os.path.join(GOLD, "rerank_hand.json")))
    qt = np.zeros(32, np.float32)
    for k, v in g["q_of_id"].items():
        qt[int(k)] = v
    ids, s32, s64 = orc.rerank(g["cand_ids"], g["cand_sims"], qt, g["lam"], 4)
    assert ids.tolist() == g["expected_order"]
    assert np.allclose(s64, g["expected_scores"], rtol=0, atol=g["tolerance"])
    assert np.array_equal(s32, s64.astype(np.float32))


def _brute_rerank(ids, sims, qt, lam, k2):
    k = len(ids)
    qs = [float(qt[i]) for i in ids]

    def z(v):
        m = sum(v) / k
        sd = math.sqrt(sum((a - m) ** 2 for a in v) / k)
        return [(a - m) / (sd + 1e-6) for a in v]
    zs, zq = z([float(s) for s in sims]), z(qs)
    sc = sorted((-((1 - lam) * a + lam * b), i) for a, b, i in zip(zs, zq, ids))
    return [i for _, i in sc[:k2]], [-s for s, _ in sc[:k2]]


def test_rerank_brute_force(orc):
    rng = np.random.default_rng(9)
    qt = rng.uniform(-1, 1, 200).astype(np.float32)
    for lam in (0.0, 0.25, 0.5, 1.0):
        ids = rng.choice(200, 24, replace=False).astype(np.int32)
        sims = np.sort(rng.uniform(0.2, 0.9, 24))[::-1].copy()
        got_i, _, got_s = orc.rerank(ids, sims, qt, lam, 6)
        bi, bs = _brute_rerank(ids.tolist(), sims.tolist(), qt, lam, 6)
        assert got_i.tolist() == bi and np.allclose(got_s, bs, rtol=0, atol=1e-12)


def test_rerank_lambda0_is_similarity_ranking_lambda1_is_q_ranking(orc):
    rng = np.random.default_rng(10)
    qt = rng.uniform(-1, 1, 500).astype(np.float32)
    qt[[3, 77, 130]] = 0.75                                    # tied Q values: lower id first at lam=1
    ids = np.array(sorted(rng.choice(500, 40, replace=False).tolist() + [3, 77, 130]), np.int32)
    ids = np.unique(ids)
    rng.shuffle(ids)
    sims = np.sort(rng.uniform(0, 1, ids.size))[::-1].copy()
    i0, _, s0 = orc.rerank(ids, sims, qt, 0.0, 8)
    assert np.array_equal(i0, ids[:8])                          # pure similarity ranking (heuristic baseline)
    assert np.all(np.diff(s0) <= 0)
    i1, _, s1 = orc.rerank(ids, sims, qt, 1.0, ids.size)
    want = sorted(ids.tolist(), key=lambda i: (-float(qt[i]), i))
    assert i1.tolist() == want                                  # monotone in Q, ties to lower id
    qv = qt[i1].astype(np.float64)
    assert np.all(np.diff(s1) <= 1e-15) and np.all((np.diff(qv) < 0) | (np.diff(s1) == 0))


def test_rerank_zscore_identities_affine_invariance_and_sets(orc):
    rng = np.random.default_rng(11)
    qt = rng.uniform(-1, 1, 300).astype(np.float64)
    ids = rng.choice(300, 32, replace=False).astype(np.int32)
    sims = np.sort(rng.uniform(0.5, 0.6, 32))[::-1].copy()
    _, _, s = orc.rerank(ids, sims, qt.astype(np.float32), 0.0, 32)     # scores == z(sim), sorted
    sd = sims.std()                                                       # numpy default: population
    assert abs(s.sum()) < 1e-9 and abs(s.var() - (sd / (sd + 1e-6)) ** 2) < 1e-9
    assert abs(s[0] - (sims[0] - sims.mean()) / (sd + 1e-6)) < 1e-9
    # Q -> aQ + b with a > 0 (power-of-two a, small-integer-over-power-of-two b keep fp32 exact)
    qa = (qt.astype(np.float32) * np.float32(0.5) + np.float32(0.25)).astype(np.float32)
    i1, _, s1 = orc.rerank(ids, sims, qt.astype(np.float32), 0.5, 8)
    i2, _, s2 = orc.rerank(ids, sims, qa, 0.5, 8)
    assert np.array_equal(i1, i2) and np.allclose(s1, s2, rtol=0, atol=2e-6)
    # k2 == k1 returns the whole pool
    i3, _, _ = orc.rerank(ids, sims, qt.astype(np.float32), 0.7, 32)
    assert sorted(i3.tolist()) == sorted(ids.tolist())
    # constant Q: ranking is the similarity ranking for any lam < 1, z(Q) == 0
    i4, _, s4 = orc.rerank(ids, sims, np.full(300, 0.3, np.float32), 0.9, 8)
    assert np.array_equal(i4, ids[:8]) and np.allclose(s4, 0.1 * s[:8], atol=1e-9)
    # a pool of one: z == 0
    i5, s5, _ = orc.rerank(ids[:1], sims[:1], qt.astype(np.float32), 0.5, 2)
    assert i5.tolist() == [ids[0], -1] and s5[0] == 0.0 and np.isneginf(s5[1])


# ----------------------------------------------------------------------------- value update

def test_update_hand_example(orc):
    g = json.load(open(os.path.join(GOLD, "q_update_hand.json")))
    for t in range(1, len(g["rewards"]) + 1):
        for fn in (orc.update_q64, orc.update_q32):
            q, sk = fn(np.array([9.0, g["q0"], 9.0], np.float32), [1] * t, g["rewards"][:t], g["alpha"])
            assert sk == 0 and q.tolist() == [9.0, g["trajectory"][t - 1], 9.0]


def test_update_closed_form_and_constant_reward(orc):
    """Unrolled recursion from the proof of the constant-step-size lemma (App. A)."""
    rng = np.random.default_rng(12)
    alpha, t = 0.1, 37
    q0 = np.float32(0.4)
    R = rng.uniform(-1, 1, t).astype(np.float32)
    ids = np.full(t, 5, np.int32)
    table = np.zeros(9, np.float32)
    table[5] = q0
    closed = (1 - alpha) ** t * float(q0) + alpha * sum((1 - alpha) ** (t - 1 - k) * float(R[k]) for k in range(t))
    q64, _ = orc.update_q64(table, ids, R, alpha)
    q32, _ = orc.update_q32(table, ids, R, alpha)
    assert abs(float(q64[5]) - closed) < 1e-7 and abs(float(q32[5]) - closed) < 2e-6
    # a reversed reward order must give a different value (the order of duplicates matters)
    q64r, _ = orc.update_q64(table, ids, R[::-1].copy(), alpha)
    assert abs(float(q64r[5]) - closed) > 1e-3
    const = np.full(t, 0.75, np.float32)
    qc, _ = orc.update_q64(table, ids, const, alpha)
    assert abs(float(qc[5]) - (0.75 + (1 - alpha) ** t * (float(q0) - 0.75))) < 1e-7


def test_update_alpha_one_keeps_last_reward_and_skips_bad_ids(orc):
    table = np.linspace(-1, 1, 16).astype(np.float32)
    ids = np.array([3, 7, 3, -1, 3, 16, 7, 100], np.int32)
    r = np.array([0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8], np.float32)
    for fn in (orc.update_q64, orc.update_q32):
        q, skipped = fn(table, ids, r, 1.0)
        assert skipped == 3 and q[3] == np.float32(0.5) and q[7] == np.float32(0.7)
        mask = np.ones(16, bool)
        mask[[3, 7]] = False
        assert np.array_equal(q[mask].view(np.uint32), table[mask].view(np.uint32))   # others bit-unchanged


def test_update_bounded_and_order_free_for_distinct_ids(orc):
    rng = np.random.default_rng(13)
    table = rng.uniform(-1, 1, 1000).astype(np.float32)
    ids = rng.integers(0, 1000, 20000).astype(np.int32)
    r = rng.uniform(-1, 1, 20000).astype(np.float32)
    for fn in (orc.update_q64, orc.update_q32):
        q, _ = fn(table, ids, r, 0.3)
        assert np.all(np.abs(q) <= 1.0)             # boundedness lemma (App. A): convex combinations
    d_ids = rng.permutation(1000)[:400].astype(np.int32)
    d_r = rng.uniform(-1, 1, 400).astype(np.float32)
    p = rng.permutation(400)
    a, _ = orc.update_q32(table, d_ids, d_r, 0.2)
    b, _ = orc.update_q32(table, d_ids[p], d_r[p], 0.2)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    q32, _ = orc.update_q32(table, ids, r, 0.3)
    q64, _ = orc.update_q64(table, ids, r, 0.3)
    assert np.max(np.abs(q32.astype(np.float64) - q64)) < 2e-6


def test_update_ema_statistics(orc):
    """E[Q_t] = mu (1-(1-a)^t) from Q_0=0 and Var -> a/(2-a) sigma_R^2 (constant-step lemma, App. A)."""
    rng = np.random.default_rng(14)
    n, alpha, p = 40000, 0.1, 0.3
    table = np.zeros(n, np.float32)
    ids = np.arange(n, dtype=np.int32)
    for t in range(1, 61):
        table, _ = orc.update_q64(table, ids, (rng.random(n) < p).astype(np.float32), alpha)
        if t in (5, 20):
            assert abs(table.mean() - p * (1 - (1 - alpha) ** t)) < 4e-3
    assert abs(table.mean() - p) < 4e-3
    assert abs(table.var() - alpha / (2 - alpha) * p * (1 - p)) < 6e-4


def test_error_clipped_variant_is_not_what_the_oracle_computes(orc):
    """Negative control from App. A's remark: clipping the error alone lets iterates grow without
    bound; the unclipped convex-combination form stays at the reward."""
    table = np.zeros(2, np.float32)
    q, _ = orc.update_q64(table, np.zeros(500, np.int32), np.full(500, 100.0, np.float32), 0.5)
    assert abs(q[0] - 100.0) < 1e-3
    clipped = 0.0
    for _ in range(500):
        clipped += 0.5 * max(-1.0, min(1.0, 100.0 - clipped))
    assert clipped > 99.0 and abs(clipped - q[0]) < 1.0     # same limit, different path ...
    early_c, early_q = 0.0, orc.update_q64(table, np.zeros(3, np.int32), np.full(3, 100.0, np.float32), 0.5)[0][0]
    for _ in range(3):
        early_c += 0.5 * max(-1.0, min(1.0, 100.0 - early_c))
    assert abs(early_q - 87.5) < 1e-4 and early_c == 1.5    # ... the oracle follows the unclipped rule


# ----------------------------------------------------------------------------- whole retrieval

def test_retrieve_end_to_end_matches_python_definition(orc):
    rng = np.random.default_rng(15)
    store = _unit(rng, 64, 8)
    q = _unit(rng, 3, 8)
    qt = rng.uniform(-1, 1, 64).astype(np.float32)
    out = orc.retrieve(store, q, qt, 16, 4, 0.5)
    brute = _brute_recall(store, q, 16)
    for b in range(3):
        ids = [p[1] for p in brute[b]]
        sims = [-p[0] for p in brute[b]]
        bi, bs = _brute_rerank(ids, sims, qt, 0.5, 4)
        assert out["ids"][b].tolist() == bi and np.allclose(out["scores64"][b], bs, atol=1e-9, rtol=0)


# ----------------------------------------------------------------------------- epsilon-greedy selection (Sec. 3.3)

def _philox_py(ctr, key):
    """Philox-4x32-10 written out with Python integers from the generator's definition (independent of the C code)."""
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & 0xffffffff, p1 & 0xffffffff, ((p0 >> 32) ^ c[3] ^ k[1]) & 0xffffffff, p0 & 0xffffffff]
        k = [(k[0] + 0x9E3779B9) & 0xffffffff, (k[1] + 0xBB67AE85) & 0xffffffff]
    return c


def test_philox_known_answers(orc):
    kat = json.load(open(os.path.join(GOLD, "philox_kat.json")))
    for v in kat["vectors"]:
        ctr, key = [int(x, 16) for x in v["ctr"]], [int(x, 16) for x in v["key"]]
        want = [int(x, 16) for x in v["out"]]
        assert list(orc.philox4x32_10(ctr, key)) == want
        assert _philox_py(ctr, key) == want
    rng = np.random.default_rng(3)
    for _ in range(200):
        ctr, key = [int(x) for x in rng.integers(0, 2**32, 4)], [int(x) for x in rng.integers(0, 2**32, 2)]
        assert list(orc.philox4x32_10(ctr, key)) == _philox_py(ctr, key)


def _pool(rng, n_table=500, count=40):
    ids = rng.permutation(n_table)[:count].astype(np.int32)
    sims = np.sort(rng.uniform(0.2, 0.9, count))[::-1].copy()
    q = rng.uniform(-1, 1, n_table).astype(np.float32)
    return ids, sims, q


def test_eps_zero_is_the_value_filter(orc):
    rng = np.random.default_rng(4)
    for _ in range(20):
        ids, sims, q = _pool(rng)
        lam = float(rng.uniform(0, 1))
        g_ids, g_s32, g_s64 = orc.rerank(ids, sims, q, lam, 8)
        e_ids, e_s32, e_s64, ex = orc.rerank_eps(ids, sims, q, lam, 8, 0.0, 99, 7, 3)
        assert np.array_equal(g_ids, e_ids) and np.array_equal(g_s64, e_s64) and not ex.any()


def test_eps_greedy_against_brute_force(orc):
    """Slot by slot in Python: greedy order from orc.rerank over the whole pool, draws from the Python Philox."""
    rng = np.random.default_rng(5)
    for trial in range(30):
        count = int(rng.integers(1, 30))
        ids, sims, q = _pool(rng, count=count)
        lam, k2 = float(rng.uniform(0, 1)), int(rng.integers(1, 12))
        eps = np.float32(rng.choice([0.05, 0.3, 0.5, 1.0]))
        seed, step, qi = int(rng.integers(0, 2**63)), int(rng.integers(0, 2**40)), int(rng.integers(0, 1000))
        order, _, order_sc = orc.rerank(ids, sims, q, lam, count)
        free = list(range(count))
        want_ids, want_sc, want_ex = [], [], []
        thr = int(float(eps) * 4294967296.0)
        for j in range(k2):
            if not free:
                want_ids.append(-1); want_sc.append(-np.inf); want_ex.append(0)
                continue
            r = _philox_py([step & 0xffffffff, step >> 32, qi, j], [seed & 0xffffffff, seed >> 32])
            explore = r[0] < thr
            pick = (r[1] * len(free)) >> 32 if explore else 0
            pos = free.pop(pick)
            want_ids.append(int(order[pos])); want_sc.append(float(order_sc[pos])); want_ex.append(int(explore))
        got_ids, _, got_sc, got_ex = orc.rerank_eps(ids, sims, q, lam, k2, float(eps), seed, step, qi)
        assert list(got_ids) == want_ids and list(got_ex) == want_ex
        assert np.array_equal(got_sc, np.array(want_sc))
        chosen = [i for i in want_ids if i >= 0]
        assert len(set(chosen)) == len(chosen) and set(chosen) <= set(ids.tolist())


def test_eps_one_explores_every_slot_and_rate_matches_eps(orc):
    rng = np.random.default_rng(6)
    ids, sims, q = _pool(rng, count=64)
    first = np.zeros(64, int)
    order, _, _ = orc.rerank(ids, sims, q, 0.5, 64)
    rank_of = {int(i): r for r, i in enumerate(order)}
    n_explored = 0
    trials = 3000
    for t in range(trials):
        e_ids, _, _, ex = orc.rerank_eps(ids, sims, q, 0.5, 4, 1.0, 1234, t, 0)
        assert ex.all()
        first[rank_of[int(e_ids[0])]] += 1
        _, _, _, ex2 = orc.rerank_eps(ids, sims, q, 0.5, 4, 0.25, 1234, t, 1)
        n_explored += int(ex2.sum())
    # first slot under eps = 1: uniform over the 64 members (expected 46.9 each; 6 sigma bounds)
    assert first.min() > 46.9 - 6 * 6.8 and first.max() < 46.9 + 6 * 6.8
    # exploration rate: 12000 Bernoulli(0.25) draws, 5 sigma
    assert abs(n_explored / (4 * trials) - 0.25) < 5 * math.sqrt(0.25 * 0.75 / (4 * trials))


def test_eps_planted_mistakes_are_caught(orc):
    """The brute-force pin above must tell apart the plausible wrong readings: picking among ALL members instead
    of the free ones, or using word 0 for the index."""
    rng = np.random.default_rng(7)
    ids, sims, q = _pool(rng, count=12)
    order, _, _ = orc.rerank(ids, sims, q, 0.5, 12)
    differs_all, differs_word = False, False
    for step in range(200):
        got, _, _, ex = orc.rerank_eps(ids, sims, q, 0.5, 6, 1.0, 5, step, 0)
        free = list(range(12))
        wrong_all, wrong_word = [], []
        free2 = list(range(12))
        for j in range(6):
            r = _philox_py([step, 0, 0, j], [5, 0])
            wrong_all.append(int(order[(r[1] * 12) >> 32]))
            wrong_word.append(int(order[free2.pop((r[0] * len(free2)) >> 32)]))
        differs_all |= wrong_all != list(got)
        differs_word |= wrong_word != list(got)
    assert differs_all and differs_word


# ----------------------------------------------------------------------------- start-point selection (Sec. 3.4)

def _sets(rng, n_table, G, max_len=40, bad=True):
    parts, off = [], [0]
    for g in range(G):
        n = int(rng.integers(0, max_len + 1))
        ids = rng.integers(0, n_table, n).astype(np.int32)              # repeats allowed
        if bad and n:
            ids[rng.random(n) < 0.1] = rng.choice([-1, -7, n_table, n_table + 5])
        parts.append(ids); off.append(off[-1] + n)
    return (np.concatenate(parts) if parts else np.zeros(0, np.int32)), np.array(off, np.int64)


def test_start_point_greedy_against_python_definition(orc):
    """eps = 0: the member with the largest value, the lower id among equals; invalid ids are no members."""
    rng = np.random.default_rng(21)
    for trial in range(20):
        n_table = int(rng.integers(1, 60))
        q = rng.choice([-1.0, -0.25, 0.0, 0.5, 1.0], n_table).astype(np.float32)   # many ties
        ids, off = _sets(rng, n_table, 12)
        got_id, got_q, ex, skipped = orc.select_by_q(ids, off, q)
        want_skipped = 0
        for g in range(12):
            members = [int(i) for i in ids[off[g]:off[g + 1]] if 0 <= i < n_table]
            want_skipped += int(off[g + 1] - off[g]) - len(members)
            if not members:
                assert got_id[g] == -1 and got_q[g] == 0.0
                continue
            best = max(float(q[i]) for i in members)
            assert got_id[g] == min(i for i in members if float(q[i]) == best)
            assert got_q[g] == q[got_id[g]]
        assert skipped == want_skipped and not ex.any()


def test_start_point_special_cases(orc):
    q = np.array([0.25, 0.25, 0.25, 0.25], np.float32)
    assert orc.select_by_q([3, 1, 2], [0, 3], q)[0][0] == 1                       # all equal: the lowest id
    assert orc.select_by_q([2], [0, 1], q)[0][0] == 2                             # a set of one
    assert orc.select_by_q([2], [0, 1], q, eps=1.0, seed=9, step=4)[0][0] == 2    # ... also when exploring
    q2 = np.array([np.nan, -np.inf, -3.0, -0.0, 0.0], np.float32)
    assert orc.select_by_q([0, 1], [0, 2], q2)[0][0] == 0                         # NaN counts as -inf: tie, lower id
    assert orc.select_by_q([0, 1, 2], [0, 3], q2)[0][0] == 2
    assert orc.select_by_q([4, 3], [0, 2], q2)[0][0] == 3                         # -0 == +0: tie, lower id
    out = orc.select_by_q([-1, 9], [0, 2], q2)
    assert out[0][0] == -1 and out[1][0] == 0.0 and out[3] == 2                   # no member at all


def test_start_point_exploration_draws(orc):
    """eps = 1 always explores and takes position floor(word1 * members / 2^32) among the members in array
    order, words from the Python Philox with counter (step, set index, 0xffffffff); the stream differs from the
    one the context slots use (last counter word = slot index)."""
    rng = np.random.default_rng(22)
    n_table = 300
    q = rng.uniform(-1, 1, n_table).astype(np.float32)
    ids, off = _sets(rng, n_table, 30, max_len=25)
    seed, step = 0x1234567890abcdef, (7 << 32) | 11
    got_id, got_q, ex, _ = orc.select_by_q(ids, off, q, eps=1.0, seed=seed, step=step)
    same_as_slot0 = 0
    for g in range(30):
        members = [int(i) for i in ids[off[g]:off[g + 1]] if 0 <= i < n_table]
        if not members:
            assert got_id[g] == -1 and ex[g] == 0
            continue
        r = _philox_py([step & 0xffffffff, step >> 32, g, 0xffffffff], [seed & 0xffffffff, seed >> 32])
        assert ex[g] == 1 and got_id[g] == members[(r[1] * len(members)) >> 32] and got_q[g] == q[got_id[g]]
        r0 = _philox_py([step & 0xffffffff, step >> 32, g, 0], [seed & 0xffffffff, seed >> 32])
        same_as_slot0 += r0[:2] == r[:2]
    assert same_as_slot0 == 0
    # rate of exploration and uniformity over positions, one set of 16 distinct members, 4000 steps
    members = rng.permutation(n_table)[:16].astype(np.int32)
    hits, explored = np.zeros(16, int), 0
    for t in range(4000):
        i, _, e, _ = orc.select_by_q(members, [0, 16], q, eps=1.0, seed=5, step=t)
        hits[list(members).index(int(i[0]))] += 1
        explored += int(orc.select_by_q(members, [0, 16], q, eps=0.25, seed=6, step=t)[2][0])
    assert hits.min() > 250 - 6 * 15.3 and hits.max() < 250 + 6 * 15.3           # binomial(4000, 1/16): sigma 15.3
    assert abs(explored / 4000 - 0.25) < 5 * math.sqrt(0.25 * 0.75 / 4000)


def test_start_point_planted_mistakes_are_caught(orc):
    """Plausible wrong readings give other answers on these inputs: ties to the higher id, the first maximum in
    array order, positions counted over invalid ids too."""
    q = np.array([0.5, 0.9, 0.9, 0.1, 0.9], np.float32)
    ids = np.array([4, 2, 1, 3], np.int32)
    got = int(orc.select_by_q(ids, [0, 4], q)[0][0])
    assert got == 1 and got != 4 and got != max(1, 2, 4)                           # first-in-array would say 4
    ids2 = np.array([-1, 3, -1, 0, 2], np.int32)
    differs = False
    for t in range(50):
        r = _philox_py([t, 0, 0, 0xffffffff], [1, 0])
        got = int(orc.select_by_q(ids2, [0, 5], q, eps=1.0, seed=1, step=t)[0][0])
        assert got == [3, 0, 2][(r[1] * 3) >> 32]
        wrong = int(ids2[(r[1] * 5) >> 32])                                       # counting the invalid ones
        differs |= wrong != got
    assert differs


# ----------------------------------------------------------------------------- stage rewards and their normalisation

def test_stage_rewards_closed_forms(orc):
    rng = np.random.default_rng(8)
    M = 2000
    feas = (rng.random(M) < 0.7).astype(np.uint8)
    lat = rng.uniform(0.1, 50, M).astype(np.float32)
    best = rng.uniform(0.1, 50, M).astype(np.float32)
    r1, _ = orc.shape_rewards(0, feas, lat, best, False)
    assert np.array_equal(r1, np.where(feas, 1.0, -1.0).astype(np.float32))          # Sec. 3.3: binary feasibility reward
    r2, _ = orc.shape_rewards(1, feas, lat, best, False)
    rho = best.astype(np.float64) / lat.astype(np.float64)
    closed = (rho * rho - 1) / (rho * rho + 1)          # tanh(ln rho) as a rational function: no tanh, no log
    assert np.all(r2[feas == 0] == -1.0)
    assert np.max(np.abs(r2[feas == 1] - closed[feas == 1])) < 1e-6
    assert np.all(np.abs(r2[feas == 1]) < 1.0)                                        # App. A: tanh(log rho) in (-1, 1)
    same, _ = orc.shape_rewards(1, np.ones(3, np.uint8), np.array([2.0, 5.0, 7.5], np.float32), np.array([2.0, 5.0, 7.5], np.float32), False)
    assert np.all(same == 0.0)                                                        # no speed-up: reward 0
    faster, _ = orc.shape_rewards(1, np.ones(2, np.uint8), np.array([1.0, 4.0], np.float32), np.array([2.0, 2.0], np.float32), False)
    assert faster[0] > 0 > faster[1] and abs(faster[0] - 0.6) < 1e-7 and abs(faster[1] + 0.6) < 1e-7   # rho = 2, 1/2: 3/5


def test_online_normalisation_against_numpy_prefix_statistics(orc):
    rng = np.random.default_rng(9)
    M = 600
    feas = (rng.random(M) < 0.8).astype(np.uint8)
    lat = rng.uniform(0.5, 5, M).astype(np.float32)
    best = rng.uniform(0.5, 5, M).astype(np.float32)
    raw, _ = orc.shape_rewards(1, feas, lat, best, False)
    raw64 = np.where(feas, np.tanh(np.log(best.astype(np.float64)) - np.log(lat.astype(np.float64))), -1.0)
    sigma_min = 0.05
    got, state = orc.shape_rewards(1, feas, lat, best, True, sigma_min)
    want = np.empty(M)
    for t in range(M):
        prev = raw64[:t]
        mu = prev.mean() if t else 0.0
        sd = prev.std() if t else 0.0                      # numpy's default is the population (1/t) form
        want[t] = (raw64[t] - mu) / max(sd, sigma_min)
    assert np.max(np.abs(got - want)) < 2e-5 * np.max(np.abs(want))
    assert abs(state[0] - M) == 0 and abs(state[1] - raw64.sum()) < 1e-9 and abs(state[2] - (raw64 ** 2).sum()) < 1e-9
    assert np.max(np.abs(got)) <= 2.0 / sigma_min + 1e-6                               # App. A: |R| <= 2 / sigma_min
    assert abs(got[0] - raw[0] / sigma_min) < 1e-5                                     # first sample: mu = 0, floor applies
    # the statistics used are the ones BEFORE the sample: a huge outlier does not normalise itself away
    # splitting a batch in two calls with the state carried over changes nothing
    a, st = orc.shape_rewards(1, feas[:250], lat[:250], best[:250], True, sigma_min)
    b, st = orc.shape_rewards(1, feas[250:], lat[250:], best[250:], True, sigma_min, state=st)
    assert np.array_equal(np.concatenate([a, b]), got) and np.array_equal(st, state)
    # clipping
    c, _ = orc.shape_rewards(1, feas, lat, best, True, sigma_min, clip=1.5)
    assert np.array_equal(c, np.clip(got, -1.5, 1.5))


def test_normalised_rewards_converge_to_the_z_score_map(orc):
    """App. A, stability of online normalisation: for a stationary stream the map tends to (r - mu) / sigma."""
    rng = np.random.default_rng(10)
    M = 20000
    lat = np.exp(rng.normal(0, 0.5, M)).astype(np.float32)
    best = np.ones(M, np.float32)
    raw = np.tanh(-np.log(lat.astype(np.float64)))
    got, _ = orc.shape_rewards(1, np.ones(M, np.uint8), lat, best, True, 1e-3)
    tail = slice(M - 2000, M)
    assert np.max(np.abs(got[tail] - (raw[tail] - raw.mean()) / raw.std())) < 0.05


# ----------------------------------------------------------------------------- typed / masked recall

def test_masked_recall_equals_recall_on_the_accepted_sub_bank(orc):
    """Pin: leaving entries out must be the same as a bank that never held them (ids mapped back)."""
    rng = np.random.default_rng(11)
    N, d = 700, 24
    rows = _unit(rng, N, d)
    q = _unit(rng, 6, d)
    types = rng.integers(0, 4, N).astype(np.uint32)
    groups = rng.integers(0, 9, N).astype(np.uint32)
    tags = types | (groups << 8)
    allow = np.array([0b0001, 0b0110, 0b1111, 0b1000, 0b1111, 0], np.uint32)
    exclude = np.array([0xffffffff, 3, 0xffffffff, 5, 8, 0xffffffff], np.uint32)
    ids, sims = orc.recall_masked(rows, tags, q, allow, exclude, 20)
    for b in range(6):
        keep = np.flatnonzero(((allow[b] >> types) & 1).astype(bool) & (groups != exclude[b]))
        if len(keep) == 0:
            assert np.all(ids[b] == -1) and np.all(np.isneginf(sims[b]))
            continue
        sub_ids, sub_sims = orc.recall(np.ascontiguousarray(rows[keep]), q[b:b + 1], 20)
        live = sub_ids[0] >= 0
        assert np.array_equal(ids[b][live], keep[sub_ids[0][live]]) and np.array_equal(sims[b][live], sub_sims[0][live])
        assert np.all(ids[b][~live] == -1)
    # accepting everything is the plain recall; types above 31 are never retrievable
    all_ids, all_sims = orc.recall_masked(rows, tags, q, np.full(6, 0xffffffff, np.uint32), np.full(6, 0xffffffff, np.uint32), 20)
    p_ids, p_sims = orc.recall(rows, q, 20)
    assert np.array_equal(all_ids, p_ids) and np.array_equal(all_sims, p_sims)
    odd = tags.copy()
    odd[:350] = 40 | (groups[:350] << 8)
    o_ids, _ = orc.recall_masked(rows, odd, q, np.full(6, 0xffffffff, np.uint32), np.full(6, 0xffffffff, np.uint32), 20)
    assert o_ids.min() >= 350
