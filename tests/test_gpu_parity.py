"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same seeded
inputs.  Ids bit-exact (lower id breaks ties; a swap is accepted only between entries whose oracle
values differ by < 1e-5), scores within 1e-5 * max(1,|score|), Q tables bit-exact against the
sequential fp32 recurrence and within 1e-6 of the fp64 one."""
import numpy as np
import pytest
import torch

from paper_2603_10846_amd import binding as B
from paper_2603_10846_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu
DT = {"f32": 0, "bf16": 1, "f16": 2}


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _unit(rng, n, d):
    x = rng.standard_normal((n, d)).astype(np.float32)
    return (x / np.linalg.norm(x, axis=1, keepdims=True)).astype(np.float32)


def _make_bank(dtype, rows, qtab=None, capacity=None, max_B=1024, max_k1=256, chunk=65536):
    N, d = rows.shape
    bank = B.MemoryBank(d, dtype, capacity or max(N, 1), max_B=max_B, max_k1=max_k1)
    for a in range(0, N, chunk):
        sl = slice(a, min(N, a + chunk))
        first = bank.append(_dev(rows[sl]),
                            None if qtab is None else _dev(qtab[0, sl]),
                            None if qtab is None else _dev(qtab[1, sl]))
        assert first == a
    return bank


# ----------------------------------------------------------------------------- store

@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_store_holds_rne_rounded_rows(orc, dtype):
    rng = np.random.default_rng(100)
    rows = (rng.standard_normal((1000, 72)) * rng.uniform(1e-3, 50, (1000, 1))).astype(np.float32)
    rows[3, :5] = [65519.9, 65520.0, 1e-8, 6.1e-5, -3.0e-8]      # fp16 overflow edge / subnormals
    bank = B.MemoryBank(72, dtype, 1000, max_B=8, max_k1=16)
    assert bank.append(_dev(rows[:600])) == 0 and bank.append(_dev(rows[600:])) == 600
    assert bank.size() == 1000
    got = bank.read_rows(0, 1000).cpu().numpy()
    want = orc.round_to_store(rows, DT[dtype])
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.array_equal(bank.read_rows(599, 3).cpu().numpy(), want[599:602])
    with pytest.raises(B.MemError) as e:
        bank.append(_dev(rows[:1]))
    assert e.value.status == B.MEM_ECAPACITY and bank.size() == 1000
    assert np.all(bank.read_q(0).cpu().numpy() == 0) and np.all(bank.read_q(1).cpu().numpy() == 0)
    bank.close()


def test_read_probe_reads_every_stored_word_once(orc):
    """The read-only pass XORs every 32-bit word of the stored rows: for whole tiles and whole k-blocks
    (no padding in the store) that is the XOR of the rows' bf16 pairs as the oracle rounds them, and fp32 words."""
    rng = np.random.default_rng(109)
    for dtype, N, d in (("bf16", 1024, 128), ("f32", 512, 64)):
        rows = rng.standard_normal((N, d)).astype(np.float32)
        bank = _make_bank(dtype, rows, max_B=8, max_k1=16)
        chk = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        nbytes = bank.read_probe(chk)
        torch.cuda.synchronize()
        bits = orc.round_to_store(rows, DT[dtype]).view(np.uint32)
        if dtype == "bf16":
            h = bits >> 16
            words = h[:, 0::2] | (h[:, 1::2] << 16)
            assert nbytes == N * d * 2
        else:
            words = bits
            assert nbytes == N * d * 4
        assert np.uint32(chk.cpu().numpy().view(np.uint32)[0]) == np.bitwise_xor.reduce(words.ravel())
        bank.close()


# ----------------------------------------------------------------------------- retrieval, small

CASES = [
    # dtype, N, d, B, k1, k2, lam, stage
    ("bf16", 5000, 128, 3, 32, 4, 0.5, 0),      # MFMA scan, 32-query tile, one pass, ragged last tile
    ("f16", 20000, 256, 2, 16, 16, 0.3, 1),     # MFMA scan, 32-query tile, two passes
    ("f32", 3000, 72, 4, 64, 8, 0.7, 0),        # VALU scan (fp32 rows, <= 4 queries), dimension padded to 128
    ("f32", 9000, 64, 1, 256, 32, 1.0, 1),      # VALU scan, largest pool of the one-wavefront-per-entry value filter
    ("bf16", 20000, 192, 5, 32, 4, 0.5, 0),     # MFMA scan, 32-query tile
    ("f16", 9000, 64, 40, 8, 2, 0.0, 1),        # MFMA scan, 64-query tile
    ("bf16", 30000, 256, 100, 64, 8, 0.25, 0),  # MFMA scan, 128-query tile
    ("bf16", 12345, 128, 260, 128, 16, 0.5, 1), # MFMA scan, two 256-query tiles
    ("f32", 20000, 128, 33, 64, 8, 0.5, 0),     # MFMA scan on fp32 rows (bf16 hi/lo split)
    ("f16", 70000, 64, 17, 256, 32, 0.7, 1),    # three passes (ratio 8 at k1 = 256)
]


@pytest.mark.parametrize("nq", [1, 2, 4])
def test_fp32_small_batch_scan_on_a_long_bank(orc, nq):
    """fp32 rows, at most four queries, a pass of 1024 tiles or more: the VALU scan then gives a whole
    256-row tile to one workgroup (shorter passes split a tile over four).  300,044 entries: the
    densest pass has more than 1024 tiles and the bank's last tile is ragged."""
    N, d, k1, k2 = 300044, 64, 64, 8
    lib = B.load()
    import ctypes as C
    st_, rh_, nt_ = (C.c_int * 8)(), (C.c_int * 8)(), (C.c_int * 8)()
    nl = lib.mem_plan_levels(N, k1, st_, rh_, nt_, 8)
    assert nl >= 2 and max(nt_[:nl]) >= 1024                 # the whole-tile variant is the one that runs
    rng = np.random.default_rng([11, nq])
    rows = _unit(rng, N, d) * rng.uniform(0.5, 2.0, (N, 1)).astype(np.float32)
    rows[N - 2] = rows[31]                                    # an exact tie, one copy in the ragged tile
    queries = _unit(rng, nq, d)
    queries[0] = rows[31] * np.float32(3.0)
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    print(f"fp32 long bank B={nq}", flush=True)
    bank = _make_bank("f32", rows, qtab, max_B=4, max_k1=64)
    gpu = parity.gpu_retrieve(bank, torch, queries, 1, k1, k2, 0.4)
    stats = parity.check_retrieve(orc, rows, queries, qtab[1], k1, k2, 0.4, gpu, threads=4)
    assert gpu["cand_ids"][0, 0] == 31 and gpu["cand_ids"][0, 1] == N - 2
    assert stats["boundary_swaps"] == 0 and stats["final_swaps"] == 0 and stats["queries"] == nq
    assert bank.counters() == (0, 0)
    bank.close()


@pytest.mark.parametrize("dtype,N,d,nq,k1,k2,lam,stage", CASES)
def test_retrieve_matches_oracle(orc, dtype, N, d, nq, k1, k2, lam, stage):
    rng = np.random.default_rng([DT[dtype], N, d, nq])
    rows = _unit(rng, N, d) * rng.uniform(0.5, 2.0, (N, 1)).astype(np.float32)   # norms must not matter
    rows[N // 2] = rows[7]                                                        # an exact duplicate row
    queries = _unit(rng, nq, d)
    queries[0] = rows[7] * np.float32(0.5)                                        # hits the duplicate pair
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    print(f"case {dtype} N={N} d={d} B={nq} k1={k1} k2={k2}", flush=True)
    bank = _make_bank(dtype, rows, qtab, max_B=max(nq, 8), max_k1=256)
    gpu = parity.gpu_retrieve(bank, torch, queries, stage, k1, k2, lam)
    st = orc.round_to_store(rows, DT[dtype])
    qr = orc.round_to_store(queries, DT[dtype])
    stats = parity.check_retrieve(orc, st, qr, qtab[stage], k1, k2, lam, gpu)
    assert gpu["cand_ids"][0, 0] == 7 and gpu["cand_ids"][0, 1] == N // 2        # tie -> lower id first
    assert abs(gpu["cand_sims"][0, 0] - 1.0) < 1e-6
    assert stats["boundary_swaps"] == 0 and stats["final_swaps"] == 0
    # the same call again gives bit-identical outputs
    again = parity.gpu_retrieve(bank, torch, queries, stage, k1, k2, lam)
    for k in gpu:
        assert np.array_equal(gpu[k].view(np.uint32), again[k].view(np.uint32)), k
    assert bank.counters() == (0, 0)
    bank.close()


def test_edge_cases(orc):
    rng = np.random.default_rng(101)
    rows = _unit(rng, 10, 64)
    q = _unit(rng, 3, 64)
    bank = B.MemoryBank(64, "f16", 300, max_B=8, max_k1=64)
    with pytest.raises(B.MemError) as e:                             # no retrieve yet: no status words to report
        bank.retrieve_flags(1)
    assert e.value.status == B.MEM_ESTATE
    # empty bank: everything padded
    out = parity.gpu_retrieve(bank, torch, q, 0, 16, 4, 0.5)
    assert np.all(out["ids"] == -1) and np.all(np.isneginf(out["scores"])) and np.all(out["cand_ids"] == -1)
    assert bank.retrieve_flags(3).cpu().numpy().tolist() == [0, 0, 0] and bank.retrieve_flags(0).numel() == 0
    with pytest.raises(B.MemError) as e:                             # more queries than that call had
        bank.retrieve_flags(4)
    assert e.value.status == B.MEM_ESTATE
    # one entry: pool of one, z-scores are 0
    bank.append(_dev(rows[:1]))
    out = parity.gpu_retrieve(bank, torch, q, 0, 16, 4, 0.5)
    assert out["ids"][:, 0].tolist() == [0, 0, 0] and np.all(out["ids"][:, 1:] == -1) and np.all(out["scores"][:, 0] == 0)
    # k1 > N and k2 == k1: whole bank comes back
    bank.append(_dev(rows[1:]))
    out = parity.gpu_retrieve(bank, torch, q, 1, 16, 16, 0.5)
    st, qr = orc.round_to_store(rows, 2), orc.round_to_store(q, 2)
    parity.check_retrieve(orc, st, qr, np.zeros(10, np.float32), 16, 16, 0.5, out)
    assert sorted(out["ids"][0][:10].tolist()) == list(range(10))
    # B = 0 is a no-op, bad arguments are rejected
    empty = torch.empty((0, 64), device="cuda:0")
    bank.retrieve(empty, 0, 4, 2, 0.5)
    qd = _dev(q)
    for kw in (dict(stage=2), dict(k1=0), dict(k2=0), dict(k1=4, k2=5), dict(k1=65), dict(lam=1.5), dict(lam=float("nan"))):
        a = dict(stage=0, k1=8, k2=2, lam=0.5)
        a.update(kw)
        with pytest.raises(B.MemError) as e:
            bank.retrieve(qd, a["stage"], a["k1"], a["k2"], a["lam"])
        assert e.value.status == B.MEM_EINVAL
    with pytest.raises(B.MemError):
        bank.retrieve(_dev(_unit(rng, 9, 64)), 0, 8, 2, 0.5)         # B > max_B
    with pytest.raises(B.MemError):
        bank.update_q(torch.zeros(1, dtype=torch.int32, device="cuda:0"), 0, torch.zeros(1, device="cuda:0"), 0.0)
    bank.close()


@pytest.mark.parametrize("dtype,N,d,nq,k1,k2", [
    ("f16", 1500, 16384, 2, 16, 4),      # largest dimension (256 k-blocks), MFMA scan
    ("f32", 1200, 16384, 1, 16, 4),      # largest dimension, fp32 VALU scan
    ("bf16", 1000, 8, 3, 8, 2),          # smallest dimension (padded to one k-block)
    ("bf16", 5000, 64, 4096, 32, 4),     # largest batch: sixteen 256-query tiles
    ("f32", 3000, 72, 4095, 16, 4),      # largest batch but one, fp32 rows through the bf16 split
])
def test_maximum_sizes(orc, dtype, N, d, nq, k1, k2):
    rng = np.random.default_rng(N + d + nq)
    rows = _unit(rng, N, d)
    q = _unit(rng, nq, d)
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    bank = _make_bank(dtype, rows, qtab, max_B=nq, max_k1=k1)
    gpu = parity.gpu_retrieve(bank, torch, q, 1, k1, k2, 0.5)
    st, qr = orc.round_to_store(rows, DT[dtype]), orc.round_to_store(q, DT[dtype])
    sample = None if nq <= 8 else sorted(set([0, 1, 255, 256, 257, 1000, 2047, 2048, 3000, nq - 2, nq - 1]))
    parity.check_retrieve(orc, st, qr, qtab[1], k1, k2, 0.5, gpu, sample=sample)
    assert np.all(gpu["cand_ids"] >= 0) and np.all(np.diff(gpu["cand_sims"], axis=1) <= 0)
    assert np.all(np.diff(gpu["scores"], axis=1) <= 0)
    assert bank.counters() == (0, 0)
    bank.close()


def _random_case(i):
    rng = np.random.default_rng(7000 + i)
    dtype = ["f32", "bf16", "f16"][int(rng.integers(0, 3))]
    N = int(rng.choice([1, 2, 31, 255, 256, 257, 1000, 5000, 8191, 8193, 20000, 40000]))
    d = int(rng.choice([8, 16, 56, 64, 72, 128, 200, 256, 512]))
    nq = int(rng.choice([1, 2, 4, 5, 31, 32, 33, 64, 65, 128, 129, 257, 300]))
    k1 = int(rng.choice([1, 2, 7, 16, 33, 64, 128, 129, 200, 256]))
    k2 = int(rng.integers(1, k1 + 1))
    lam = float(rng.choice([0.0, 1.0, rng.uniform(0, 1)]))
    return dtype, N, d, nq, k1, k2, lam, int(rng.integers(0, 2))


@pytest.mark.parametrize("i", range(60))
def test_random_configurations(orc, i):
    """Seeded random shapes around the kernels' tile and dispatch boundaries (row tiles of 256, query tiles of
    32 / 64 / 128 / 256, the 4-query switch of fp32 stores, the 128-entry switch of the value filter, one or
    several passes), duplicated rows for exact ties, every query or 16 sampled ones against the oracle."""
    dtype, N, d, nq, k1, k2, lam, stage = _random_case(i)
    rng = np.random.default_rng(9000 + i)
    rows = _unit(rng, N, d)
    if N >= 31:
        rows[rng.integers(0, N, 8)] = rows[int(rng.integers(0, N))]       # exact ties on similarity
    q = _unit(rng, nq, d)
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    bank = _make_bank(dtype, rows, qtab, max_B=nq, max_k1=k1, chunk=int(rng.choice([97, 256, 1000, 65536])))   # ragged appends
    gpu = parity.gpu_retrieve(bank, torch, q, stage, k1, k2, lam)
    st, qr = orc.round_to_store(rows, DT[dtype]), orc.round_to_store(q, DT[dtype])
    sample = None if nq <= 16 else sorted(set(rng.integers(0, nq, 14).tolist() + [0, nq - 1]))
    parity.check_retrieve(orc, st, qr, qtab[stage], k1, k2, lam, gpu, sample=sample)
    # the same call with epsilon-greedy slot filling, wherever the greedy order of the pool is not a near-tie
    eps, seed, step = float(rng.choice([0.1, 0.5, 1.0])), int(rng.integers(0, 2**63)), int(rng.integers(0, 2**40))
    ids, sc, cid, _, ex = bank.retrieve_eps(_dev(q), stage, k1, k2, lam, eps, seed, step, want_candidates=True)
    torch.cuda.synchronize()
    ids, cid, ex = ids.cpu().numpy(), cid.cpu().numpy(), ex.cpu().numpy()
    assert np.array_equal(cid, gpu["cand_ids"])
    k1e = min(k1, N)
    for b in (range(nq) if sample is None else sample):
        pool = cid[b][:k1e]
        sims = orc.sims_of(st, qr[b], pool)
        _, _, order_sc = orc.rerank(pool, sims, qtab[stage], lam, k1e)
        gaps = -np.diff(order_sc)
        if np.any((gaps > 0) & (gaps < 1e-7)):                    # (exact ties are ordered by id on both sides)
            continue
        w_ids, _, _, w_ex = orc.rerank_eps(pool, sims, qtab[stage], lam, k2, eps, seed, step, b)
        assert np.array_equal(ids[b], w_ids) and np.array_equal(ex[b], w_ex), f"query {b}"
    assert bank.counters() == (0, 0)
    bank.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_degenerate_rows_and_queries_give_well_formed_results(orc, dtype):
    """A zero row, a row with a NaN, a row with an infinity, a zero query and a NaN query: the results
    for them are unspecified, but every call returns, every id is -1 or a real entry, no id repeats within
    a pool, and the entry points that follow are unaffected."""
    rng = np.random.default_rng(555)
    N, d = (20000 if dtype == "bf16" else 3000), 64            # the larger bank takes two passes (a NaN threshold)
    rows = _unit(rng, N, d)
    rows[5] = 0.0
    rows[17, 3] = np.nan
    rows[40, 0] = np.inf
    q = _unit(rng, 8, d)
    q[6] = 0.0
    q[7, 1] = np.nan
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    qtab[1, 100] = np.nan                                                # a poisoned value too
    bank = _make_bank(dtype, rows, qtab, max_B=8, max_k1=300)
    for nq in (3, 8):
        for k1, k2, stage in ((16, 4, 0), (200, 8, 1), (300, 300, 1)):
            out = parity.gpu_retrieve(bank, torch, q[:nq], stage, k1, k2, 0.5)
            for name in ("ids", "cand_ids"):
                a = out[name]
                assert a.min() >= -1 and a.max() < N, (name, nq, k1)
                for b in range(nq):
                    live = a[b][a[b] >= 0]
                    assert live.size == np.unique(live).size, (name, nq, k1, b)
            ids, _, _, _, ex = bank.retrieve_eps(_dev(q[:nq]), stage, k1, k2, 0.5, 0.5, 3, 4)
            ids = ids.cpu().numpy()
            assert ids.min() >= -1 and ids.max() < N
    ids = out["ids"].reshape(-1).astype(np.int32)
    bank.update_q(_dev(ids), 1, _dev(np.ones(ids.size, np.float32)), 0.1)
    got, _, _ = bank.select_by_q(_dev(np.arange(N, dtype=np.int32)), _dev(np.array([0, N], np.int64)), 1)
    assert 0 <= int(got[0]) < N
    bank.close()
    # a clean bank right afterwards behaves as usual
    clean = _unit(rng, 2000, d)
    bank = _make_bank(dtype, clean, max_B=8, max_k1=32)
    gpu = parity.gpu_retrieve(bank, torch, q[:6], 0, 32, 4, 0.5)
    parity.check_retrieve(orc, orc.round_to_store(clean, DT[dtype]), orc.round_to_store(q[:6], DT[dtype]),
                          np.zeros(2000, np.float32), 32, 4, 0.5, gpu)
    bank.close()


def test_calls_on_a_side_stream_and_two_banks_at_once(orc):
    """The stream is an argument of every call: work issued on a non-default stream gives the same results,
    and two banks alive on one device do not disturb each other."""
    rng = np.random.default_rng(77)
    rows_a, rows_b = _unit(rng, 9000, 128), _unit(rng, 5000, 64)
    qa, qb = _unit(rng, 40, 128), _unit(rng, 3, 64)
    bank_a = _make_bank("bf16", rows_a, max_B=64, max_k1=32)
    bank_b = _make_bank("f32", rows_b, max_B=8, max_k1=32)
    ref_a = parity.gpu_retrieve(bank_a, torch, qa, 0, 32, 4, 0.5)
    ref_b = parity.gpu_retrieve(bank_b, torch, qb, 0, 16, 4, 0.5)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        got_b = bank_b.retrieve(_dev(qb), 0, 16, 4, 0.5, want_candidates=True)
        got_a = bank_a.retrieve(_dev(qa), 0, 32, 4, 0.5, want_candidates=True)
        ids = got_a[0].reshape(-1).contiguous()
        bank_a.update_q(ids, 0, torch.ones(ids.numel(), device="cuda:0"), 0.25)
    side.synchronize()
    assert np.array_equal(got_a[0].cpu().numpy(), ref_a["ids"]) and np.array_equal(got_a[2].cpu().numpy(), ref_a["cand_ids"])
    assert np.array_equal(got_b[0].cpu().numpy(), ref_b["ids"]) and np.array_equal(got_b[1].cpu().numpy(), ref_b["scores"])
    want, _ = orc.update_q32(np.zeros(9000, np.float32), ref_a["ids"].reshape(-1).astype(np.int32),
                             np.ones(ref_a["ids"].size, np.float32), 0.25)
    assert np.array_equal(bank_a.read_q(0).cpu().numpy().view(np.uint32), want.view(np.uint32))
    assert np.all(bank_b.read_q(0).cpu().numpy() == 0)
    bank_a.close()
    bank_b.close()


@pytest.mark.parametrize("dtype,N,d,nq,k1,k2", [("f32", 4096, 768, 1, 32, 4), ("bf16", 20000, 256, 40, 64, 8), ("f16", 30000, 128, 200, 128, 16)])
def test_retrieve_and_update_replayed_from_a_hip_graph(orc, dtype, N, d, nq, k1, k2):
    """The hot calls launch kernels and nothing else (no allocation, no wait, no memset), so a caller can
    record them into a HIP graph once the first calls have done their per-device set-up.  Four replays
    with new queries each, eager work and waits in between: every replay must equal the same calls
    issued eagerly on a twin bank, bit for bit (outputs and the value table), and the oracle."""
    rng = np.random.default_rng([DT[dtype], N, d, nq, 5])
    rows = _unit(rng, N, d)
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    rewards = _dev(rng.uniform(0, 1, nq * k2).astype(np.float32))
    eager = _make_bank(dtype, rows, qtab, max_B=max(nq, 8), max_k1=128)
    graphed = _make_bank(dtype, rows, qtab, max_B=max(nq, 8), max_k1=128)
    q_in = _dev(_unit(rng, nq, d))
    out = (torch.empty((nq, k2), dtype=torch.int32, device="cuda:0"), torch.empty((nq, k2), dtype=torch.float32, device="cuda:0"),
           torch.empty((nq, k1), dtype=torch.int32, device="cuda:0"), torch.empty((nq, k1), dtype=torch.float32, device="cuda:0"))
    flags = torch.empty(nq, dtype=torch.int32, device="cuda:0")

    def step(bank, q, o):
        bank.retrieve(q, 1, k1, k2, 0.5, out=o)
        bank.update_q(o[0].reshape(-1), 1, rewards, 0.1)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(graphed, q_in, out)                         # per-device set-up happens in the first call
    side.synchronize()
    graphed.q.copy_(_dev(qtab))                          # undo that step's update
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(graphed, q_in, out)
        B._check(graphed.lib.mem_retrieve_flags(graphed.h, B._ptr(flags), nq, B._stream()), "mem_retrieve_flags")
    table = qtab[1].copy()
    for rep in range(4):
        queries = _unit(rng, nq, d)
        q_in.copy_(_dev(queries))
        graph.replay()
        torch.cuda.synchronize()
        e_out = eager.retrieve(_dev(queries), 1, k1, k2, 0.5, want_candidates=True)
        eager.update_q(e_out[0].reshape(-1), 1, rewards, 0.1)
        torch.cuda.synchronize()
        for got, want in zip(out, e_out):
            assert torch.equal(got.view(torch.int32), want.view(torch.int32)), f"replay {rep}"
        assert torch.equal(graphed.q.view(torch.int32), eager.q.view(torch.int32)), f"replay {rep}: value table"
        assert int(flags.abs().sum()) == 0
        gpu = {"ids": out[0].cpu().numpy(), "scores": out[1].cpu().numpy(), "cand_ids": out[2].cpu().numpy(), "cand_sims": out[3].cpu().numpy()}
        stats = parity.check_retrieve(orc, orc.round_to_store(rows, DT[dtype]), orc.round_to_store(queries, DT[dtype]), table, k1, k2, 0.5, gpu)
        assert stats["boundary_swaps"] == 0 and stats["final_swaps"] == 0
        table, _ = orc.update_q32(table, gpu["ids"].reshape(-1).astype(np.int32), rewards.cpu().numpy(), 0.1)
        assert np.array_equal(graphed.read_q(1).cpu().numpy().view(np.uint32), table.view(np.uint32)), f"replay {rep}: oracle's table"
    del graph
    eager.close()
    graphed.close()


def test_survivor_list_overflow_is_counted(orc):
    """More rows tie with the pool's last member than a survivor list holds (8192): the query is counted by
    mem_counters, the call still returns a valid pool of exact ties, and later calls are unaffected."""
    rng = np.random.default_rng(107)
    v = _unit(rng, 1, 128)
    rows = np.concatenate([np.repeat(v, 16000, axis=0), _unit(rng, 4000, 128)])
    rows = rows[rng.permutation(len(rows))]
    copies = set(np.flatnonzero(np.all(rows == v[0], axis=1)).tolist())
    bank = _make_bank("bf16", rows, max_B=8, max_k1=64)
    q = np.concatenate([v, _unit(rng, 5, 128)])
    out = parity.gpu_retrieve(bank, torch, q, 0, 64, 8, 0.0)
    flags = bank.retrieve_flags(len(q)).cpu().numpy()          # per call and per query, no device-wide wait
    skipped, overflows = bank.counters()
    assert skipped == 0 and overflows >= 1
    pool = out["cand_ids"][0]
    assert len(set(pool.tolist())) == 64 and set(pool.tolist()) <= copies
    assert np.all(np.abs(out["cand_sims"][0] - 1.0) < 1e-5)
    # the queries of the same call whose pools have no such mass of ties match the oracle
    st, qr = orc.round_to_store(rows, DT["bf16"]), orc.round_to_store(q, DT["bf16"])
    sims = (qr.astype(np.float64) @ st.astype(np.float64).T)
    sims /= np.linalg.norm(qr.astype(np.float64), axis=1)[:, None] * np.linalg.norm(st.astype(np.float64), axis=1)[None, :]
    kth = np.sort(sims, axis=1)[:, -64]
    crowded = [(sims[b] >= kth[b] - 1e-3).sum() > 4096 for b in range(len(q))]
    assert crowded[0] and overflows >= 1
    safe = [b for b in range(len(q)) if not crowded[b]]
    assert len(safe) >= 3
    assert flags[0] & 1 and all(flags[b] == 0 for b in safe)
    parity.check_retrieve(orc, st, qr, np.zeros(len(rows), np.float32), 64, 8, 0.0, out, sample=safe)
    before = bank.counters()[1]
    out2 = parity.gpu_retrieve(bank, torch, q[safe], 0, 64, 8, 0.0)
    parity.check_retrieve(orc, st, qr[safe], np.zeros(len(rows), np.float32), 64, 8, 0.0, out2)
    assert bank.counters()[1] == before and not bank.retrieve_flags(len(safe)).cpu().numpy().any()
    # the exhaustive call answers the flagged query exactly: the copies tie exactly, so the pool is their 64 lowest ids
    ids, sc, cid, csim = bank.retrieve_exact(_dev(q), 0, 64, 8, 0.0, want_candidates=True)
    torch.cuda.synchronize()
    ex = {"ids": ids.cpu().numpy(), "scores": sc.cpu().numpy(), "cand_ids": cid.cpu().numpy(), "cand_sims": csim.cpu().numpy()}
    assert ex["cand_ids"][0].tolist() == sorted(copies)[:64]
    stats = parity.check_retrieve(orc, st, qr, np.zeros(len(rows), np.float32), 64, 8, 0.0, ex)
    assert stats["boundary_swaps"] == 0 and stats["order_swaps"] == 0 and stats["final_swaps"] == 0
    assert not bank.retrieve_flags(len(q)).cpu().numpy().any() and bank.counters()[1] == before
    bank.close()


@pytest.mark.parametrize("dtype,N,d,nq,k1,k2", [("bf16", 30000, 128, 7, 64, 8), ("f32", 9000, 72, 2, 256, 32), ("f16", 20000, 64, 70, 300, 16),
                                                ("bf16", 100, 64, 3, 128, 16), ("f16", 9000, 64, 5, 2048, 64)])
def test_exhaustive_retrieve_matches_oracle_and_the_scan(orc, dtype, N, d, nq, k1, k2):
    rng = np.random.default_rng([17, N, nq, k1])
    rows = _unit(rng, N, d) * rng.uniform(0.5, 2.0, (N, 1)).astype(np.float32)
    rows[N // 2] = rows[7]
    q = _unit(rng, nq, d)
    q[0] = rows[7]
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    print(f"exhaustive {dtype} N={N} B={nq} k1={k1}", flush=True)
    bank = _make_bank(dtype, rows, qtab, max_B=max(nq, 8), max_k1=max(k1, 256))
    ids, sc, cid, csim = bank.retrieve_exact(_dev(q), 1, k1, k2, 0.5, want_candidates=True)
    torch.cuda.synchronize()
    ex = {"ids": ids.cpu().numpy(), "scores": sc.cpu().numpy(), "cand_ids": cid.cpu().numpy(), "cand_sims": csim.cpu().numpy()}
    st, qr = orc.round_to_store(rows, DT[dtype]), orc.round_to_store(q, DT[dtype])
    stats = parity.check_retrieve(orc, st, qr, qtab[1], k1, k2, 0.5, ex)
    assert stats["boundary_swaps"] == 0 and stats["final_swaps"] == 0
    assert ex["cand_ids"][0, 0] == 7 and (N <= 7 or ex["cand_ids"][0, 1] == N // 2)
    # the ordinary call agrees bit for bit on such data (no ties within fp32 resolution at a pool's edge)
    ref = parity.gpu_retrieve(bank, torch, q, 1, k1, k2, 0.5)
    for k in ex:
        assert np.array_equal(ex[k].view(np.uint32), ref[k].view(np.uint32)), k
    assert bank.counters() == (0, 0)
    bank.close()


@pytest.mark.parametrize("dtype,nq,k1", [("bf16", 5, 64), ("bf16", 130, 100), ("f32", 2, 32), ("f16", 40, 200)])
def test_crowded_band_of_distinct_near_ties(orc, dtype, nq, k1):
    """Thousands of entries whose similarities to a query differ by less than the scan's rounding margin
    (successive refinements of one kernel give such near-duplicates): far more than the 512 candidates that
    are re-scored at once.  The pool must still be the oracle's up to the resolution of an fp32 similarity:
    no list overflows, and whatever differs from the oracle's pool lies within 3e-7 of its last member."""
    rng = np.random.default_rng([13, nq, k1])
    d, n_near, n_far = 128, 3000, 9000
    v = _unit(rng, 1, d)
    near = v + np.float32(0.001) * rng.standard_normal((n_near, d)).astype(np.float32) * rng.uniform(0, 1, (n_near, 1)).astype(np.float32)
    rows = np.concatenate([near / np.linalg.norm(near, axis=1, keepdims=True), _unit(rng, n_far, d)]).astype(np.float32)
    rows = rows[rng.permutation(len(rows))]
    q = _unit(rng, nq, d)
    q[0] = v[0]
    if nq > 3:
        q[3] = (v[0] + np.float32(0.001) * rng.standard_normal(d)).astype(np.float32)
    qtab = rng.uniform(-1, 1, (2, len(rows))).astype(np.float32)
    print(f"crowded band {dtype} B={nq} k1={k1}", flush=True)
    bank = _make_bank(dtype, rows, qtab, max_B=max(nq, 8), max_k1=256)
    gpu = parity.gpu_retrieve(bank, torch, q, 1, k1, 8, 0.5)
    assert not bank.retrieve_flags(nq).cpu().numpy().any() and bank.counters() == (0, 0)
    st, qr = orc.round_to_store(rows, DT[dtype]), orc.round_to_store(q, DT[dtype])
    o_ids, o_sims = orc.recall(st, qr, k1, threads=8)
    in_band = ((o_sims[0, k1 - 1] - orc.sims_of(st, qr[0], np.arange(len(rows), dtype=np.int32))) < 2e-5).sum()
    assert in_band > 600                                        # the case is what it claims to be
    for b in range(nq):
        only_gpu = sorted(set(gpu["cand_ids"][b].tolist()) - set(o_ids[b].tolist()))
        if only_gpu:
            s_ = orc.sims_of(st, qr[b], np.array(only_gpu, np.int32))
            assert np.all(s_ > o_sims[b, k1 - 1] - 3e-7), (b, only_gpu, s_, o_sims[b, k1 - 1])
    stats = parity.check_retrieve(orc, st, qr, qtab[1], k1, 8, 0.5, gpu, ora_recall=(o_ids, o_sims))
    print("crowded band stats", stats, flush=True)
    bank.close()


# ----------------------------------------------------------------------------- value update

def _check_update(orc, bank, stage, table, ids, rewards, alpha):
    bank.update_q(_dev(ids), stage, _dev(rewards), alpha)
    got = bank.read_q(stage).cpu().numpy()
    w32, skipped = orc.update_q32(table, ids, rewards, alpha)
    w64, _ = orc.update_q64(table, ids, rewards, alpha)
    assert np.array_equal(got.view(np.uint32), w32.view(np.uint32))
    assert np.max(np.abs(got.astype(np.float64) - w64)) <= 1e-6
    return got, skipped


def test_update_q_duplicates_order_and_untouched_entries(orc):
    rng = np.random.default_rng(102)
    N = 5000
    rows = _unit(rng, N, 64)
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    bank = _make_bank("bf16", rows, qtab, max_B=8, max_k1=16)
    tables = [qtab[0].copy(), qtab[1].copy()]
    skipped_total = 0
    # (a) few ids, (b) heavy duplication incl. a long run, (c) out-of-range ids, (d) more than one launch chunk
    batches = [
        (0, np.array([3, 4, 3, 3], np.int32), np.array([1, 0, 0, 1], np.float32), 0.1),
        (1, np.concatenate([np.full(3000, 17), rng.integers(0, 50, 4000)]).astype(np.int32), None, 0.05),
        (0, np.array([-1, 5, N, 5, 2**31 - 1, 6, -2**31], np.int32), None, 0.5),
        (1, rng.integers(0, N, 20000).astype(np.int32), None, 0.3),
        (0, rng.permutation(N)[:4097].astype(np.int32), None, 1.0),
    ]
    for stage, ids, rewards, alpha in batches:
        if rewards is None:
            rewards = rng.uniform(-1, 1, ids.size).astype(np.float32)
        perm = rng.permutation(ids.size)
        ids, rewards = ids[perm], rewards[perm]
        other = bank.read_q(1 - stage).cpu().numpy()
        tables[stage], sk = _check_update(orc, bank, stage, tables[stage], ids, rewards, alpha)
        skipped_total += sk
        assert np.array_equal(bank.read_q(1 - stage).cpu().numpy().view(np.uint32), other.view(np.uint32))
    assert bank.counters() == (skipped_total, 0) and skipped_total == 4
    # alpha = 1: an id keeps the LAST reward given to it in array order
    ids = np.array([9, 8, 9, 9, 8], np.int32)
    r = np.array([0.1, 0.2, 0.3, 0.4, 0.5], np.float32)
    bank.update_q(_dev(ids), 0, _dev(r), 1.0)
    got = bank.read_q(0).cpu().numpy()
    assert got[9] == np.float32(0.4) and got[8] == np.float32(0.5)
    bank.update_q(_dev(ids[:0]), 0, _dev(r[:0]), 0.5)          # M = 0
    bank.close()


def test_update_q_zipf_batch(orc):
    """Heavily duplicated ids (Zipf s=1.1 through a fixed bijection), rewards U[0,1], step 0.05."""
    w = synth.scaled(synth.LARGE, N=1 << 18, d=64)
    rng = np.random.default_rng(103)
    bank = _make_bank("bf16", _unit(rng, 4096, 64), capacity=w.N, max_B=8, max_k1=16)
    # the Q tables cover the whole capacity only once the bank holds that many entries
    bank.append(_dev(_unit(rng, w.N - 4096, 64)))
    ids, rewards = synth.zipf_update(w, M=16384)
    top = np.bincount(ids).max()
    assert top > 1000                                           # one id really does dominate
    table = np.zeros(w.N, np.float32)
    got, _ = _check_update(orc, bank, 1, table, ids, rewards, 0.05)
    assert np.count_nonzero(got) == np.unique(ids).size
    bank.close()


# ----------------------------------------------------------------------------- the named workloads

def test_tiny_workload(orc):
    w = synth.TINY
    rows, q, qtab = synth.bank(w), synth.queries(w), synth.q_tables(w)
    bank = _make_bank(w.dtype, rows, qtab, max_B=8, max_k1=64)
    gpu = parity.gpu_retrieve(bank, torch, q, synth.DRAFT, w.k1, w.k2, w.lam)
    stats = parity.check_retrieve(orc, rows, q, qtab[0], w.k1, w.k2, w.lam, gpu)
    assert stats["boundary_swaps"] == 0 and stats["final_swaps"] == 0
    ids = gpu["ids"][0].astype(np.int32)
    rewards = np.array([1, 0, 1, 1], np.float32)
    _check_update(orc, bank, synth.DRAFT, qtab[0], ids, rewards, w.alpha)
    bank.close()


def test_mid_workload(orc):
    w = synth.MID
    rows, q = synth.bank(w), synth.queries(w)
    bank = _make_bank(w.dtype, rows, max_B=64, max_k1=64)
    tables = [np.zeros(w.N, np.float32), np.zeros(w.N, np.float32)]
    hits = [np.zeros(w.N, np.int64), np.zeros(w.N, np.int64)]
    for stage, ids, rewards in synth.ema_rounds(w):
        bank.update_q(_dev(ids), stage, _dev(rewards), w.alpha)
        tables[stage], _ = orc.update_q32(tables[stage], ids, rewards, w.alpha)
        hits[stage] += np.bincount(ids, minlength=w.N)
    for stage in (0, 1):
        got = bank.read_q(stage).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), tables[stage].view(np.uint32))
        # E[Q] after t Bernoulli(0.3) rewards from Q_0 = 0 is 0.3 (1 - 0.9^t)  (App. A, EMA lemma)
        assert abs(got.mean() - (0.3 * (1 - 0.9 ** hits[stage])).mean()) < 2e-3
    recall = orc.recall(rows, q, w.k1, threads=8)
    for stage in (0, 1):
        for lam in (0.0, 0.5, 1.0):
            print(f"mid stage={stage} lam={lam}", flush=True)
            gpu = parity.gpu_retrieve(bank, torch, q, stage, w.k1, w.k2, lam)
            stats = parity.check_retrieve(orc, rows, q, tables[stage], w.k1, w.k2, lam, gpu, ora_recall=recall)
            assert stats["boundary_swaps"] == 0
            if lam == 0.0:
                assert np.array_equal(gpu["ids"], gpu["cand_ids"][:, :w.k2])
    bank.close()


def _sampled_check(orc, w, bank, rows_rounded, q, qtab_stage, stage, sample, lam):
    gpu = parity.gpu_retrieve(bank, torch, q, stage, w.k1, w.k2, lam)
    qr = orc.round_to_store(q, DT[w.dtype])
    stats = parity.check_retrieve(orc, rows_rounded, qr, qtab_stage, w.k1, w.k2, lam, gpu, sample=sample, threads=16)
    # properties that hold for every query at any size
    assert np.all(gpu["cand_ids"] >= 0) and np.all(np.diff(gpu["cand_sims"], axis=1) <= 0)
    assert np.all(np.diff(gpu["scores"], axis=1) <= 0)
    for b in range(q.shape[0]):
        assert set(gpu["ids"][b].tolist()) <= set(gpu["cand_ids"][b].tolist())
    return gpu, stats


def test_clustered_workload_full_size(orc):
    """N = 1,048,576 x 1024 bf16, B = 256, k1 = 128, k2 = 16: the launch configuration the benchmark
    times.  The oracle checks all 256 queries over the full bank; near-ties are common here."""
    w = synth.CLUSTERED
    qtab = synth.q_tables(w)
    bank = B.MemoryBank(w.d, w.dtype, w.N, max_B=w.B, max_k1=w.k1)
    rounded = np.empty((w.N, w.d), np.float32)
    for j in range(synth.n_chunks(w)):
        c = synth.bank_chunk(w, j)
        a = j * synth.CHUNK_ROWS
        bank.append(_dev(c), _dev(qtab[0, a:a + len(c)]), _dev(qtab[1, a:a + len(c)]))
        rounded[a:a + len(c)] = orc.round_to_store(c, DT[w.dtype])
    print("clustered bank built", flush=True)
    q = synth.queries(w)
    sample = list(range(w.B))
    gpu, stats = _sampled_check(orc, w, bank, rounded, q, qtab[0], 0, sample, w.lam)
    print("clustered stats", stats, flush=True)
    assert stats["queries"] == w.B
    # near-ties are allowed (and counted) only inside 1e-5; with fp64 re-scoring of the pool there are none
    assert stats["boundary_swaps"] == 0 and stats["order_swaps"] == 0 and stats["final_swaps"] == 0
    # secondary bound for 16-bit storage: similarities of the rounded vectors stay within 2e-2
    # (relative) of the similarities of the unrounded fp32 vectors
    for b in sample[:3]:
        ids = gpu["cand_ids"][b][:8]
        raw = np.stack([synth.bank_chunk(w, int(i) // synth.CHUNK_ROWS)[int(i) % synth.CHUNK_ROWS] for i in ids])
        true = raw.astype(np.float64) @ q[b].astype(np.float64)
        assert np.all(np.abs(gpu["cand_sims"][b][:8] - true) <= 2e-2 * np.abs(true))
    g0 = parity.gpu_retrieve(bank, torch, q, 0, w.k1, w.k2, 0.0)
    assert np.array_equal(g0["ids"], g0["cand_ids"][:, :w.k2])          # lambda = 0: similarity ranking
    # the exhaustive call (every entry scored in fp64, no thresholds) on four of the queries: judged by the oracle
    # like the scan's result, and here equal to it
    import time
    qd = _dev(q[:4])
    bank.retrieve_exact(qd, 0, w.k1, w.k2, w.lam)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ids, sc, cid, csim = bank.retrieve_exact(qd, 0, w.k1, w.k2, w.lam, want_candidates=True)
    torch.cuda.synchronize()
    print(f"exhaustive retrieve, 4 queries over {w.N} entries: {(time.perf_counter() - t0) * 1e3:.1f} ms", flush=True)
    ex = {"ids": ids.cpu().numpy(), "scores": sc.cpu().numpy(), "cand_ids": cid.cpu().numpy(), "cand_sims": csim.cpu().numpy()}
    qr4 = orc.round_to_store(q[:4], DT[w.dtype])
    parity.check_retrieve(orc, rounded, qr4, qtab[0], w.k1, w.k2, w.lam, ex, threads=4)
    for k in ex:
        assert np.array_equal(ex[k].view(np.uint32), gpu[k][:4].view(np.uint32)), k
    assert bank.counters() == (0, 0)
    bank.close()


def test_large_workload_reduced(orc):
    """Shape of the large batched workload (d = 1536 bf16, B = 1024, k1 = 128, refine stage) on a
    262,144-entry bank, 8 sampled queries against the oracle."""
    w = synth.scaled(synth.LARGE, N=1 << 18)
    rows = synth.bank(w)
    qtab = synth.q_tables(w)
    bank = _make_bank(w.dtype, rows, qtab, max_B=w.B, max_k1=w.k1)
    rounded = orc.round_to_store(rows, DT[w.dtype])
    q = synth.queries(w)
    _, stats = _sampled_check(orc, w, bank, rounded, q, qtab[1], 1, [0, 255, 256, 511, 600, 767, 1000, 1023], w.lam)
    print("large stats", stats, flush=True)
    assert bank.counters() == (0, 0)
    bank.close()


def test_stream_workload_reduced(orc):
    """Shape of the streaming workload (d = 4096 fp16, B = 128, k1 = 256, k2 = 32, lambda 0.7): the
    bank grows by 16,384-entry chunks from 32,768; every step appends, retrieves (alternating
    stage) and updates the B*k2 returned ids with Bernoulli(0.2) rewards."""
    w = synth.scaled(synth.STREAM, N=1 << 17)
    chunk, n0, steps = 16384, 32768, 4
    bank = B.MemoryBank(w.d, w.dtype, n0 + steps * chunk, max_B=w.B, max_k1=w.k1)
    rows = np.concatenate([synth.bank_chunk(w, j, chunk) for j in range(n0 // chunk + steps)])
    rounded = orc.round_to_store(rows, DT[w.dtype])
    bank.append(_dev(rows[:n0]))
    tables = [np.zeros(n0 + steps * chunk, np.float32) for _ in range(2)]
    n = n0
    for t in range(steps):
        bank.append(_dev(rows[n:n + chunk]))
        n += chunk
        stage = t % 2
        q = synth.queries(w, step=t)
        print(f"stream step {t} N={n}", flush=True)
        gpu = parity.gpu_retrieve(bank, torch, q, stage, w.k1, w.k2, w.lam)
        qr = orc.round_to_store(q, DT[w.dtype])
        parity.check_retrieve(orc, rounded[:n], qr, tables[stage][:n], w.k1, w.k2, w.lam, gpu, sample=[0, 64, 127])
        ids = gpu["ids"].reshape(-1).astype(np.int32)
        rewards = synth.bernoulli_rewards(w, t, ids.size)
        bank.update_q(_dev(ids), stage, _dev(rewards), w.alpha)
        tables[stage][:n], _ = orc.update_q32(tables[stage][:n], ids, rewards, w.alpha)
        assert np.array_equal(bank.read_q(stage).cpu().numpy().view(np.uint32), tables[stage][:n].view(np.uint32))
    assert bank.counters() == (0, 0)
    bank.close()


# ----------------------------------------------------------------------------- epsilon-greedy selection (Sec. 3.3)

@pytest.mark.parametrize("dtype,N,d,nq,k1,k2,eps", [
    ("f32", 3000, 96, 3, 40, 8, 0.3),        # VALU scan
    ("bf16", 20000, 256, 70, 128, 16, 0.25),  # MFMA scan, pool of the bench configuration
    ("f16", 9000, 192, 33, 256, 32, 1.0),     # largest pool, every slot random
    ("f32", 50, 64, 5, 64, 64, 0.5),          # pool smaller than k1, k2 = k1: all members chosen, padding
])
def test_retrieve_eps_matches_oracle(orc, dtype, N, d, nq, k1, k2, eps):
    """Same pool as the greedy call; the slots must be the ones the oracle fills from the GPU's pool with the same
    (seed, step, query, slot) draws: ids, flags and slot order bit-exact, scores within tolerance."""
    rng = np.random.default_rng(N + k1)
    rows, q = _unit(rng, N, d), _unit(rng, nq, d)
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    bank = _make_bank(dtype, rows, qtab, max_B=128)
    seed, step, lam, stage = 0x9E3779B97F4A7C15, (1 << 33) + 5, 0.5, 1
    greedy = parity.gpu_retrieve(bank, torch, q, stage, k1, k2, lam)
    ids, sc, cid, csim, ex = bank.retrieve_eps(_dev(q), stage, k1, k2, lam, eps, seed, step, want_candidates=True)
    torch.cuda.synchronize()
    ids, sc, cid, ex = ids.cpu().numpy(), sc.cpu().numpy(), cid.cpu().numpy(), ex.cpu().numpy()
    assert np.array_equal(cid, greedy["cand_ids"])                       # the pool does not depend on eps
    store, qs = orc.round_to_store(rows, DT[dtype]), orc.round_to_store(q, DT[dtype])
    k1e = min(k1, N)
    n_explored = 0
    for b in range(nq):
        pool = cid[b][:k1e]
        sims = orc.sims_of(store, qs[b], pool)
        w_ids, _, w_sc, w_ex = orc.rerank_eps(pool, sims, qtab[stage], lam, k2, eps, seed, step, b)
        assert np.array_equal(ids[b], w_ids), f"query {b}: {ids[b]} vs {w_ids}"
        assert np.array_equal(ex[b], w_ex)
        live = w_ids >= 0
        assert np.all(np.abs(sc[b][live].astype(np.float64) - w_sc[live]) <= parity.TOL * np.maximum(1.0, np.abs(w_sc[live])))
        assert np.all(np.isneginf(sc[b][~live]))
        n_explored += int(w_ex.sum())
    if eps == 1.0:
        assert n_explored == nq * min(k2, k1e)
    # eps = 0 through the same entry point is the greedy result, and a different step gives other draws
    ids0, sc0, _, _, ex0 = bank.retrieve_eps(_dev(q), stage, k1, k2, lam, 0.0, seed, step)
    assert np.array_equal(ids0.cpu().numpy(), greedy["ids"]) and not ex0.cpu().numpy().any()
    assert np.array_equal(sc0.cpu().numpy(), greedy["scores"])
    if eps >= 0.25 and nq * k2 >= 64:
        ids2, _, _, _, _ = bank.retrieve_eps(_dev(q), stage, k1, k2, lam, eps, seed, step + 1)
        assert not np.array_equal(ids2.cpu().numpy(), ids)
    with pytest.raises(B.MemError):
        bank.retrieve_eps(_dev(q), stage, k1, k2, lam, 1.5, seed, step)
    bank.close()


# ----------------------------------------------------------------------------- stage rewards (Sec. 3.3, 3.4, App. A)

def test_stage_rewards_and_online_normalisation(orc):
    rng = np.random.default_rng(108)
    N = 4000
    bank = _make_bank("f32", _unit(rng, N, 64), max_B=8, max_k1=16)
    tol = lambda ref: 1e-6 * np.maximum(1.0, np.abs(ref))
    state = [None, None]
    for M in (1, 1023, 1024, 1025, 5000):           # pieces of 1024 inside the kernel: below, at, above, several
        feas = (rng.random(M) < 0.75).astype(np.uint8)
        lat = rng.uniform(0.2, 30, M).astype(np.float32)
        best = rng.uniform(0.2, 30, M).astype(np.float32)
        # stage 1 rewards: exact
        r1 = bank.shape_rewards(0, _dev(feas)).cpu().numpy()
        assert np.array_equal(r1, np.where(feas, 1.0, -1.0).astype(np.float32))
        # stage 2 raw rewards
        r2 = bank.shape_rewards(1, _dev(feas), _dev(lat), _dev(best)).cpu().numpy()
        w2, _ = orc.shape_rewards(1, feas, lat, best, False)
        assert np.all(np.abs(r2 - w2) <= tol(w2)) and np.all(r2[feas == 0] == -1.0)
        # normalised, statistics carried from call to call (both stages keep their own)
        for stage, clip in ((1, 0.0), (0, 2.5)):
            got = bank.shape_rewards(stage, _dev(feas), _dev(lat), _dev(best), normalise=True, sigma_min=0.05, clip=clip)
            want, state[stage] = orc.shape_rewards(stage, feas, lat, best, True, 0.05, clip, state=state[stage])
            got = got.cpu().numpy()
            assert np.all(np.abs(got - want) <= tol(want)), (M, stage, np.max(np.abs(got - want)))
            n, mu, sd = bank.reward_stats(stage)
            s = state[stage]
            assert n == s[0] and abs(mu - s[1] / s[0]) < 1e-12 and abs(sd - np.sqrt(max(s[2] / s[0] - (s[1] / s[0]) ** 2, 0))) < 1e-9
    # the rewards feed the value update: Q after the update is the sequential fp32 recurrence on them
    ids = rng.integers(0, N, 5000).astype(np.int32)
    rewards = bank.shape_rewards(1, _dev(feas), _dev(lat), _dev(best), normalise=True, sigma_min=0.05)
    bank.update_q(_dev(ids), 1, rewards, 0.1)
    want_q, _ = orc.update_q32(np.zeros(N, np.float32), ids, rewards.cpu().numpy(), 0.1)
    assert np.array_equal(bank.read_q(1).cpu().numpy().view(np.uint32), want_q.view(np.uint32))
    bank.reward_stats_reset(1)
    assert bank.reward_stats(1) == (0.0, 0.0, 0.0) and bank.reward_stats(0)[0] > 0
    with pytest.raises(B.MemError):
        bank.shape_rewards(1, _dev(feas), _dev(lat), _dev(best), normalise=True, sigma_min=0.0)
    with pytest.raises(B.MemError):
        bank.shape_rewards(1, _dev(feas))            # stage 2 needs the latencies
    bank.close()


# ----------------------------------------------------------------------------- typed / masked retrieval

def _check_masked(orc, bank, dtype, rows, q, tags, allow, exclude, qtab, stage, k1, k2, lam):
    ids, sc, cid, csim = bank.retrieve_masked(_dev(q), stage, k1, k2, lam, torch.from_numpy(allow.astype(np.int64)),
                                              torch.from_numpy(exclude.astype(np.int64)), want_candidates=True)
    torch.cuda.synchronize()
    gpu = {"ids": ids.cpu().numpy(), "scores": sc.cpu().numpy(), "cand_ids": cid.cpu().numpy(), "cand_sims": csim.cpu().numpy()}
    st, qr = orc.round_to_store(rows, DT[dtype]), orc.round_to_store(q, DT[dtype])
    types, groups = tags & 0xff, tags >> 8
    total = {"queries": 0, "boundary_swaps": 0}
    for b in range(len(q)):
        keep = np.flatnonzero((types < 32) & ((allow[b] >> (types & 31)) & 1).astype(bool) & (groups != exclude[b]))
        # the pool may only hold accepted entries ...
        pool = gpu["cand_ids"][b]
        assert set(pool[pool >= 0].tolist()) <= set(keep.tolist()), f"query {b}: pool holds entries it does not accept"
        # ... and must be the oracle's masked top-k1: compare on the sub-bank of accepted entries (ids mapped)
        if len(keep) == 0:
            assert np.all(pool == -1) and np.all(gpu["ids"][b] == -1)
            continue
        back = {int(g): i for i, g in enumerate(keep)}
        sub = {"cand_ids": np.array([[back.get(int(i), -1) for i in pool]], np.int32), "cand_sims": gpu["cand_sims"][b:b + 1],
               "ids": np.array([[back.get(int(i), -1) for i in gpu["ids"][b]]], np.int32), "scores": gpu["scores"][b:b + 1]}
        s = parity.check_retrieve(orc, np.ascontiguousarray(st[keep]), qr[b:b + 1], qtab[stage][keep], k1, k2, lam, sub)
        total["queries"] += 1
        total["boundary_swaps"] += s["boundary_swaps"]
    # the oracle's own masked recall agrees too (ids, up to boundary near-ties already judged above)
    o_ids, _ = orc.recall_masked(st, tags, qr, allow, exclude, k1)
    if total["boundary_swaps"] == 0:
        assert np.array_equal(np.sort(o_ids, axis=1), np.sort(gpu["cand_ids"], axis=1))
    return total


def test_masked_retrieval_with_a_crowded_band(orc):
    """Typed retrieval over a bank with thousands of near-duplicates of one row: the accepted half of them
    crowds the band after the last pass (the refinement of the selection also runs with empty list slots),
    eps-greedy selection on the same bank stays consistent with the greedy pool."""
    rng = np.random.default_rng(131)
    d, n_near, n_far = 128, 2600, 6000
    v = _unit(rng, 1, d)
    near = v + np.float32(0.001) * rng.standard_normal((n_near, d)).astype(np.float32) * rng.uniform(0, 1, (n_near, 1)).astype(np.float32)
    rows = np.concatenate([near / np.linalg.norm(near, axis=1, keepdims=True), _unit(rng, n_far, d)]).astype(np.float32)
    rows = rows[rng.permutation(len(rows))]
    N = len(rows)
    tags = (rng.integers(0, 2, N) | (rng.integers(0, 50, N) << 8)).astype(np.uint32)      # two types, 50 groups
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    q = _unit(rng, 6, d)
    q[0] = v[0]
    q[5] = v[0]
    allow = np.array([1, 3, 2, 1, 3, 2], np.uint32)
    exclude = np.array([0xffffffff, 7, 0xffffffff, 3, 0xffffffff, 11], np.uint32)
    bank = _make_bank("bf16", rows, qtab, max_B=8, max_k1=256)
    bank.set_tags(0, torch.from_numpy(tags.astype(np.int64)))
    total = _check_masked(orc, bank, "bf16", rows, q, tags, allow, exclude, qtab, 0, 64, 8, 0.5)
    assert total["queries"] == 6 and not bank.retrieve_flags(6).cpu().numpy().any()
    # eps-greedy on the crowded, unmasked bank: eps = 0 equals the greedy call bit for bit
    a = bank.retrieve(_dev(q), 0, 64, 8, 0.5, want_candidates=True)
    b_ = bank.retrieve_eps(_dev(q), 0, 64, 8, 0.5, 0.0, 1, 2, want_candidates=True)
    torch.cuda.synchronize()
    for x, y in zip(a, b_[:4]):
        assert np.array_equal(x.cpu().numpy().view(np.uint32), y.cpu().numpy().view(np.uint32))
    bank.close()


@pytest.mark.parametrize("dtype,N,d,nq", [("f32", 5000, 96, 3), ("bf16", 30000, 256, 70), ("f16", 12000, 128, 200), ("bf16", 9000, 64, 1)])
def test_masked_retrieval_matches_oracle(orc, dtype, N, d, nq):
    rng = np.random.default_rng(N + nq)
    rows, q = _unit(rng, N, d), _unit(rng, nq, d)
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    types = rng.choice(4, N, p=[0.55, 0.3, 0.13, 0.02]).astype(np.uint32)      # type 3 is rare
    groups = rng.integers(0, 40, N).astype(np.uint32)
    tags = types | (groups << 8)
    bank = _make_bank(dtype, rows, qtab, max_B=256)
    # before tags are attached the call is refused
    with pytest.raises(B.MemError) as e:
        bank.retrieve_masked(_dev(q), 0, 8, 2, 0.5, torch.zeros(nq, dtype=torch.int64), torch.zeros(nq, dtype=torch.int64))
    assert e.value.status == B.MEM_ESTATE
    bank.set_tags(0, torch.from_numpy(tags[:N // 2].astype(np.int64)))
    bank.set_tags(N // 2, torch.from_numpy(tags[N // 2:].astype(np.int64)))
    allow = rng.choice([0b0001, 0b0010, 0b0011, 0b0100, 0b1111, 0b1000], nq).astype(np.uint32)
    exclude = np.where(rng.random(nq) < 0.5, rng.integers(0, 40, nq), 0xffffffff).astype(np.uint32)
    k1, k2 = (64, 8) if nq > 1 else (32, 4)
    got = _check_masked(orc, bank, dtype, rows, q, tags, allow, exclude, qtab, 1, k1, k2, 0.5)
    assert got["queries"] == nq
    # accepting everything reproduces the plain call bit for bit
    plain = parity.gpu_retrieve(bank, torch, q, 1, k1, k2, 0.5)
    ids, sc, cid, csim = bank.retrieve_masked(_dev(q), 1, k1, k2, 0.5, torch.full((nq,), 0xffffffff, dtype=torch.int64),
                                              torch.full((nq,), 0xffffffff, dtype=torch.int64), want_candidates=True)
    assert np.array_equal(cid.cpu().numpy(), plain["cand_ids"]) and np.array_equal(ids.cpu().numpy(), plain["ids"])
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), plain["scores"].view(np.uint32))
    # a query that accepts nothing, and one whose accepted entries are fewer than k1
    few = np.zeros(N, np.uint32)
    few[rng.permutation(N)[:10]] = 5
    bank.set_tags(0, torch.from_numpy(few.astype(np.int64)))
    allow2 = np.array([0, 1 << 5] + [1] * (nq - 2), np.uint32)[:nq] if nq >= 2 else np.array([1 << 5], np.uint32)
    got = _check_masked(orc, bank, dtype, rows, q, few, allow2, np.full(nq, 0xffffffff, np.uint32), qtab, 0, k1, k2, 0.5)
    assert bank.counters() == (0, 0)
    bank.close()


# ----------------------------------------------------------------------------- pools larger than 256 (Sec. 4.4, pool-size study)

@pytest.mark.parametrize("dtype,N,d,nq,k1,k2", [
    ("bf16", 40000, 128, 24, 960, 32),      # 30x over-retrieval
    ("f16", 30000, 64, 9, 2048, 64),        # the largest pool
    ("f32", 20000, 96, 3, 300, 300),        # VALU scan, k2 = k1: the whole pool comes back
    ("bf16", 700, 64, 6, 1024, 16),         # pool larger than the bank
])
def test_large_pools_match_oracle(orc, dtype, N, d, nq, k1, k2):
    rng = np.random.default_rng(N + k1)
    rows, q = _unit(rng, N, d), _unit(rng, nq, d)
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    bank = _make_bank(dtype, rows, qtab, max_B=32, max_k1=2048)
    st, qr = orc.round_to_store(rows, DT[dtype]), orc.round_to_store(q, DT[dtype])
    for stage, lam in ((0, 0.5), (1, 1.0)):
        gpu = parity.gpu_retrieve(bank, torch, q, stage, k1, k2, lam)
        stats = parity.check_retrieve(orc, st, qr, qtab[stage], k1, k2, lam, gpu)
        assert stats["queries"] == nq
    # a small pool through the same handle still takes the small-pool kernels and matches
    gpu = parity.gpu_retrieve(bank, torch, q, 0, 64, 8, 0.5)
    parity.check_retrieve(orc, st, qr, qtab[0], 64, 8, 0.5, gpu)
    # epsilon-greedy over the large pool
    seed, step = 77, 12345
    ids, sc, cid, _, ex = bank.retrieve_eps(_dev(q), 0, k1, k2, 0.5, 0.3, seed, step, want_candidates=True)
    ids, sc, cid, ex = ids.cpu().numpy(), sc.cpu().numpy(), cid.cpu().numpy(), ex.cpu().numpy()
    k1e = min(k1, N)
    for b in range(nq):
        pool = cid[b][:k1e]
        w_ids, _, w_sc, w_ex = orc.rerank_eps(pool, orc.sims_of(st, qr[b], pool), qtab[0], 0.5, k2, 0.3, seed, step, b)
        assert np.array_equal(ids[b], w_ids) and np.array_equal(ex[b], w_ex)
        live = w_ids >= 0
        assert np.all(np.abs(sc[b][live].astype(np.float64) - w_sc[live]) <= parity.TOL * np.maximum(1.0, np.abs(w_sc[live])))
    assert bank.counters() == (0, 0)
    bank.close()


# ----------------------------------------------------------------------------- a bank saved and continued

def test_bank_saved_and_restored_gives_identical_results(orc):
    rng = np.random.default_rng(109)
    N, d = 6000, 80
    rows, q = _unit(rng, N, d), _unit(rng, 12, d)
    qtab = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    a = _make_bank("bf16", rows, qtab, capacity=8000, max_B=16, max_k1=64)
    a.set_tags(0, torch.from_numpy((rng.integers(0, 3, N) | (rng.integers(0, 5, N) << 8)).astype(np.int64)))
    a.update_q(_dev(rng.integers(0, N, 500).astype(np.int32)), 1, _dev(rng.random(500).astype(np.float32)), 0.2)
    saved = a.state()
    want = parity.gpu_retrieve(a, torch, q, 1, 64, 8, 0.5)
    al, ex = torch.full((12,), 0b101, dtype=torch.int64), torch.full((12,), 2, dtype=torch.int64)
    want_m = [t.cpu().numpy() for t in a.retrieve_masked(_dev(q), 1, 64, 8, 0.5, al, ex)[:2]]
    a.close()
    b = B.MemoryBank(d, "bf16", 8000, max_B=16, max_k1=64)
    assert b.size() == 0
    b.load_state(saved)
    assert b.size() == N
    got = parity.gpu_retrieve(b, torch, q, 1, 64, 8, 0.5)
    for k in want:
        assert np.array_equal(want[k].view(np.uint32), got[k].view(np.uint32)), k
    got_m = [t.cpu().numpy() for t in b.retrieve_masked(_dev(q), 1, 64, 8, 0.5, al, ex)[:2]]
    assert np.array_equal(want_m[0], got_m[0]) and np.array_equal(want_m[1].view(np.uint32), got_m[1].view(np.uint32))
    # and it keeps growing from where it was
    assert b.append(_dev(_unit(rng, 10, d))) == N
    with pytest.raises(B.MemError):
        b.lib and B._check(b.lib.mem_restore(b.h, 9000), "mem_restore")
    b.close()


# ----------------------------------------------------------------------------- start-point selection (Sec. 3.4)

def _start_sets(rng, N, G, lens):
    parts, off = [], [0]
    for g in range(G):
        n = int(lens[g % len(lens)])
        ids = rng.integers(0, N, n).astype(np.int32)
        if n:
            ids[rng.random(n) < 0.05] = rng.choice([-1, N, N + 3, 2**31 - 1, -2**31])
        parts.append(ids); off.append(off[-1] + n)
    return np.concatenate(parts), np.array(off, np.int64)


@pytest.mark.parametrize("eps", [0.0, 0.3, 1.0])
def test_select_by_q_matches_oracle(orc, eps):
    """Ids, values and exploration flags bit-exact: empty sets, singletons, sets spanning several chunks of the
    workgroup, repeated ids, ids outside the bank, tied values (the table has few distinct values, +-0, NaN, -inf)."""
    rng = np.random.default_rng(300)
    N = 20000
    qtab = np.zeros((2, N), np.float32)
    qtab[0] = rng.uniform(-1, 1, N)
    qtab[1] = rng.choice(np.array([-np.inf, -1.0, -0.0, 0.0, 0.5, np.nan], np.float32), N)
    bank = _make_bank("bf16", _unit(rng, N, 64), qtab, max_B=8, max_k1=16)
    lens = [0, 1, 2, 7, 63, 64, 65, 255, 256, 257, 1000, 1024, 1025, 5000, 0, 33]
    ids, off = _start_sets(rng, N, 64, lens)
    skipped_total = 0
    for stage, seed, step in ((0, 11, 0), (1, 2**63 + 5, (9 << 32) | 77)):
        got_id, got_q, got_ex = bank.select_by_q(_dev(ids), _dev(off), stage, eps, seed, step)
        want_id, want_q, want_ex, skipped = orc.select_by_q(ids, off, qtab[stage], eps, seed, step)
        skipped_total += skipped
        assert np.array_equal(got_id.cpu().numpy(), want_id)
        assert np.array_equal(got_q.cpu().numpy().view(np.uint32), want_q.view(np.uint32))
        assert np.array_equal(got_ex.cpu().numpy(), want_ex)
        if eps == 0.0:
            assert not want_ex.any()
        if eps == 1.0:
            assert want_ex[want_id >= 0].all()
    assert bank.counters() == (skipped_total, 0) and skipped_total > 0
    bank.close()


def test_select_by_q_follows_updates_and_rejects_bad_arguments(orc):
    """The selection reads the table mem_update_q writes; argument errors are reported, not executed."""
    rng = np.random.default_rng(301)
    N = 3000
    bank = _make_bank("f16", _unit(rng, N, 32), max_B=8, max_k1=16)
    ids = np.array([5, 9, 12, 700, 2999], np.int32)
    off = np.array([0, 5], np.int64)
    got, val, _ = bank.select_by_q(_dev(ids), _dev(off), 1)
    assert int(got[0]) == 5 and float(val[0]) == 0.0                       # all values 0: the lowest id
    bank.update_q(_dev(np.array([700, 12, 700], np.int32)), 1, _dev(np.array([1.0, 0.2, 1.0], np.float32)), 0.5)
    table, _ = orc.update_q32(np.zeros(N, np.float32), np.array([700, 12, 700], np.int32),
                              np.array([1.0, 0.2, 1.0], np.float32), 0.5)
    got, val, _ = bank.select_by_q(_dev(ids), _dev(off), 1)
    assert int(got[0]) == 700 and float(val[0]) == table[700]
    got, _, _ = bank.select_by_q(_dev(ids), _dev(off), 0)                  # the other stage's table is untouched
    assert int(got[0]) == 5
    # offsets that point outside the id array are clamped to it
    got, _, _ = bank.select_by_q(_dev(ids), _dev(np.array([-4, 3, 99], np.int64)), 1)
    assert got.cpu().tolist() == [12, 700]
    empty = bank.select_by_q(_dev(ids), _dev(np.array([0], np.int64)), 1)
    assert empty[0].numel() == 0
    for kwargs in ({"stage": 2}, {"eps": 1.5}, {"eps": float("nan")}, {"eps": -0.1}):
        args = {"stage": 1, "eps": 0.0}
        args.update(kwargs)
        with pytest.raises(B.MemError) as e:
            bank.select_by_q(_dev(ids), _dev(off), args["stage"], args["eps"])
        assert e.value.status == B.MEM_EINVAL
    bank.close()
