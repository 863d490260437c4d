"""Parity at the full sizes of the two largest workloads: sampled queries against the oracle over the
WHOLE bank.

  large   4,194,304 x 1536 bf16, 1024 queries, 32 of them sampled: runs by default (about three minutes).
  stream  d = 4096 fp16, 128 queries, k1 = 256, 32 of them sampled: by default on a 589,824-entry bank
          (2.4e9 stored elements, so every offset beyond 2^31 elements is exercised; under a minute);
          at the full 8,388,608 entries (68.7 GB, the oracle needs eleven minutes to stream through
          them) only when EVOMEM_FULL_SIZE=1 is set:
              EVOMEM_FULL_SIZE=1 python -m pytest tests/test_gpu_full_size.py -m gpu -x -q -s
The bank never exists on the host.  Pass 1 generates each 65,536-row chunk, appends it to the GPU
bank and hands the same fp32 rows to the oracle, which keeps a running top-k1 per sampled query.
After the GPU retrieve, pass 2 regenerates the chunks and collects only the rows that either side
named; ids are then renumbered in increasing order (which keeps every lower-id tie-break) and the
usual checks run on that small table."""
import os
import time

import numpy as np
import pytest
import torch

from paper_2603_10846_amd import binding as B
from paper_2603_10846_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu
DT = {"f32": 0, "bf16": 1, "f16": 2}
DEV = "cuda:0"


def _device_chunk(w, j, rows):
    """fp32 rows of chunk j, normalised Gaussian, generated on the device from the seed (SEED + index, j)."""
    g = torch.Generator(device=DEV).manual_seed((synth.SEED + w.index) * 100003 + j)
    x = torch.randn((rows, w.d), device=DEV, generator=g)
    return x / x.norm(dim=1, keepdim=True)


def _full_size_check(orc, w, stage, sample, chunk_of, say):
    nchunks = synth.n_chunks(w)
    rng = np.random.default_rng(synth.SEED + w.index)
    qtab = rng.uniform(-1, 1, (2, w.N)).astype(np.float32)
    q = synth.queries(w)
    qr = orc.round_to_store(q, DT[w.dtype])
    sel = np.ascontiguousarray(qr[sample])
    bank = B.MemoryBank(w.d, w.dtype, w.N, max_B=w.B, max_k1=w.k1)
    run_ids = np.full((len(sample), w.k1), -1, np.int32)
    run_sims = np.full((len(sample), w.k1), -np.inf, np.float64)
    t0 = time.time()
    for j in range(nchunks):
        a = j * synth.CHUNK_ROWS
        rows = min(synth.CHUNK_ROWS, w.N - a)
        x = chunk_of(w, j, rows)
        xd = x if torch.is_tensor(x) else torch.from_numpy(x).to(DEV)
        dev = lambda v: torch.from_numpy(np.ascontiguousarray(v)).to(DEV)
        assert bank.append(xd, dev(qtab[0, a:a + rows]), dev(qtab[1, a:a + rows])) == a
        xh = orc.round_to_store(x.cpu().numpy() if torch.is_tensor(x) else x, DT[w.dtype])
        part = orc.recall(xh, sel, w.k1, id_base=a, threads=16)
        run_ids, run_sims = orc.merge_recall([(run_ids, run_sims), part], w.k1)
        if j % 4 == 3 or j == nchunks - 1:
            say(f"{w.name}: chunk {j + 1}/{nchunks} appended and scanned by the oracle, {time.time() - t0:.0f} s")
    gpu = parity.gpu_retrieve(bank, torch, q, stage, w.k1, w.k2, w.lam)
    say(f"{w.name}: GPU retrieve done")
    # properties for every query
    assert np.all(gpu["cand_ids"] >= 0) and np.all(np.diff(gpu["cand_sims"], axis=1) <= 0)
    assert np.all(np.diff(gpu["scores"], axis=1) <= 0)
    # the rows either side named, renumbered in increasing id order
    need = np.unique(np.concatenate([gpu["cand_ids"][sample].ravel(), run_ids.ravel()]))
    need = need[need >= 0]
    small = np.empty((need.size, w.d), np.float32)
    for j in np.unique(need // synth.CHUNK_ROWS):
        a = int(j) * synth.CHUNK_ROWS
        rows = min(synth.CHUNK_ROWS, w.N - a)
        x = chunk_of(w, int(j), rows)
        where = np.nonzero(need // synth.CHUNK_ROWS == j)[0]
        local = need[where] - a
        picked = x[torch.from_numpy(local).to(DEV)].cpu().numpy() if torch.is_tensor(x) else x[local]
        small[where] = orc.round_to_store(picked, DT[w.dtype])
    say(f"{w.name}: {need.size} rows collected for the comparison")
    renum = lambda ids: np.where(ids >= 0, np.searchsorted(need, np.maximum(ids, 0)), -1).astype(np.int32)
    gpu_small = {"ids": gpu["ids"].copy(), "scores": gpu["scores"], "cand_ids": gpu["cand_ids"].copy(), "cand_sims": gpu["cand_sims"]}
    for b in sample:
        gpu_small["ids"][b] = renum(gpu["ids"][b])
        gpu_small["cand_ids"][b] = renum(gpu["cand_ids"][b])
    stats = parity.check_retrieve(orc, small, qr, qtab[stage][need], w.k1, w.k2, w.lam, gpu_small,
                                  ora_recall=(renum(run_ids), run_sims), sample=sample)
    say(f"{w.name}: {stats}")
    assert bank.counters() == (0, 0)
    bank.close()
    return stats


def _sample32(B):
    """32 query rows: both ends of every 256-query tile the scan forms, the rest spread evenly."""
    edges = {0, B - 1} | {t for t in range(256, B, 256)} | {t - 1 for t in range(256, B, 256)}
    rest = [int(x) for x in np.linspace(5, B - 6, 32 - len(edges))]
    return sorted(edges | set(rest))


def test_large_workload_full_size(orc, capsys):
    w = synth.LARGE
    with capsys.disabled():
        say = lambda s: print(s, flush=True)
        sample = _sample32(w.B)
        assert len(sample) == 32
        stats = _full_size_check(orc, w, synth.REFINE, sample, lambda w, j, rows: synth.bank_chunk(w, j), say)
        assert stats["queries"] == 32


def test_stream_workload_beyond_2g_elements(orc, capsys):
    w = synth.scaled(synth.STREAM, N=9 * synth.CHUNK_ROWS)
    assert w.N * w.d > 2**31
    with capsys.disabled():
        say = lambda s: print(s, flush=True)
        sample = _sample32(w.B)
        stats = _full_size_check(orc, w, synth.DRAFT, sample, _device_chunk, say)
        assert stats["queries"] == 32


@pytest.mark.skipif(os.environ.get("EVOMEM_FULL_SIZE") != "1", reason="set EVOMEM_FULL_SIZE=1 (eleven minutes)")
def test_stream_workload_full_size(orc, capsys):
    w = synth.STREAM
    with capsys.disabled():
        say = lambda s: print(s, flush=True)
        _full_size_check(orc, w, synth.REFINE, _sample32(w.B), _device_chunk, say)
