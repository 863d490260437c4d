"""The retrieve variant that allocates nothing (its scratch is an array inside the library) against
the ordinary entry point, through the C ABI: same inputs, outputs compared bit for bit, two calls in
a row of which the second is smaller, then its limits.  The ordinary entry point is itself checked
against the oracle by the parity tests."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2603_10846_amd import binding as B

pytestmark = pytest.mark.gpu


def _unit(rng, n, d):
    x = rng.standard_normal((n, d)).astype(np.float32)
    return x / np.linalg.norm(x, axis=1, keepdims=True)


def _outs(nq, k1, k2):
    dev = "cuda:0"
    return (torch.full((nq, k2), -7, dtype=torch.int32, device=dev), torch.full((nq, k2), 7.0, dtype=torch.float32, device=dev),
            torch.full((nq, k1), -7, dtype=torch.int32, device=dev), torch.full((nq, k1), 7.0, dtype=torch.float32, device=dev))


def _same(a, b):
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert np.array_equal(x.cpu().numpy().view(np.uint32), y.cpu().numpy().view(np.uint32))


@pytest.mark.parametrize("dtype,N,d", [("bf16", 70000, 256), ("f32", 30000, 72), ("f16", 9000, 2048)])
def test_static_retrieve_equals_retrieve(dtype, N, d):
    rng = np.random.default_rng([5, N, d])
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    bank = B.MemoryBank(d, dtype, N, max_B=64, max_k1=256)
    bank.append(dev(_unit(rng, N, d)), dev(rng.uniform(-1, 1, N).astype(np.float32)), dev(rng.uniform(-1, 1, N).astype(np.float32)))
    # two calls in a row, the second with a smaller batch, pool and final count (and the other stage)
    for nq, stage, k1, k2, lam in ((64, 0, 256, 32, 0.5), (3, 1, 16, 4, 0.25), (40, 1, 128, 16, 1.0), (1, 0, 64, 8, 0.0)):
        print(f"static retrieve {dtype} N={N} d={d} B={nq} k1={k1}", flush=True)
        q = dev(_unit(rng, nq, d))
        want = bank.retrieve(q, stage, k1, k2, lam, out=_outs(nq, k1, k2))
        got = bank.retrieve_static(q, stage, k1, k2, lam, _outs(nq, k1, k2))
        _same(got, want)
    # the handle's own workspace is not touched by the static call
    before = bank.workspace.clone()
    q = dev(_unit(rng, 17, d))
    bank.retrieve_static(q, 0, 32, 4, 0.5, _outs(17, 32, 4))
    torch.cuda.synchronize()
    assert torch.equal(before, bank.workspace)
    assert bank.counters() == (0, 0)
    bank.close()


def test_static_retrieve_limits_and_optional_outputs():
    rng = np.random.default_rng(6)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    bank = B.MemoryBank(64, "bf16", 5000, max_B=128, max_k1=512)
    bank.append(dev(_unit(rng, 5000, 64)))
    q = dev(_unit(rng, 65, 64))
    for nq, k1 in ((65, 16), (8, 257)):                       # beyond the built-in array's limits
        with pytest.raises(B.MemError) as e:
            bank.retrieve_static(q[:nq], 0, k1, 4, 0.5, _outs(nq, k1, 4))
        assert e.value.status == B.MEM_EINVAL
    wide = B.MemoryBank(2112, "f16", 256, max_B=8, max_k1=16)  # 2112 > 2048 dimensions
    with pytest.raises(B.MemError) as e:
        wide.retrieve_static(dev(_unit(rng, 2, 2112)), 0, 4, 2, 0.5, _outs(2, 4, 2))
    assert e.value.status == B.MEM_EINVAL
    wide.close()
    # without the candidate outputs; an empty batch is a no-op
    ids, sc, _, _ = _outs(8, 16, 4)
    bank.retrieve_static(q[:8], 0, 16, 4, 0.5, (ids, sc, None, None))
    want = bank.retrieve(q[:8], 0, 16, 4, 0.5)
    _same((ids, sc), want[:2])
    bank.retrieve_static(q[:0], 0, 16, 4, 0.5, _outs(0, 16, 4))
    bank.close()
