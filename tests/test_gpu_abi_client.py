"""The C ABI called from plain C (tests/abi_client.c, built with gcc): no Python and no torch between
the caller and the library.  What the program prints is checked against the CPU oracle."""
import os
import struct
import subprocess

import numpy as np
import pytest

from paper_2603_10846_amd import binding
from tests import parity

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def _build(tmp_path):
    exe = str(tmp_path / "abi_client")
    libdir = os.path.dirname(binding.LIB_PATH)
    cmd = ["gcc", "-O1", "-std=c11", "-Wall", "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
           os.path.join(HERE, "abi_client.c"), "-o", exe, "-L", libdir, "-levomem", "-L", "/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True, capture_output=True)
    return exe


def test_c_caller_matches_oracle(orc, tmp_path):
    rng = np.random.default_rng(2603)
    N, d, B, k1, k2, stage, lam, alpha = 2500, 72, 5, 24, 6, 1, 0.5, 0.1
    rows = rng.standard_normal((N, d)).astype(np.float32)
    q = rng.standard_normal((B, d)).astype(np.float32)
    q0 = rng.uniform(-1, 1, (2, N)).astype(np.float32)
    rewards = rng.integers(0, 2, B * k2).astype(np.float32)
    path = tmp_path / "input.bin"
    with open(path, "wb") as f:
        f.write(struct.pack("<6i2f", N, d, B, k1, k2, stage, lam, alpha))
        for a in (rows, q, q0, rewards):
            f.write(np.ascontiguousarray(a, np.float32).tobytes())
    exe = _build(tmp_path)
    print("running the C client", flush=True)
    res = subprocess.run([exe, str(path)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    out = {}
    for line in res.stdout.splitlines():
        key, *vals = line.split()
        out.setdefault(key, []).append(vals)
    assert out["size"] == [[str(N)]] and out["done"] == [[]] and out["counters"] == [["0", "0"]]
    assert out["einval"] == [[str(binding.MEM_EINVAL)]]
    gpu = {"ids": np.array([[int(x) for x in v[1:]] for v in out["ids"]], np.int32),
           "scores": np.array([[float(x) for x in v[1:]] for v in out["scores"]], np.float32),
           "cand_ids": np.array([[int(x) for x in v[1:]] for v in out["cand"]], np.int32),
           "cand_sims": np.array([[float(x) for x in v[1:]] for v in out["csim"]], np.float32)}
    stats = parity.check_retrieve(orc, rows, q, q0[stage], k1, k2, lam, gpu)
    assert stats["queries"] == B
    # value tables: the updated stage bit-exact against the sequential fp32 recurrence, the other untouched
    want, skipped = orc.update_q32(q0[stage], gpu["ids"].reshape(-1), rewards, alpha)
    assert skipped == 0
    got = {int(v[0]): np.array([int(x, 16) for x in v[1:]], np.uint32) for v in out["q"]}
    assert np.array_equal(got[stage], want.view(np.uint32))
    assert np.array_equal(got[1 - stage], q0[1 - stage].view(np.uint32))
