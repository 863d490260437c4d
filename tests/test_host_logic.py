"""CPU-side tests of the C-ABI library: it loads, exports every declared symbol, sizes its buffers
sensibly, rejects bad arguments before touching the GPU, and plans scan passes that cover every
tile exactly once.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

from paper_2603_10846_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return B.load()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "evomem.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(mem_[a-z_0-9]+)\s*\(", hdr))
    assert declared, "no declarations found"
    assert declared == set(B.SYMBOLS), declared ^ set(B.SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_buffer_sizes(lib):
    assert lib.mem_store_bytes(1024, B.MEM_BF16, 1048576) == 1048576 * 1024 * 2
    assert lib.mem_store_bytes(768, B.MEM_F32, 4096) == 4096 * 768 * 4
    assert lib.mem_store_bytes(72, B.MEM_F16, 1000) == 1024 * 128 * 2          # rows to 256, dims to 64
    assert lib.mem_store_bytes(7, B.MEM_F16, 1000) == 0
    assert lib.mem_store_bytes(64, 3, 1000) == 0
    assert lib.mem_store_bytes(64, B.MEM_F16, 0) == 0
    assert lib.mem_store_bytes(64, B.MEM_F16, 2**31) == 0
    w = lib.mem_workspace_bytes(1024, B.MEM_BF16, 1048576, 256, 128)
    assert w > 256 * 8192 * 8 and w % 256 == 0
    assert lib.mem_workspace_bytes(1024, B.MEM_BF16, 1048576, 0, 128) == 0
    assert lib.mem_workspace_bytes(1024, B.MEM_BF16, 1048576, 256, 2049) == 0
    big = lib.mem_workspace_bytes(1024, B.MEM_BF16, 1048576, 256, 2048)         # room for the larger selected lists
    assert big - w == 256 * (2048 + 256 - 512) * 8
    assert lib.mem_workspace_bytes(1024, B.MEM_BF16, 1048576, 5000, 128) == 0


def test_argument_errors_without_gpu(lib):
    h = C.c_void_p()
    fake = C.c_void_p(256 * 1000)
    args = dict(d=64, dt=B.MEM_F32, cap=1000)
    wb = lib.mem_workspace_bytes(64, B.MEM_F32, 1000, 8, 16)

    def create(d=64, dt=B.MEM_F32, cap=1000, store=fake, inv=fake, q=fake, ws=fake, wbytes=wb, mb=8, mk=16, dev=0):
        return lib.mem_create(C.byref(h), d, dt, cap, store, inv, q, ws, wbytes, mb, mk, dev)
    assert lib.mem_create(None, 64, 0, 1000, fake, fake, fake, fake, wb, 8, 16, 0) == B.MEM_EINVAL
    assert create(d=12) == B.MEM_EINVAL and create(d=0) == B.MEM_EINVAL
    assert create(dt=7) == B.MEM_EINVAL and create(cap=0) == B.MEM_EINVAL
    assert create(store=None) == B.MEM_EINVAL and create(q=None) == B.MEM_EINVAL
    assert create(store=C.c_void_p(1000)) == B.MEM_EINVAL                      # misaligned
    assert create(mb=0) == B.MEM_EINVAL and create(mk=3000) == B.MEM_EINVAL and create(dev=-1) == B.MEM_EINVAL
    assert create(dev=16) == B.MEM_EINVAL                                      # device ordinals 0..15
    assert create(wbytes=wb - 1) == B.MEM_EWORKSPACE
    assert h.value is None
    # null handle everywhere
    n = C.c_int64()
    assert lib.mem_size(None, C.byref(n)) == B.MEM_EINVAL
    assert lib.mem_append(None, fake, 1, None, None, None, None) == B.MEM_EINVAL
    assert lib.mem_retrieve(None, fake, 1, 0, 4, 2, 0.5, fake, fake, None, None, None) == B.MEM_EINVAL
    assert lib.mem_update_q(None, fake, 1, 0, fake, 0.1, None) == B.MEM_EINVAL
    assert lib.mem_read_q(None, 0, 0, 1, fake, None) == B.MEM_EINVAL
    assert lib.mem_read_rows(None, 0, 1, fake, None) == B.MEM_EINVAL
    assert lib.mem_counters(None, None, None) == B.MEM_EINVAL
    assert lib.mem_profile_enable(None, 1) == B.MEM_EINVAL
    assert lib.mem_destroy(None) == B.MEM_EINVAL
    assert lib.mem_strerror(B.MEM_ECAPACITY) == b"bank capacity exceeded"
    assert lib.mem_strerror(99) == b"unknown status"


def test_null_handle_on_the_later_entry_points(lib):
    fake = C.c_void_p(256 * 1000)
    assert lib.mem_retrieve_eps(None, fake, 1, 0, 4, 2, 0.5, 0.1, 1, 2, fake, fake, None, None, None, None) == B.MEM_EINVAL
    assert lib.mem_retrieve_masked(None, fake, 1, 0, 4, 2, 0.5, fake, fake, fake, fake, None, None, None) == B.MEM_EINVAL
    assert lib.mem_select_by_q(None, fake, 4, fake, 1, 1, 0.0, 0, 0, fake, fake, None, None) == B.MEM_EINVAL
    assert lib.mem_attach_tags(None, fake) == B.MEM_EINVAL
    assert lib.mem_set_tags(None, 0, 1, fake, None) == B.MEM_EINVAL
    assert lib.mem_restore(None, 0) == B.MEM_EINVAL


def test_a_missing_library_named_by_the_environment_is_an_error():
    """EVOMEM_LIB selects another build of the library; a path that does not exist must not be
    papered over by building or loading something else."""
    import subprocess
    import sys
    code = ("import os, sys; sys.path.insert(0, %r); os.environ['EVOMEM_LIB'] = '/nonexistent/libevomem.so';\n"
            "from paper_2603_10846_amd import binding\n"
            "try:\n    binding.load()\nexcept FileNotFoundError as e:\n    print('refused')\n" % ROOT)
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    assert out.stdout.strip() == "refused", out.stderr[-500:]


@pytest.mark.parametrize("N,k1", [(1, 1), (255, 4), (4096, 32), (8192, 256), (8193, 256), (65536, 64),
                                  (1000003, 128), (1048576, 128), (4194304, 128), (8388608, 256),
                                  (3000000, 7), (2**31 - 257, 256)])
def test_scan_plan_covers_every_tile_once(lib, N, k1):
    s, r, n = (C.c_int * 16)(), (C.c_int * 16)(), (C.c_int * 16)()
    c = lib.mem_plan_levels(N, k1, s, r, n, 16)
    assert 1 <= c <= 16
    nt = (N + 255) // 256
    assert s[c - 1] == 1 and r[0] == 0
    assert n[0] * 256 <= 8192                      # the pass without a threshold fits the survivor list
    total = 0
    for i in range(c):
        U = (nt + s[i] - 1) // s[i]
        if i == 0:
            assert n[i] == U
        else:
            assert r[i] >= 2 and s[i - 1] == s[i] * r[i]
            assert n[i] == U - (U + r[i] - 1) // r[i]
            # expected survivors of a pass (k1 * density ratio) leave headroom in the list
            assert k1 * r[i] <= 8192 // 2
        total += n[i]
    assert total == nt
    if nt <= 40000:                                 # enumerate: every tile exactly once
        seen = set()
        for i in range(c):
            for j in range(n[i]):
                u = j if r[i] == 0 else (j // (r[i] - 1)) * r[i] + j % (r[i] - 1) + 1
                t = u * s[i]
                assert 0 <= t < nt and t not in seen
                seen.add(t)
        assert len(seen) == nt
    assert lib.mem_plan_levels(0, 4, s, r, n, 16) == -1 and lib.mem_plan_levels(100, 0, s, r, n, 16) == -1
