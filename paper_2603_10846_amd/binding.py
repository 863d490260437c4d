"""ctypes binding of libevomem.so (include/evomem.h): argument marshalling only.

PyTorch is used for device memory and streams; every step of the method runs in the library's
HIP kernels.  There is no CPU fallback: importing works without a GPU (so that symbol and
argument-check tests can run), but `load()` raises if the shared library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# EVOMEM_LIB selects another build of the same library (e.g. one compiled with other flags)
LIB_PATH = os.environ.get("EVOMEM_LIB") or os.path.join(_HERE, "libevomem.so")
SRC = os.path.join(_HERE, "csrc", "evomem.hip")

MEM_OK, MEM_EINVAL, MEM_ECAPACITY, MEM_EWORKSPACE, MEM_EHIP, MEM_ESTATE = range(6)
MEM_F32, MEM_BF16, MEM_F16 = 0, 1, 2
MEM_STAGE_DRAFT, MEM_STAGE_REFINE = 0, 1
DTYPES = {"f32": MEM_F32, "bf16": MEM_BF16, "f16": MEM_F16}

SYMBOLS = {
    # name: (restype, argtypes)
    "mem_store_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int64]),
    "mem_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int64, C.c_int, C.c_int]),
    "mem_create": (C.c_int, [C.POINTER(C.c_void_p), C.c_int, C.c_int, C.c_int64, C.c_void_p, C.c_void_p,
                             C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_int]),
    "mem_append": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                             C.POINTER(C.c_int64), C.c_void_p]),
    "mem_retrieve": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float,
                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mem_retrieve_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mem_retrieve_exact": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mem_retrieve_flags": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]),
    "mem_retrieve_eps": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float, C.c_float,
                                   C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p]),
    "mem_attach_tags": (C.c_int, [C.c_void_p, C.c_void_p]),
    "mem_set_tags": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "mem_retrieve_masked": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mem_shape_rewards": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_float,
                                    C.c_float, C.c_void_p, C.c_void_p]),
    "mem_reward_stats": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "mem_reward_stats_reset": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p]),
    "mem_restore": (C.c_int, [C.c_void_p, C.c_int64]),
    "mem_update_q": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_float, C.c_void_p]),
    "mem_select_by_q": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_uint64,
                                  C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mem_size": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64)]),
    "mem_read_q": (C.c_int, [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "mem_read_rows": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "mem_counters": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
    "mem_read_probe": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_int64), C.c_void_p]),
    "mem_profile_enable": (C.c_int, [C.c_void_p, C.c_int]),
    "mem_profile_read": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_float),
                                   C.POINTER(C.c_int64)]),
    "mem_plan_levels": (C.c_int, [C.c_int64, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int), C.c_int]),
    "mem_strerror": (C.c_char_p, [C.c_int]),
    "mem_destroy": (C.c_int, [C.c_void_p]),
}

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library() -> str:
    """Compile csrc/evomem.hip for gfx950 into libevomem.so next to this file."""
    subprocess.check_call(["hipcc", *HIPCC_FLAGS, "-o", LIB_PATH, SRC])
    return LIB_PATH


_lib = None


def load():
    """Load the built library; build it first if it is missing.  Raises if neither works."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            if os.environ.get("EVOMEM_LIB"):
                raise FileNotFoundError(f"EVOMEM_LIB names {LIB_PATH}, which does not exist")
            build_library()
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(lib, name)          # AttributeError if the library does not export it
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


class MemError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {load().mem_strerror(status).decode()} (status {status})")


def _check(status: int, where: str):
    if status != MEM_OK:
        raise MemError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class MemoryBank:
    """A bank on one GPU.  Owns the torch tensors the library works in."""

    def __init__(self, d: int, dtype: str, capacity: int, max_B: int = 1024, max_k1: int = 256,
                 device: str = "cuda:0"):
        lib = load()
        if not torch.cuda.is_available():
            raise RuntimeError("evomem needs a GPU: there is no CPU path")
        self.lib, self.d, self.dtype, self.capacity = lib, d, DTYPES[dtype], capacity
        self._tags = None
        self.device = torch.device(device)
        sb = lib.mem_store_bytes(d, self.dtype, capacity)
        wb = lib.mem_workspace_bytes(d, self.dtype, capacity, max_B, max_k1)
        if sb == 0 or wb == 0:
            raise MemError(MEM_EINVAL, "mem_store_bytes/mem_workspace_bytes")
        self.store = torch.empty(sb, dtype=torch.uint8, device=self.device)
        self.invnorm = torch.empty((capacity + 255) // 256 * 256, dtype=torch.float32, device=self.device)
        self.q = torch.zeros((2, capacity), dtype=torch.float32, device=self.device)
        self.workspace = torch.empty(wb, dtype=torch.uint8, device=self.device)
        h = C.c_void_p()
        torch.cuda.synchronize(self.device)
        _check(lib.mem_create(C.byref(h), d, self.dtype, capacity, _ptr(self.store), _ptr(self.invnorm),
                              _ptr(self.q), _ptr(self.workspace), wb, max_B, max_k1,
                              self.device.index or 0), "mem_create")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            torch.cuda.synchronize(self.device)
            self.lib.mem_destroy(self.h)
            self.h = None

    __del__ = close

    def size(self) -> int:
        n = C.c_int64()
        _check(self.lib.mem_size(self.h, C.byref(n)), "mem_size")
        return n.value

    def append(self, emb: torch.Tensor, q0_draft=None, q0_refine=None) -> int:
        assert emb.is_cuda and emb.dtype == torch.float32 and emb.is_contiguous() and emb.shape[1] == self.d
        first = C.c_int64()
        _check(self.lib.mem_append(self.h, _ptr(emb), emb.shape[0], _ptr(q0_draft), _ptr(q0_refine),
                                   C.byref(first), _stream()), "mem_append")
        return first.value

    def retrieve(self, queries: torch.Tensor, stage: int, k1: int, k2: int, lam: float,
                 want_candidates: bool = False, out=None):
        assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous()
        B = queries.shape[0]
        if out is None:
            ids = torch.empty((B, k2), dtype=torch.int32, device=self.device)
            scores = torch.empty((B, k2), dtype=torch.float32, device=self.device)
            cid = torch.empty((B, k1), dtype=torch.int32, device=self.device) if want_candidates else None
            csim = torch.empty((B, k1), dtype=torch.float32, device=self.device) if want_candidates else None
        else:
            ids, scores, cid, csim = out
        _check(self.lib.mem_retrieve(self.h, _ptr(queries), B, stage, k1, k2, lam, _ptr(ids), _ptr(scores),
                                     _ptr(cid), _ptr(csim), _stream()), "mem_retrieve")
        return ids, scores, cid, csim

    def retrieve_exact(self, queries: torch.Tensor, stage: int, k1: int, k2: int, lam: float, want_candidates: bool = False):
        """mem_retrieve by exhaustive selection (every entry scored in fp64; no list can overflow)."""
        assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous()
        B = queries.shape[0]
        ids = torch.empty((B, k2), dtype=torch.int32, device=self.device)
        scores = torch.empty((B, k2), dtype=torch.float32, device=self.device)
        cid = torch.empty((B, k1), dtype=torch.int32, device=self.device) if want_candidates else None
        csim = torch.empty((B, k1), dtype=torch.float32, device=self.device) if want_candidates else None
        _check(self.lib.mem_retrieve_exact(self.h, _ptr(queries), B, stage, k1, k2, lam, _ptr(ids), _ptr(scores),
                                           _ptr(cid), _ptr(csim), _stream()), "mem_retrieve_exact")
        return ids, scores, cid, csim

    def retrieve_flags(self, B: int) -> torch.Tensor:
        """Status words (int32[B]) of the latest retrieve: bit 0 = a survivor list of that query overflowed."""
        out = torch.empty(B, dtype=torch.int32, device=self.device)
        _check(self.lib.mem_retrieve_flags(self.h, _ptr(out), B, _stream()), "mem_retrieve_flags")
        return out

    def retrieve_static(self, queries: torch.Tensor, stage: int, k1: int, k2: int, lam: float, out):
        """mem_retrieve with the library's built-in scratch array; `out` = (ids, scores, cand_ids or None,
        cand_sims or None) are the caller's tensors: nothing is allocated here or in the library."""
        ids, scores, cid, csim = out
        _check(self.lib.mem_retrieve_static(self.h, _ptr(queries), queries.shape[0], stage, k1, k2, lam, _ptr(ids),
                                            _ptr(scores), _ptr(cid), _ptr(csim), _stream()), "mem_retrieve_static")
        return out

    def retrieve_eps(self, queries: torch.Tensor, stage: int, k1: int, k2: int, lam: float, eps: float, seed: int,
                     step: int, want_candidates: bool = False):
        """Epsilon-greedy selection; returns (ids, scores, cand_ids, cand_sims, explored uint8 [B][k2])."""
        assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous()
        B = queries.shape[0]
        ids = torch.empty((B, k2), dtype=torch.int32, device=self.device)
        scores = torch.empty((B, k2), dtype=torch.float32, device=self.device)
        explored = torch.empty((B, k2), dtype=torch.uint8, device=self.device)
        cid = torch.empty((B, k1), dtype=torch.int32, device=self.device) if want_candidates else None
        csim = torch.empty((B, k1), dtype=torch.float32, device=self.device) if want_candidates else None
        _check(self.lib.mem_retrieve_eps(self.h, _ptr(queries), B, stage, k1, k2, lam, eps, seed, step, _ptr(ids),
                                         _ptr(scores), _ptr(cid), _ptr(csim), _ptr(explored), _stream()),
               "mem_retrieve_eps")
        return ids, scores, cid, csim, explored

    def update_q(self, ids: torch.Tensor, stage: int, rewards: torch.Tensor, alpha: float):
        assert ids.is_cuda and ids.dtype == torch.int32 and rewards.dtype == torch.float32
        assert ids.is_contiguous() and rewards.is_contiguous() and ids.numel() == rewards.numel()
        _check(self.lib.mem_update_q(self.h, _ptr(ids), ids.numel(), stage, _ptr(rewards), alpha, _stream()),
               "mem_update_q")

    def select_by_q(self, set_ids: torch.Tensor, set_offsets: torch.Tensor, stage: int, eps: float = 0.0,
                    seed: int = 0, step: int = 0):
        """Start point of each of G sets (ids int32 concatenated, offsets int64[G + 1]) by the stage's values,
        epsilon-greedy.  Returns (ids int32[G], values f32[G], explored u8[G])."""
        assert set_ids.is_cuda and set_ids.dtype == torch.int32 and set_ids.is_contiguous()
        assert set_offsets.is_cuda and set_offsets.dtype == torch.int64 and set_offsets.is_contiguous()
        G = set_offsets.numel() - 1
        ids = torch.empty(max(G, 0), dtype=torch.int32, device=self.device)
        vals = torch.empty(max(G, 0), dtype=torch.float32, device=self.device)
        explored = torch.empty(max(G, 0), dtype=torch.uint8, device=self.device)
        _check(self.lib.mem_select_by_q(self.h, _ptr(set_ids), set_ids.numel(), _ptr(set_offsets), G, stage, eps, seed,
                                        step, _ptr(ids), _ptr(vals), _ptr(explored), _stream()), "mem_select_by_q")
        return ids, vals, explored

    def set_tags(self, first: int, tags: torch.Tensor):
        """Tags of entries first..: an integer tensor of values < 2^32 (type = tag & 0xff, group = tag >> 8)."""
        if self._tags is None:
            self._tags = torch.empty(self.capacity, dtype=torch.int32, device=self.device)
            _check(self.lib.mem_attach_tags(self.h, _ptr(self._tags)), "mem_attach_tags")
        t = tags.to(device=self.device, dtype=torch.int64).to(torch.int32).contiguous()   # wraps to the 32-bit pattern
        _check(self.lib.mem_set_tags(self.h, first, t.numel(), _ptr(t), _stream()), "mem_set_tags")

    def retrieve_masked(self, queries: torch.Tensor, stage: int, k1: int, k2: int, lam: float, allow_types: torch.Tensor,
                        exclude_group: torch.Tensor, want_candidates: bool = False):
        assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous()
        B = queries.shape[0]
        al = allow_types.to(device=self.device, dtype=torch.int64).to(torch.int32).contiguous()
        ex = exclude_group.to(device=self.device, dtype=torch.int64).to(torch.int32).contiguous()
        assert al.numel() == B and ex.numel() == B
        ids = torch.empty((B, k2), dtype=torch.int32, device=self.device)
        scores = torch.empty((B, k2), dtype=torch.float32, device=self.device)
        cid = torch.empty((B, k1), dtype=torch.int32, device=self.device) if want_candidates else None
        csim = torch.empty((B, k1), dtype=torch.float32, device=self.device) if want_candidates else None
        _check(self.lib.mem_retrieve_masked(self.h, _ptr(queries), B, stage, k1, k2, lam, _ptr(al), _ptr(ex), _ptr(ids),
                                            _ptr(scores), _ptr(cid), _ptr(csim), _stream()), "mem_retrieve_masked")
        return ids, scores, cid, csim

    def shape_rewards(self, stage: int, feasible: torch.Tensor, latency=None, best_latency=None, normalise: bool = False,
                      sigma_min: float = 0.1, clip: float = 0.0) -> torch.Tensor:
        assert feasible.is_cuda and feasible.dtype == torch.uint8 and feasible.is_contiguous()
        for t in (latency, best_latency):
            assert t is None or (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == feasible.numel())
        out = torch.empty(feasible.numel(), dtype=torch.float32, device=self.device)
        _check(self.lib.mem_shape_rewards(self.h, stage, _ptr(feasible), _ptr(latency), _ptr(best_latency), feasible.numel(),
                                          int(normalise), sigma_min, clip, _ptr(out), _stream()), "mem_shape_rewards")
        return out

    def reward_stats(self, stage: int):
        n, mu, sd = C.c_double(), C.c_double(), C.c_double()
        _check(self.lib.mem_reward_stats(self.h, stage, C.byref(n), C.byref(mu), C.byref(sd)), "mem_reward_stats")
        return n.value, mu.value, sd.value

    def reward_stats_reset(self, stage: int):
        _check(self.lib.mem_reward_stats_reset(self.h, stage, _stream()), "mem_reward_stats_reset")

    def state(self) -> dict:
        """Everything that makes up the bank, as host tensors (for saving)."""
        out = {"d": self.d, "dtype": self.dtype, "capacity": self.capacity, "size": self.size(),
               "store": self.store.cpu(), "invnorm": self.invnorm.cpu(), "q": self.q.cpu()}
        if self._tags is not None:
            out["tags"] = self._tags.cpu()
        return out

    def load_state(self, st: dict):
        """Continue from a bank saved with state() (same d, dtype and capacity)."""
        assert (st["d"], st["dtype"], st["capacity"]) == (self.d, self.dtype, self.capacity)
        self.store.copy_(st["store"])
        self.invnorm.copy_(st["invnorm"])
        self.q.copy_(st["q"])
        if "tags" in st:
            self.set_tags(0, torch.zeros(0, dtype=torch.int64))       # attaches the tag buffer
            self._tags.copy_(st["tags"])
        torch.cuda.synchronize(self.device)
        _check(self.lib.mem_restore(self.h, st["size"]), "mem_restore")

    def read_q(self, stage: int, first: int = 0, n: int | None = None) -> torch.Tensor:
        n = self.size() - first if n is None else n
        dst = torch.empty(n, dtype=torch.float32, device=self.device)
        _check(self.lib.mem_read_q(self.h, stage, first, n, _ptr(dst), _stream()), "mem_read_q")
        return dst

    def read_rows(self, first: int, n: int) -> torch.Tensor:
        dst = torch.empty((n, self.d), dtype=torch.float32, device=self.device)
        _check(self.lib.mem_read_rows(self.h, first, n, _ptr(dst), _stream()), "mem_read_rows")
        return dst

    def counters(self):
        a, b = C.c_int64(), C.c_int64()
        _check(self.lib.mem_counters(self.h, C.byref(a), C.byref(b)), "mem_counters")
        return a.value, b.value

    def read_probe(self, checksum: torch.Tensor) -> int:
        """One read-only pass over the stored rows (XOR of all words into the int32 tensor `checksum`); returns bytes read."""
        assert checksum.is_cuda and checksum.numel() >= 1 and checksum.element_size() == 4
        n = C.c_int64()
        _check(self.lib.mem_read_probe(self.h, _ptr(checksum), C.byref(n), _stream()), "mem_read_probe")
        return n.value

    def profile_enable(self, on: bool = True):
        _check(self.lib.mem_profile_enable(self.h, int(on)), "mem_profile_enable")

    def profile_read(self, capacity: int = 4096):
        """[(milliseconds, bank rows scanned), ...] for the scan launches since the last read."""
        n, ms, rows = C.c_int(), (C.c_float * capacity)(), (C.c_int64 * capacity)()
        _check(self.lib.mem_profile_read(self.h, capacity, C.byref(n), ms, rows), "mem_profile_read")
        return [(ms[i], rows[i]) for i in range(n.value)]
