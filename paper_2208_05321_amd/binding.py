"""ctypes binding of libfreqcache.so: same calls and names as include/freqcache.h, marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfreqcache.so")
_lib = None

FC_WARM = 1
FC_TRANSMIT_STAGED = 2
FC_EVICT_DMA = 4
FC_NO_PRESORT = 8
FC_DIRTY_TRACK = 16
FC_INPUTS_READY = 32
FC_MISS_DMA = 64

ERR_NAMES = {
    0: "OK", -1: "INVALID_ARG", -2: "ID_OUT_OF_RANGE", -3: "BAD_OFFSETS", -4: "BATCH_EXCEEDS_CACHE",
    -5: "NOT_PERMUTATION", -6: "OOM_DEVICE", -7: "OOM_PINNED", -8: "HIP", -9: "NOT_PINNED", -10: "BAD_SLOT",
    -11: "SCRATCH_EXCEEDED", -12: "COUNT_OVERFLOW",
}
NOALLOC_MAX_IDS = 524288
STAT_FIELDS = ("n_ids", "n_unique", "n_hit_unique", "n_hit_ids", "n_miss", "n_evict", "bytes_h2d", "bytes_d2h")

# every symbol include/freqcache.h declares
EXPORTS = (
    "cache_create", "cache_reserve", "cache_warm", "cache_prepare", "cache_prepare_next", "cache_plan_next", "cache_advance", "embedding_bag_fwd", "embedding_bag_bwd_sgd", "embedding_bag_bwd_sgd_noalloc", "cache_flush",
    "cache_check", "cache_destroy", "cache_last_stats", "cache_copy_state", "cache_last_lists", "cache_copy_rows",
    "cache_host_weight", "cache_strerror", "cache_profile_enable", "cache_profile_count", "cache_profile_name",
    "cache_profile_get", "freq_create", "freq_add", "freq_build", "freq_destroy", "table_reorder",
)


class FreqCacheError(RuntimeError):
    def __init__(self, code: int, what: str = ""):
        self.code = code
        self.name = ERR_NAMES.get(code, str(code))
        super().__init__(f"freqcache: {self.name} ({what})" if what else f"freqcache: {self.name}")


class _Stats(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int64) for f in STAT_FIELDS]


def load_library(path: str | None = None):
    """Load the built library; building is a separate step (paper_2208_05321_amd.build)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    # torch first: one process must not end up with two HIP runtimes (torch ships its own; whichever is loaded first
    # serves both, and the streams and device memory handed across the C ABI are torch's)
    import torch  # noqa: F401
    if not os.path.exists(p):
        raise FileNotFoundError(f"{p} is not built: run `python -m paper_2208_05321_amd.build` first")
    L = ctypes.CDLL(p)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    L.cache_create.argtypes = [i64, i32, i64, vp, vp, i64, i32, vp, ctypes.POINTER(vp)]
    L.cache_reserve.argtypes = [vp, i64, i32]
    L.cache_warm.argtypes = [vp]
    L.cache_prepare.argtypes = [vp, vp, i64, vp, i64, vp]
    L.cache_prepare_next.argtypes = [vp, vp, i64, vp, i64, vp]
    L.cache_plan_next.argtypes = [vp, vp, i64, vp, i64, vp]
    L.cache_advance.argtypes = [vp]
    L.embedding_bag_fwd.argtypes = [vp, vp, i64, vp, i64, vp]
    L.embedding_bag_bwd_sgd.argtypes = [vp, vp, i64, vp, i64, vp, ctypes.c_float]
    L.embedding_bag_bwd_sgd_noalloc.argtypes = [vp, vp, i64, vp, i64, vp, ctypes.c_float]
    L.cache_flush.argtypes = [vp]
    L.cache_check.argtypes = [vp]
    L.cache_destroy.argtypes = [vp]
    L.cache_last_stats.argtypes = [vp, ctypes.POINTER(_Stats)]
    L.cache_copy_state.argtypes = [vp, vp, vp]
    L.cache_last_lists.argtypes = [vp, vp, vp, vp, vp]
    L.cache_copy_rows.argtypes = [vp, vp]
    L.cache_host_weight.argtypes = [vp]
    L.cache_host_weight.restype = vp
    L.cache_strerror.argtypes = [ctypes.c_int]
    L.cache_strerror.restype = ctypes.c_char_p
    L.cache_profile_enable.argtypes = [vp, i32]
    L.cache_profile_count.argtypes = []
    L.cache_profile_name.argtypes = [i32]
    L.cache_profile_name.restype = ctypes.c_char_p
    L.cache_profile_get.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    L.freq_create.argtypes = [i64, vp, ctypes.POINTER(vp)]
    L.freq_add.argtypes = [vp, vp, i64]
    L.freq_build.argtypes = [vp, vp, vp, vp]
    L.freq_destroy.argtypes = [vp]
    L.table_reorder.argtypes = [vp, vp, vp, i64, i32, vp]
    for name in EXPORTS:
        if name not in ("cache_host_weight", "cache_strerror", "cache_profile_name"):
            getattr(L, name).restype = ctypes.c_int
    if path is None:
        _lib = L
    return L


def _ptr(t):
    """Device / host address of a torch tensor or numpy array (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


class FreqCache:
    """One embedding table behind the software cache.  Thin wrapper: each method is one C-ABI call."""

    def __init__(self, num_rows: int, dim: int, cache_rows: int, freq_rank: np.ndarray, host_weight=None,
                 staging_rows: int = 0, warm: bool = False, staged: bool = False, stream=None,
                 dma_evict: bool = False, presort: bool = True, dirty_tracking: bool = False,
                 inputs_ready: bool = False, miss_dma: bool = False):
        import torch

        if not torch.cuda.is_available():
            raise FreqCacheError(-8, "no GPU visible; this library has no CPU path")
        self._L = load_library()
        self._torch = torch
        self.num_rows, self.dim, self.cache_rows = int(num_rows), int(dim), int(cache_rows)
        fr = np.ascontiguousarray(freq_rank, dtype=np.int32)
        if fr.shape != (self.num_rows,):
            raise FreqCacheError(-1, "freq_rank must have num_rows entries")
        self._host_keepalive = host_weight
        if host_weight is not None:
            assert host_weight.dtype == torch.float32 and host_weight.is_contiguous()
            assert host_weight.numel() == self.num_rows * self.dim
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        flags = (FC_WARM if warm else 0) | (FC_TRANSMIT_STAGED if staged else 0) | (FC_EVICT_DMA if dma_evict else 0) | (0 if presort else FC_NO_PRESORT) | (FC_DIRTY_TRACK if dirty_tracking else 0) | (FC_INPUTS_READY if inputs_ready else 0) | (FC_MISS_DMA if miss_dma else 0)
        h = ctypes.c_void_p()
        rc = self._L.cache_create(self.num_rows, self.dim, self.cache_rows, fr.ctypes.data, _ptr(host_weight),
                                  int(staging_rows), flags, ctypes.c_void_p(self.stream.cuda_stream), ctypes.byref(h))
        self._h = h if rc == 0 else None
        self._check(rc, "cache_create")

    def _check(self, rc: int, what: str):
        if rc != 0:
            raise FreqCacheError(rc, what)

    def close(self):
        if getattr(self, "_h", None):
            self._L.cache_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the five calls of the hot path ----
    def host_weight(self) -> np.ndarray:
        """The pinned, frequency-ordered host table as a numpy view [num_rows, dim]."""
        p = self._L.cache_host_weight(self._h)
        buf = (ctypes.c_float * (self.num_rows * self.dim)).from_address(p)
        return np.frombuffer(buf, dtype=np.float32).reshape(self.num_rows, self.dim)

    def reserve(self, max_ids: int, pipelined: bool = False):
        self._check(self._L.cache_reserve(self._h, int(max_ids), int(bool(pipelined))), "cache_reserve")

    def warm(self):
        self._check(self._L.cache_warm(self._h), "cache_warm")

    def prepare(self, ids, offsets, out=None):
        """cache_prepare: ids int64[n] and offsets int64[num_bags+1] on the GPU -> slots int32[n]."""
        torch = self._torch
        n = ids.numel()
        assert ids.dtype == torch.int64 and offsets.dtype == torch.int64 and ids.is_cuda and offsets.is_cuda
        slots = out if out is not None else torch.empty(n, dtype=torch.int32, device=ids.device)
        rc = self._L.cache_prepare(self._h, _ptr(ids), n, _ptr(offsets), offsets.numel() - 1, _ptr(slots))
        self._check(rc, "cache_prepare")
        return slots

    def prepare_next(self, ids, offsets, out=None):
        """cache_prepare_next: look-ahead prepare of the next batch (protects the current batch's rows too)."""
        torch = self._torch
        n = ids.numel()
        assert ids.dtype == torch.int64 and offsets.dtype == torch.int64 and ids.is_cuda and offsets.is_cuda
        slots = out if out is not None else torch.empty(n, dtype=torch.int32, device=ids.device)
        rc = self._L.cache_prepare_next(self._h, _ptr(ids), n, _ptr(offsets), offsets.numel() - 1, _ptr(slots))
        self._check(rc, "cache_prepare_next")
        return slots

    def plan_next(self, ids, offsets, out=None):
        """cache_plan_next: index half of cache_prepare for the next batch, ahead of time; rows move at advance().
        ids / offsets must be complete, or enqueued on the cache's stream before the previous advance() / prepare():
        the library's streams do not wait for work enqueued after that call (see include/freqcache.h)."""
        torch = self._torch
        n = ids.numel()
        assert ids.dtype == torch.int64 and offsets.dtype == torch.int64 and ids.is_cuda and offsets.is_cuda
        slots = out if out is not None else torch.empty(n, dtype=torch.int32, device=ids.device)
        rc = self._L.cache_plan_next(self._h, _ptr(ids), n, _ptr(offsets), offsets.numel() - 1, _ptr(slots))
        self._check(rc, "cache_plan_next")
        return slots

    def advance(self):
        self._check(self._L.cache_advance(self._h), "cache_advance")

    def embedding_bag_fwd(self, slots, offsets, out=None):
        torch = self._torch
        nb = offsets.numel() - 1
        if out is None:
            out = torch.empty((nb, self.dim), dtype=torch.float32, device=offsets.device)
        rc = self._L.embedding_bag_fwd(self._h, _ptr(slots), slots.numel(), _ptr(offsets), nb, _ptr(out))
        self._check(rc, "embedding_bag_fwd")
        return out

    def embedding_bag_bwd_sgd(self, slots, offsets, grad_out, lr: float):
        nb = offsets.numel() - 1
        assert grad_out.dtype == self._torch.float32 and grad_out.is_contiguous() and grad_out.numel() == nb * self.dim
        rc = self._L.embedding_bag_bwd_sgd(self._h, _ptr(slots), slots.numel(), _ptr(offsets), nb, _ptr(grad_out),
                                           float(lr))
        self._check(rc, "embedding_bag_bwd_sgd")

    def embedding_bag_bwd_sgd_noalloc(self, slots, offsets, grad_out, lr: float):
        nb = offsets.numel() - 1
        assert grad_out.dtype == self._torch.float32 and grad_out.is_contiguous() and grad_out.numel() == nb * self.dim
        rc = self._L.embedding_bag_bwd_sgd_noalloc(self._h, _ptr(slots), slots.numel(), _ptr(offsets), nb, _ptr(grad_out),
                                                   float(lr))
        self._check(rc, "embedding_bag_bwd_sgd_noalloc")

    def flush(self):
        self._check(self._L.cache_flush(self._h), "cache_flush")

    def check(self):
        self._check(self._L.cache_check(self._h), "cache_check")

    # ---- introspection ----
    def stats(self) -> dict:
        s = _Stats()
        self._check(self._L.cache_last_stats(self._h, ctypes.byref(s)), "cache_last_stats")
        return {f: int(getattr(s, f)) for f in STAT_FIELDS}

    def state(self, with_rank_slot: bool = True):
        sr = np.empty(self.cache_rows, dtype=np.int32)
        rs = np.empty(self.num_rows, dtype=np.int32) if with_rank_slot else None
        self._check(self._L.cache_copy_state(self._h, sr.ctypes.data, _ptr(rs)), "cache_copy_state")
        return sr, rs

    def last_lists(self) -> dict:
        s = self.stats()
        m, v = s["n_miss"], s["n_evict"]
        out = {"miss_ranks": np.empty(m, np.int32), "evict_ranks": np.empty(v, np.int32),
               "evict_slots": np.empty(v, np.int32), "fill_slots": np.empty(m, np.int32)}
        rc = self._L.cache_last_lists(self._h, _ptr(out["miss_ranks"]), _ptr(out["evict_ranks"]),
                                      _ptr(out["evict_slots"]), _ptr(out["fill_slots"]))
        self._check(rc, "cache_last_lists")
        return out

    def rows(self) -> np.ndarray:
        out = np.empty((self.cache_rows, self.dim), dtype=np.float32)
        self._check(self._L.cache_copy_rows(self._h, out.ctypes.data), "cache_copy_rows")
        return out

    # ---- per-kernel timing ----
    def profile(self, on: bool):
        self._check(self._L.cache_profile_enable(self._h, int(on)), "cache_profile_enable")

    def profile_report(self) -> dict:
        rep = {}
        for k in range(self._L.cache_profile_count()):
            ms, cnt = ctypes.c_double(), ctypes.c_int64()
            self._check(self._L.cache_profile_get(self._h, k, ctypes.byref(ms), ctypes.byref(cnt)), "cache_profile_get")
            if cnt.value:
                rep[self._L.cache_profile_name(k).decode()] = {"ms": ms.value, "launches": cnt.value}
        return rep


class FreqCounter:
    """Static module on the GPU: accumulate id counts over a trace, then build freq_rank (one C-ABI call each)."""

    def __init__(self, num_rows: int, stream=None):
        import torch

        if not torch.cuda.is_available():
            raise FreqCacheError(-8, "no GPU visible; this library has no CPU path")
        self._L = load_library()
        self.num_rows = int(num_rows)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = ctypes.c_void_p()
        rc = self._L.freq_create(self.num_rows, ctypes.c_void_p(self.stream.cuda_stream), ctypes.byref(h))
        self._h = h if rc == 0 else None
        if rc:
            raise FreqCacheError(rc, "freq_create")

    def add(self, ids):
        rc = self._L.freq_add(self._h, _ptr(ids), ids.numel())
        if rc:
            raise FreqCacheError(rc, "freq_add")

    def build(self, with_counts: bool = False):
        fr = np.empty(self.num_rows, dtype=np.int32)
        inv = np.empty(self.num_rows, dtype=np.int32)
        cnt = np.empty(self.num_rows, dtype=np.int32) if with_counts else None
        rc = self._L.freq_build(self._h, fr.ctypes.data, inv.ctypes.data, _ptr(cnt))
        if rc:
            raise FreqCacheError(rc, "freq_build")
        return (fr, inv, cnt) if with_counts else (fr, inv)

    def close(self):
        if getattr(self, "_h", None):
            self._L.freq_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def table_reorder(src_pinned, dst_pinned, inv_rank: np.ndarray, stream=None):
    """dst[r] = src[inv_rank[r]] for two pinned torch tensors [N, D] (C-ABI call table_reorder)."""
    import torch

    L = load_library()
    st = stream if stream is not None else torch.cuda.current_stream()
    inv = np.ascontiguousarray(inv_rank, dtype=np.int32)
    n, d = src_pinned.shape
    rc = L.table_reorder(_ptr(src_pinned), _ptr(dst_pinned), inv.ctypes.data, n, d, ctypes.c_void_p(st.cuda_stream))
    if rc:
        raise FreqCacheError(rc, "table_reorder")
