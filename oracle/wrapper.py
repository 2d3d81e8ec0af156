"""ctypes binding of the C oracle (test infrastructure; see fc_oracle.c)."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fc_oracle.c")
_LIB = os.path.join(_HERE, "libfc_oracle.so")
_lib = None

ERR_NAMES = {0: "OK", 1: "INVALID_ARG", 2: "ID_OUT_OF_RANGE", 3: "BAD_OFFSETS", 4: "BATCH_EXCEEDS_CACHE",
             5: "NOT_PERMUTATION", 6: "OOM"}


class OracleError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        self.name = ERR_NAMES.get(code, str(code))
        super().__init__(f"oracle error {self.name}")


def build(force: bool = False) -> str:
    """gcc -O2, no fp contraction, no fast-math: fp32 results follow the source order exactly."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-Wall",
                               "-shared", "-fPIC", _SRC, "-o", _LIB])
    return _LIB


def _load(path: str | None = None):
    """The oracle library (built on demand); `path` loads another build of it (used by the mutation tests)."""
    global _lib
    if _lib is None or path is not None:
        if path is None:
            path_env = os.environ.get("FC_ORACLE_LIB")      # another build of fc_oracle.c (the sanitizer run of tests/)
            if not path_env:
                build()
        else:
            path_env = None
        L = ctypes.CDLL(path or path_env or _LIB)
        vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float
        L.fco_create.argtypes = [i64, i32, i64, vp, vp, i32, ctypes.POINTER(vp)]
        L.fco_create.restype = ctypes.c_int
        L.fco_prepare.argtypes = [vp, vp, i64, vp, i64, vp]
        L.fco_prepare.restype = ctypes.c_int
        L.fco_prepare_lookahead.argtypes = [vp, vp, i64, vp, i64, vp]
        L.fco_prepare_lookahead.restype = ctypes.c_int
        L.fco_embedding_bag_fwd.argtypes = [vp, vp, i64, vp, i64, vp]
        L.fco_embedding_bag_fwd.restype = ctypes.c_int
        L.fco_bag_sum.argtypes = [vp, i64, i32, vp, i64, vp, i64, vp]
        L.fco_bag_sum.restype = ctypes.c_int
        L.fco_embedding_bag_bwd_sgd.argtypes = [vp, vp, i64, vp, i64, vp, f32]
        L.fco_embedding_bag_bwd_sgd.restype = ctypes.c_int
        L.fco_flush.argtypes = [vp]
        L.fco_flush.restype = ctypes.c_int
        L.fco_destroy.argtypes = [vp]
        L.fco_destroy.restype = None
        L.fco_stats.argtypes = [vp, vp]
        L.fco_stats.restype = None
        L.fco_set_dirty_tracking.argtypes = [vp, i32]
        L.fco_set_dirty_tracking.restype = ctypes.c_int
        for name in ("fco_slot_rank", "fco_rank_slot", "fco_cache", "fco_miss_ranks", "fco_evict_ranks",
                     "fco_evict_slots", "fco_fill_slots", "fco_dirty"):
            getattr(L, name).argtypes = [vp]
            getattr(L, name).restype = vp
        if path is not None:
            return L
        _lib = L
    return _lib


STAT_FIELDS = ("n_ids", "n_unique", "n_hit_unique", "n_hit_ids", "n_miss", "n_evict", "bytes_h2d", "bytes_d2h")


def bag_sum(weight: np.ndarray, slots: np.ndarray, offsets: np.ndarray) -> np.ndarray:
    """EmbeddingBag-sum of the rows `slots` of any fp32 weight array [rows, dim], position order, fp32
    (the arithmetic of Oracle.embedding_bag_fwd, on rows the caller supplies)."""
    L = _load()
    weight = np.ascontiguousarray(weight, dtype=np.float32)
    slots = np.ascontiguousarray(slots, dtype=np.int32)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    out = np.empty((offsets.shape[0] - 1, weight.shape[1]), dtype=np.float32)
    rc = L.fco_bag_sum(weight.ctypes.data, weight.shape[0], weight.shape[1], slots.ctypes.data, slots.shape[0],
                       offsets.ctypes.data, offsets.shape[0] - 1, out.ctypes.data)
    if rc:
        raise OracleError(rc)
    return out


class Oracle:
    """Owns the oracle's cached weight and maps; `host` (fp32 [N, D], rank-ordered) is the caller's array
    and is updated in place by evictions and flush."""

    def __init__(self, freq_rank: np.ndarray, host: np.ndarray, cache_rows: int, warm: bool = True, lib=None,
                 dirty_tracking: bool = False):
        L = lib if lib is not None else _load()
        self._L = L
        self.freq_rank = np.ascontiguousarray(freq_rank, dtype=np.int32)
        assert host.dtype == np.float32 and host.flags.c_contiguous and host.ndim == 2
        self.host = host
        self.N, self.D = host.shape
        self.C = int(cache_rows)
        h = ctypes.c_void_p()
        if self.freq_rank.shape[0] != self.N:
            raise OracleError(1)
        rc = L.fco_create(self.N, self.D, self.C, self.freq_rank.ctypes.data, host.ctypes.data, int(bool(warm)),
                          ctypes.byref(h))
        if rc:
            raise OracleError(rc)
        self._h = h
        if dirty_tracking:          # variant beyond the paper: only victims updated since they were loaded are written back
            L.fco_set_dirty_tracking(h, 1)

    def close(self):
        if getattr(self, "_h", None):
            self._L.fco_destroy(self._h)
            self._h = None

    __del__ = close

    def prepare(self, ids: np.ndarray, offsets: np.ndarray, lookahead: bool = False) -> np.ndarray:
        """Algorithm 1; lookahead=True also protects the rows of the previously prepared batch."""
        ids = np.ascontiguousarray(ids, dtype=np.int64)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        slots = np.empty(ids.shape[0], dtype=np.int32)
        fn = self._L.fco_prepare_lookahead if lookahead else self._L.fco_prepare
        rc = fn(self._h, ids.ctypes.data, ids.shape[0], offsets.ctypes.data, offsets.shape[0] - 1,
                                 slots.ctypes.data)
        if rc:
            raise OracleError(rc)
        return slots

    def embedding_bag_fwd(self, slots: np.ndarray, offsets: np.ndarray) -> np.ndarray:
        slots = np.ascontiguousarray(slots, dtype=np.int32)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        out = np.empty((offsets.shape[0] - 1, self.D), dtype=np.float32)
        rc = self._L.fco_embedding_bag_fwd(self._h, slots.ctypes.data, slots.shape[0], offsets.ctypes.data,
                                           offsets.shape[0] - 1, out.ctypes.data)
        if rc:
            raise OracleError(rc)
        return out

    def embedding_bag_bwd_sgd(self, slots: np.ndarray, offsets: np.ndarray, grad_out: np.ndarray, lr: float) -> None:
        slots = np.ascontiguousarray(slots, dtype=np.int32)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        grad_out = np.ascontiguousarray(grad_out, dtype=np.float32)
        assert grad_out.shape == (offsets.shape[0] - 1, self.D)
        rc = self._L.fco_embedding_bag_bwd_sgd(self._h, slots.ctypes.data, slots.shape[0], offsets.ctypes.data,
                                               offsets.shape[0] - 1, grad_out.ctypes.data, float(lr))
        if rc:
            raise OracleError(rc)

    def flush(self) -> None:
        rc = self._L.fco_flush(self._h)
        if rc:
            raise OracleError(rc)

    # ---- observables ----
    def stats(self) -> dict:
        a = np.zeros(8, dtype=np.int64)
        self._L.fco_stats(self._h, a.ctypes.data)
        return dict(zip(STAT_FIELDS, (int(x) for x in a)))

    def _view(self, fn, count, dtype):
        p = getattr(self._L, fn)(self._h)
        if count == 0:
            return np.empty(0, dtype=dtype)
        buf = (ctypes.c_char * (count * np.dtype(dtype).itemsize)).from_address(p)
        return np.frombuffer(buf, dtype=dtype, count=count).copy()

    @property
    def slot_rank(self):
        return self._view("fco_slot_rank", self.C, np.int32)

    @property
    def rank_slot(self):
        return self._view("fco_rank_slot", self.N, np.int32)

    @property
    def cache(self):
        return self._view("fco_cache", self.C * self.D, np.float32).reshape(self.C, self.D)

    @property
    def dirty(self):
        return self._view("fco_dirty", self.C, np.uint8)

    def last_lists(self) -> dict:
        s = self.stats()
        return {
            "miss_ranks": self._view("fco_miss_ranks", s["n_miss"], np.int32),
            "evict_ranks": self._view("fco_evict_ranks", s["n_evict"], np.int32),
            "evict_slots": self._view("fco_evict_slots", s["n_evict"], np.int32),
            "fill_slots": self._view("fco_fill_slots", s["n_miss"], np.int32),
        }
