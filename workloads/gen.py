"""Seeded synthetic workloads: tables, Zipf id streams, frequency ranks, gradients.

Everything here is *input generation*.  Shapes follow the paper's experimental
setup (Section 5.1, Table 1: 26 sparse features concatenated into one table,
embedding dim 128, batch 16K / 64K) and its observation that a tiny share of
rows takes most accesses (Section 3, Figure 2), which a bounded Zipf law per
feature reproduces.  The real click logs are not used anywhere.

Definitions
-----------
* table value  W0[id, c] = ((h24(seed, id, c) / 2^24) - 0.5) * 0.1   (fp32),
  h24 = top 24 bits of a splitmix-style 64-bit mix; a pure function of its
  coordinates so any row can be regenerated anywhere.
* bounded Zipf(alpha) over K items: popularity position
  k = floor(x), x drawn from the continuous density ~ x^-alpha on [1, K+1),
  by inverse CDF of a uniform variate; P(k) ~ k^(1-alpha) - (k+1)^(1-alpha).
* position k of feature f is mapped to a row id through a seeded per-feature
  permutation, so that frequency rank is not the identity map.
* frequency rank ("idx_map", Section 4.2): analytic = ids sorted by descending
  P(k) of the sampler, ties by lower id; empirical = ids sorted by descending
  count over a separate seeded warm-up trace, ties by lower id.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfc_fill.so")
_lib = None

CONFIG_NAMES = ("c1", "c2", "c3", "c4", "c5", "c5u", "avz", "c2d64", "c2d32", "c2d16")


def build_native(force: bool = False) -> str:
    """Compile fill.c (OpenMP) next to this file; returns the library path."""
    src = os.path.join(_HERE, "fill.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-ffp-contract=off", src, "-o", _LIB_PATH, "-lm"]
        )
    return _LIB_PATH


def _native():
    global _lib
    if _lib is None:
        try:
            alt = os.environ.get("FC_FILL_LIB")               # another build of fill.c (the sanitizer run of tests/)
            if not alt:
                build_native()
            lib = ctypes.CDLL(alt or _LIB_PATH)
            lib.fc_fill_table.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64]
            lib.fc_fill_table.restype = None
            lib.fc_fill_normal.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64]
            lib.fc_fill_normal.restype = None
            _lib = lib
        except Exception:  # pragma: no cover - no compiler: numpy path below
            _lib = False
    return _lib


_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_G = np.uint64(0x9E3779B97F4A7C15)
_A = np.uint64(0xD1B54A32D192ED03)
_B = np.uint64(0x8CB92BA72F3D8DD7)


def _mix64(z: np.ndarray) -> np.ndarray:
    z = z ^ (z >> np.uint64(30))
    z = z * _M1
    z = z ^ (z >> np.uint64(27))
    z = z * _M2
    z = z ^ (z >> np.uint64(31))
    return z


def table_values(seed: int, ids: np.ndarray, dim: int) -> np.ndarray:
    """W0[ids, :] as fp32 [len(ids), dim] (numpy implementation of the definition)."""
    ids = np.asarray(ids).astype(np.uint64)
    with np.errstate(over="ignore"):
        key = (np.uint64(seed + 1) * _G) + ids[:, None] * _A + np.arange(dim, dtype=np.uint64)[None, :] * _B
        bits = _mix64(key) >> np.uint64(40)
    u = bits.astype(np.float32) * np.float32(1.0 / 16777216.0)
    return (u - np.float32(0.5)) * np.float32(0.1)


def fill_host_table(out: np.ndarray, seed: int, row_ids: np.ndarray | None) -> np.ndarray:
    """out[r, :] = W0[row_ids[r], :] (identity ids when row_ids is None).

    `out` is a C-contiguous fp32 [rows, dim] array (may be a view of pinned memory).
    """
    assert out.dtype == np.float32 and out.flags.c_contiguous and out.ndim == 2
    rows, dim = out.shape
    lib = _native()
    if lib:
        rid = None
        if row_ids is not None:
            rid = np.ascontiguousarray(row_ids, dtype=np.int32)
            assert rid.shape[0] == rows
        lib.fc_fill_table(out.ctypes.data, rid.ctypes.data if rid is not None else None, rows, dim, seed)
    else:  # pragma: no cover
        step = max(1, (1 << 22) // dim)
        for a in range(0, rows, step):
            b = min(rows, a + step)
            ids = np.arange(a, b) if row_ids is None else row_ids[a:b]
            out[a:b] = table_values(seed, ids, dim)
    return out


def _normal_numpy(count: int, seed: int) -> np.ndarray:
    i = np.arange(0, count, 2, dtype=np.uint64)
    with np.errstate(over="ignore"):
        a = _mix64(np.uint64(seed + 1) * _G + i * _A)
    u1 = ((a >> np.uint64(40)).astype(np.float64) + 0.5) / 16777216.0
    u2 = (((a >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.float64) + 0.5) / 16777216.0
    rad = np.sqrt(-2.0 * np.log(u1))
    out = np.empty(2 * i.shape[0], dtype=np.float32)
    out[0::2] = rad * np.cos(2 * np.pi * u2)
    out[1::2] = rad * np.sin(2 * np.pi * u2)
    return out[:count]


def normal_values(count: int, seed: int, out: np.ndarray | None = None) -> np.ndarray:
    """`count` seeded ~N(0,1) fp32 values (inputs only; exact distribution is immaterial)."""
    lib = _native()
    if out is None:
        out = np.empty(count, dtype=np.float32)
    if lib:
        lib.fc_fill_normal(out.ctypes.data, count, seed)
    else:  # pragma: no cover
        out[:] = _normal_numpy(count, seed)
    return out


def zipf_positions(u: np.ndarray, K: np.ndarray | int, alpha: float) -> np.ndarray:
    """Map uniforms u in [0,1) to popularity positions k in [1, K] (bounded Zipf, see module doc)."""
    K = np.asarray(K, dtype=np.float64)
    e = 1.0 - alpha
    x = (((K + 1.0) ** e - 1.0) * u + 1.0) ** (1.0 / e)
    k = np.floor(x).astype(np.int64)
    return np.minimum(np.maximum(k, 1), K.astype(np.int64))


def zipf_probability(k: np.ndarray, K: int, alpha: float) -> np.ndarray:
    e = 1.0 - alpha
    k = k.astype(np.float64)
    return (k ** e - (k + 1.0) ** e) / (1.0 - (K + 1.0) ** e)


def log_uniform_cardinalities(num_features: int, total: int, lo: int, hi: int, seed: int) -> np.ndarray:
    """F integer cardinalities, log-uniform in [lo, hi], adjusted to sum exactly to `total`."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0xCA2D]))
    lo = max(1, min(lo, total // num_features))
    hi = max(lo, min(hi, total))
    c = np.exp(rng.uniform(np.log(lo), np.log(hi), size=num_features))
    fixed = np.zeros(num_features, dtype=bool)
    for _ in range(64):
        free_total = total - c[fixed].sum()
        c[~fixed] *= free_total / c[~fixed].sum()
        over = (~fixed) & (c > hi)
        under = (~fixed) & (c < lo)
        if not over.any() and not under.any():
            break
        c[over] = hi
        c[under] = lo
        fixed |= over | under
        if fixed.all():
            break
    c = np.maximum(np.floor(c).astype(np.int64), 1)
    # put the rounding residual on the largest feature(s)
    resid = int(total - c.sum())
    order = np.argsort(-c, kind="stable")
    j = 0
    while resid != 0:
        i = order[j % num_features]
        step = resid if abs(resid) < c[i] - 1 or resid > 0 else -(c[i] - 1)
        c[i] += step
        resid -= step
        j += 1
    assert c.sum() == total and (c >= 1).all()
    return c


@dataclass
class Workload:
    name: str
    num_rows: int
    dim: int
    cache_rows: int
    cards: np.ndarray            # int64 [F], sums to num_rows
    alpha: float
    samples: int                 # samples per batch; bags per batch = samples * F
    num_batches: int
    lr: float
    grad_kind: str = "normal"    # "ones" | "normal"
    multi_hot: bool = False
    bag_mean: float = 20.0
    bag_max: int = 64
    id_dist: str = "zipf"        # "zipf" | "uniform"
    drift_every: int = 0         # batches between rotations of the hot set (0 = none)
    drift_frac: float = 0.0
    rank_kind: str = "analytic"  # "analytic" | "empirical"
    warm_samples: int = 0        # warm-up trace length for empirical ranks
    seed: int = 0
    grad_pool: int = 4           # distinct gradient tensors, cycled over batches
    feat_off: np.ndarray = field(default=None, repr=False)
    perm: np.ndarray = field(default=None, repr=False)        # int32 [N]: (feature, position) -> id
    freq_rank: np.ndarray = field(default=None, repr=False)   # int32 [N]: id -> rank
    inv_rank: np.ndarray = field(default=None, repr=False)    # int32 [N]: rank -> id
    _grads: dict = field(default_factory=dict, repr=False)

    @property
    def num_features(self) -> int:
        return int(self.cards.shape[0])

    @property
    def bags_per_batch(self) -> int:
        return self.samples * self.num_features

    # ---- static structure -------------------------------------------------
    def finalize(self) -> "Workload":
        F = self.num_features
        self.feat_off = np.zeros(F + 1, dtype=np.int64)
        np.cumsum(self.cards, out=self.feat_off[1:])
        assert int(self.feat_off[-1]) == self.num_rows
        perm = np.empty(self.num_rows, dtype=np.int32)
        for f in range(F):
            rng = np.random.Generator(np.random.Philox(key=[self.seed, 0x9E00 + f]))
            a, b = int(self.feat_off[f]), int(self.feat_off[f + 1])
            perm[a:b] = rng.permutation(b - a).astype(np.int32) + np.int32(a)
        self.perm = perm
        if self.rank_kind == "analytic":
            score = np.empty(self.num_rows, dtype=np.float64)   # indexed by id
            for f in range(F):
                a, b = int(self.feat_off[f]), int(self.feat_off[f + 1])
                K = b - a
                if self.id_dist == "uniform":
                    p = np.full(K, 1.0 / K)
                else:
                    p = zipf_probability(np.arange(1, K + 1), K, self.alpha)
                score[perm[a:b]] = p / F
        else:
            counts = np.zeros(self.num_rows, dtype=np.int64)
            for ids in self.warmup_trace():
                counts += np.bincount(ids, minlength=self.num_rows)
            score = counts.astype(np.float64)
        order = np.argsort(-score, kind="stable")               # rank -> id, ties by lower id
        self.inv_rank = order.astype(np.int32)
        self.freq_rank = np.empty(self.num_rows, dtype=np.int32)
        self.freq_rank[order] = np.arange(self.num_rows, dtype=np.int32)
        return self

    def warmup_trace(self):
        """The seeded warm-up trace empirical ranks are counted on (Section 4.2: id frequencies from a scan of the data, or
        of a sample of it), in chunks of ids; a different seed than the batches of the run."""
        left, t = self.warm_samples, 0
        while left > 0:
            s = min(left, 1 << 18)
            ids, _ = self._draw(s, seed=self.seed + 7919, t=t, shift_batch=0)
            yield ids
            left -= s
            t += 1

    # ---- per-batch inputs ---------------------------------------------------
    def _draw(self, samples: int, seed: int, t: int, shift_batch: int):
        F = self.num_features
        rng = np.random.Generator(np.random.Philox(key=[seed, t]))
        if self.multi_hot:
            sizes = np.clip(rng.poisson(self.bag_mean, size=(samples, F)), 1, self.bag_max).astype(np.int64).ravel()
            feat = np.repeat(np.tile(np.arange(F), samples), sizes)
            offsets = np.zeros(sizes.shape[0] + 1, dtype=np.int64)
            np.cumsum(sizes, out=offsets[1:])
        else:
            feat = np.tile(np.arange(F), samples)
            offsets = np.arange(samples * F + 1, dtype=np.int64)
        K = self.cards[feat]
        u = rng.random(feat.shape[0])
        if self.id_dist == "uniform":
            k = np.minimum((u * K).astype(np.int64), K - 1) + 1
        else:
            k = zipf_positions(u, K, self.alpha)
        pos = k - 1
        if self.drift_every and shift_batch:
            shift = (shift_batch // self.drift_every) * np.maximum(1, np.round(self.drift_frac * self.cards).astype(np.int64))
            pos = (pos + shift[feat]) % K
        ids = self.perm[self.feat_off[feat] + pos].astype(np.int64)
        return ids, offsets

    def batch(self, t: int):
        """(ids int64[n], offsets int64[num_bags+1]) of batch t; ids already offset into the one table."""
        return self._draw(self.samples, seed=self.seed + 1, t=t, shift_batch=t)

    def grad(self, t: int, num_bags: int) -> np.ndarray:
        """Upstream gradient of the pooled output for batch t, fp32 [num_bags, dim]."""
        if self.grad_kind == "ones":
            key = ("ones", num_bags)
            if key not in self._grads:
                self._grads = {key: np.ones((num_bags, self.dim), dtype=np.float32)}
            return self._grads[key]
        key = (t % self.grad_pool, num_bags)
        if key not in self._grads:
            if len(self._grads) >= self.grad_pool:
                self._grads.clear()
            self._grads[key] = normal_values(num_bags * self.dim, self.seed * 1000 + 17 + key[0]).reshape(num_bags, self.dim)
        return self._grads[key]

    def host_table(self, out: np.ndarray | None = None) -> np.ndarray:
        """Rank-ordered initial table: row rho holds W0[id with frequency rank rho] (Section 4.2)."""
        if out is None:
            out = np.empty((self.num_rows, self.dim), dtype=np.float32)
        return fill_host_table(out, self.seed, self.inv_rank)


def make_workload(name: str, scale: float = 1.0, cache_ratio: float = 0.015, num_batches: int | None = None,
                  seed: int = 0) -> Workload:
    """The five benchmark configurations, plus "c5u" (config 5's uniform-id run), "avz" (the paper's second dataset
    shape) and "c2d64/32/16" (config 2 at the per-rank row width of a 2/4/8-way column split).

    scale < 1 shrinks rows, cardinalities and batch together for CPU-sized tests; the
    cache stays at `cache_ratio` of the rows.
    """
    def sc(x, lo=1):
        return max(lo, int(round(x * scale)))

    if name == "c1":
        N = 100_000
        w = Workload(name, N, 16, int(N * cache_ratio), np.array([N], dtype=np.int64), 1.1, 1024, 50, 0.01,
                     grad_kind="ones", seed=seed)
    elif name == "c2":
        N = sc(10_000_000, 2600)
        cards = log_uniform_cardinalities(26, N, 10, sc(2_000_000, 10), seed)
        w = Workload(name, N, 128, int(N * cache_ratio), cards, 1.05, sc(16_384, 8), 200, 0.01, seed=seed)
    elif name == "c3":
        N = sc(33_800_000, 2600)
        cards = log_uniform_cardinalities(26, N, 10, sc(10_000_000, 10), seed + 1)
        w = Workload(name, N, 128, int(N * cache_ratio), cards, 1.05, sc(16_384, 8), 500, 0.01,
                     rank_kind="empirical", warm_samples=sc(10_000_000, 1000), seed=seed)
    elif name == "c4":
        N = sc(100_000_000, 2600)
        cards = log_uniform_cardinalities(26, N, 10, sc(30_000_000, 10), seed + 2)
        w = Workload(name, N, 128, int(N * cache_ratio), cards, 1.2, sc(65_536, 8), 300, 0.01,
                     drift_every=100, drift_frac=0.01, seed=seed)
    elif name in ("c5", "c5u"):
        F = 8
        per = sc(6_250_000, 64)
        cards = np.full(F, per, dtype=np.int64)
        N = per * F
        w = Workload(name, N, 256, int(N * cache_ratio), cards, 1.05, sc(8_192, 4), 200, 0.01,
                     multi_hot=True, id_dist="uniform" if name == "c5u" else "zipf", seed=seed)
    elif name == "avz":
        # second workload shape of the paper (Table 1, Section 5.2): 13 sparse features, 9,445,823 rows, batch 64K
        N = sc(9_445_823, 1300)
        cards = log_uniform_cardinalities(13, N, 10, sc(4_000_000, 10), seed + 3)
        w = Workload(name, N, 128, int(N * cache_ratio), cards, 1.05, sc(65_536, 8), 200, 0.01, seed=seed)
    elif name in ("c2d64", "c2d32", "c2d16"):
        # config 2 as one rank of a column-wise (tensor-parallel) split over 2 / 4 / 8 GPUs sees it (Section 5.1):
        # same ids and index work, dim / P columns per row
        N = sc(10_000_000, 2600)
        cards = log_uniform_cardinalities(26, N, 10, sc(2_000_000, 10), seed)
        w = Workload(name, N, int(name[3:]), int(N * cache_ratio), cards, 1.05, sc(16_384, 8), 200, 0.01, seed=seed)
    else:
        raise ValueError(f"unknown config {name!r}")
    if num_batches is not None:
        w.num_batches = num_batches
    return w.finalize()
