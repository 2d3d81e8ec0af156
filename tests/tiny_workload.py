"""Small random workloads with the same interface as workloads.Workload, for edge-case parity tests."""
import numpy as np

from workloads import table_values


class TinyWorkload:
    def __init__(self, num_rows, dim, cache_rows, seed=0, multi_hot=True, max_bag=5, bags=64, hot=None, lr=0.1,
                 distinct_cap=None, allow_empty=True):
        self.name = "tiny"
        self.num_rows, self.dim, self.cache_rows = num_rows, dim, cache_rows
        self.seed, self.multi_hot, self.max_bag, self.bags, self.lr = seed, multi_hot, max_bag, bags, lr
        self.hot = hot                       # None or list of ids that take most lookups
        self.distinct_cap = distinct_cap if distinct_cap is not None else cache_rows
        self.allow_empty = allow_empty
        rng = np.random.default_rng(seed)
        self.freq_rank = rng.permutation(num_rows).astype(np.int32)
        self.inv_rank = np.argsort(self.freq_rank).astype(np.int32)
        self.grad_pool = 3

    def host_table(self, out=None):
        vals = table_values(self.seed, self.inv_rank, self.dim)
        if out is None:
            return vals.copy()
        out[:] = vals
        return out

    def batch(self, t):
        rng = np.random.default_rng([self.seed, t, 1])
        if self.multi_hot:
            lo = 0 if self.allow_empty else 1
            sizes = rng.integers(lo, self.max_bag + 1, size=self.bags)
        else:
            sizes = np.ones(self.bags, dtype=np.int64)
        n = int(sizes.sum())
        offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        pool = rng.permutation(self.num_rows)[: max(1, min(self.distinct_cap, self.num_rows))]
        ids = pool[rng.integers(0, len(pool), size=n)]
        if self.hot is not None and n:
            mask = rng.random(n) < 0.7
            ids = np.where(mask, np.asarray(self.hot)[rng.integers(0, len(self.hot), size=n)], ids)
            # keep the number of distinct rows within the cap
            uniq = np.unique(ids)
            if len(uniq) > self.distinct_cap:
                keep = set(uniq[: self.distinct_cap].tolist())
                ids = np.array([i if i in keep else uniq[0] for i in ids])
        return ids.astype(np.int64), offsets

    def grad(self, t, num_bags):
        rng = np.random.default_rng([self.seed, t % self.grad_pool, 2])
        return rng.standard_normal((num_bags, self.dim)).astype(np.float32)
