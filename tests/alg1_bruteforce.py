"""Brute-force statement of the cache policy of Algorithm 1 (Section 4.3) with plain Python containers, for tiny tables.

Independent of the C oracle in structure: residency is a dict {row: slot} plus a list of slot contents, the batch's rows
are a Python set, victims come from `sorted(...)` over the residents the batch does not use, empty slots from a scan of
the list.  The policy in words: the rows the batch needs that are not resident are loaded, smallest row first, into the
lowest-numbered empty slots; if there are not enough empty slots, as many residents as are lacking are written back and
dropped first, chosen among the residents the batch (and, with a look-ahead, the previous batch) does not use, the
largest row index (least frequent) first.  Used to pin the oracle; never used by the GPU path.
"""
import numpy as np


class BruteForceCache:
    def __init__(self, idx_map, cpu_weight, cache_rows, warm):
        self.row_of_id = [int(r) for r in idx_map]
        self.cpu_weight = cpu_weight                      # [N, D], rank-ordered, updated in place
        self.cuda_weight = np.zeros((cache_rows, cpu_weight.shape[1]), dtype=cpu_weight.dtype)
        self.content = [None] * cache_rows                # slot -> row held, None = empty
        self.where = {}                                   # row -> slot, residents only
        if warm:
            for s in range(cache_rows):
                self._load(s, s)
        self.evicted = np.empty(0, dtype=np.int64)
        self.missed = np.empty(0, dtype=np.int64)
        self.targets = np.empty(0, dtype=np.int64)
        self.hit_ids = 0

    # ---- what the tests compare ----
    @property
    def cache_idx_map(self):
        return np.array([-1 if r is None else r for r in self.content], dtype=np.int64)

    def _load(self, row, slot):
        self.cuda_weight[slot] = self.cpu_weight[row]
        self.content[slot] = row
        self.where[row] = slot

    def _write_back(self, row):
        slot = self.where.pop(row)
        self.cpu_weight[row] = self.cuda_weight[slot]
        self.content[slot] = None

    def prepare_cache(self, ids, also_protect=None):
        """also_protect: rows that may not be evicted either (look-ahead: the previous batch's rows)."""
        rows = [self.row_of_id[int(i)] for i in ids]
        self.hit_ids = sum(1 for r in rows if r in self.where)
        needed = set(rows)
        lacking = sorted(needed - self.where.keys())
        keep = needed if also_protect is None else needed | {int(r) for r in also_protect}
        empties = [s for s, r in enumerate(self.content) if r is None]
        short = len(lacking) - len(empties)
        gone = []
        if short > 0:
            candidates = sorted((r for r in self.where if r not in keep), reverse=True)
            assert len(candidates) >= short, "more distinct rows than the cache can hold"
            gone = candidates[:short]
            for r in gone:
                self._write_back(r)
            empties = [s for s, r in enumerate(self.content) if r is None]
        placed = empties[: len(lacking)]
        for row, slot in zip(lacking, placed):
            self._load(row, slot)
        self.evicted = np.array(sorted(gone), dtype=np.int64)
        self.missed = np.array(lacking, dtype=np.int64)
        self.targets = np.array(placed, dtype=np.int64)
        return np.array([self.where[r] for r in rows], dtype=np.int64)
