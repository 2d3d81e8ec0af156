"""Algorithm 1 of the paper rendered with whole-array operations (unique / isin / nonzero /
index_fill / argsort / index_copy), the way the paper says its prototype runs it (Section 4.3).

Independent of the C oracle: a single slot->cpu_row_idx array, the -2 masking trick for the
protected rows and a descending stable argsort for victim selection; no inverse map.  Only for
tiny tables (every lookup is a linear search).  Used to pin the oracle; never used by the GPU path.
"""
import numpy as np


class ArrayOpsCache:
    def __init__(self, idx_map, cpu_weight, cache_rows, warm):
        self.idx_map = np.asarray(idx_map, dtype=np.int64)
        self.cpu_weight = cpu_weight                      # [N, D], rank-ordered, updated in place
        self.cuda_weight = np.zeros((cache_rows, cpu_weight.shape[1]), dtype=cpu_weight.dtype)
        self.cache_idx_map = np.full(cache_rows, -1, dtype=np.int64)
        if warm:
            self.cache_idx_map[:] = np.arange(cache_rows)
            self.cuda_weight[:] = cpu_weight[:cache_rows]
        self.evicted = np.empty(0, dtype=np.int64)
        self.missed = np.empty(0, dtype=np.int64)
        self.targets = np.empty(0, dtype=np.int64)

    def prepare_cache(self, ids, also_protect=None):
        """also_protect: extra cpu_row_idxs for the backlist (look-ahead: the previous batch's rows)."""
        rows_of_ids = self.idx_map[np.asarray(ids, dtype=np.int64)]
        cpu_row_idxs = np.unique(rows_of_ids)
        comm_cpu_row_idxs = cpu_row_idxs[np.isin(cpu_row_idxs, self.cache_idx_map, invert=True)]
        self.hit_ids = int(np.isin(rows_of_ids, self.cache_idx_map).sum())
        backlist = cpu_row_idxs if also_protect is None else np.union1d(cpu_row_idxs, also_protect)
        self._prepare_cpu_row_idx_on_gpu(comm_cpu_row_idxs, backlist)
        # one gpu_row_idx per input id
        return np.array([np.nonzero(self.cache_idx_map == r)[0][0] for r in rows_of_ids], dtype=np.int64)

    def _prepare_cpu_row_idx_on_gpu(self, cpu_row_idxs, backlist):
        m = self.cache_idx_map
        free_capacity = int((m == -1).sum())
        evict_num = cpu_row_idxs.size - free_capacity
        self.evicted = np.empty(0, dtype=np.int64)
        if evict_num > 0:
            mask = np.isin(m, backlist)
            invalid_idx = np.nonzero(mask)[0]
            backup = m[invalid_idx].copy()
            m[invalid_idx] = -2                                           # below every real row index
            evict_gpu_row_idxs = np.argsort(-m, kind="stable")[:evict_num]  # largest cpu_row_idx first
            m[invalid_idx] = backup
            target_cpu_row_idx = m[evict_gpu_row_idxs]
            assert (target_cpu_row_idx >= 0).all()
            self.cpu_weight[target_cpu_row_idx] = self.cuda_weight[evict_gpu_row_idxs]   # move_to_cpu
            m[evict_gpu_row_idxs] = -1
            self.evicted = np.sort(target_cpu_row_idx)
        target_gpu_row_idxs = np.nonzero(m == -1)[0][: cpu_row_idxs.size]
        self.cuda_weight[target_gpu_row_idxs] = self.cpu_weight[cpu_row_idxs]            # move_to_gpu
        m[target_gpu_row_idxs] = cpu_row_idxs
        self.missed = cpu_row_idxs
        self.targets = target_gpu_row_idxs
