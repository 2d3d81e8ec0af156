"""`-m gpu`: configs 3, 4, 5 at their full sizes (17-51 GB pinned host tables, twice: one per side).

One case per config runs by default (15-40 s each, mostly building inputs) when the box has the host memory for
it; FC_FULL_CONFIGS=1 adds the other cache ratios / transmitters, FC_SKIP_FULL=1 skips them all.
Configs 1 and 2 run at full size in test_gpu_parity.py / test_gpu_edge.py.
"""
import os
import sys
import time

import numpy as np
import pytest

from tests.parity import run_parity, run_parity_planned
from workloads import make_workload

pytestmark = [pytest.mark.gpu, pytest.mark.slow,
              pytest.mark.skipif(os.environ.get("FC_SKIP_FULL") == "1", reason="FC_SKIP_FULL=1")]
EXTENDED = os.environ.get("FC_FULL_CONFIGS") == "1"


def need_host_gb(gb):
    avail = 0
    for line in open("/proc/meminfo"):
        if line.startswith("MemAvailable:"):
            avail = int(line.split()[1]) / 1e6
    if avail < gb:
        pytest.skip(f"needs {gb} GB of host memory, {avail:.0f} GB available")


def log(msg):
    print(msg, flush=True)


CASES = [("c3", 0.015, 4, True, 45), ("c4", 0.015, 3, False, 130), ("c5", 0.015, 3, False, 130), ("avz", 0.015, 3, True, 15)]
if EXTENDED:
    CASES += [("c3", 0.005, 4, False, 45), ("c3", 0.05, 3, False, 45), ("c4", 0.015, 3, True, 130), ("c5", 0.015, 3, True, 130)]


@pytest.mark.parametrize("name,ratio,batches,dma,host_gb", CASES)
def test_full_size(name, ratio, batches, dma, host_gb):
    need_host_gb(host_gb)
    t0 = time.time()
    w = make_workload(name, cache_ratio=ratio)
    log(f"{name} ratio {ratio} dma {dma}: rows {w.num_rows} dim {w.dim} cache {w.cache_rows} "
        f"bags/batch {w.bags_per_batch} built in {time.time() - t0:.0f}s")
    # first batches of the drifting config 4 look alike; also take batches around the first rotation of the hot set
    tot = run_parity(w, batches, warm=True, deep_every=batches - 1, values_every=batches - 1, log=log, dma_evict=dma)
    log(f"  totals {tot} in {time.time() - t0:.0f}s")
    assert tot["miss"] > 0


@pytest.mark.parametrize("name,batches,host_gb,free", [("c2", 10, 12, False), ("c2", 24, 12, True), ("c4", 4, 130, True), ("c5", 3, 130, True)])
def test_full_size_pipelined_schedule(name, batches, host_gb, free):
    """The launch configuration bench.py times: DMA evict transmitter, cache_plan_next(t+1) beside batch t's forward /
    backward, rows fetched ahead of time, cache_advance; `free`: no synchronisation inside the loop, as in the timed
    region (every slot array, pooled output and the final tables are compared afterwards)."""
    need_host_gb(host_gb)
    w = make_workload(name)
    log(f"{name} pipelined, free-running {free}: rows {w.num_rows} dim {w.dim} cache {w.cache_rows} bags/batch {w.bags_per_batch}")
    run_parity_planned(w, batches, warm=True, dma_evict=True, free_running=free)


def test_config5_uniform_ids_overflow_then_micro_batches():
    """Config 5's adversarial run: a full batch of uniform ids touches more distinct rows than the cache holds
    (an error, state unchanged); half batches fit."""
    need_host_gb(130)
    import torch
    from oracle import Oracle, OracleError
    from paper_2208_05321_amd import FreqCache, FreqCacheError
    from tests.parity import compare_prepare
    w = make_workload("c5u")
    log(f"c5u: rows {w.num_rows} cache {w.cache_rows}")
    dev = torch.device("cuda:0")
    gpu = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, host_weight=None, warm=False)
    host = gpu.host_weight()
    w.host_table(out=host)
    gpu.warm()
    orc = Oracle(w.freq_rank, host.copy(), w.cache_rows, warm=True)
    ids, off = w.batch(0)
    assert len(np.unique(ids)) > w.cache_rows
    with pytest.raises(FreqCacheError) as e:
        gpu.prepare(torch.from_numpy(ids).to(dev), torch.from_numpy(off).to(dev))
    assert e.value.name == "BATCH_EXCEEDS_CACHE"
    with pytest.raises(OracleError):
        orc.prepare(ids, off)
    nb = len(off) - 1
    for k, (b0, b1) in enumerate(((0, nb // 2), (nb // 2, nb))):
        o = off[b0:b1 + 1] - off[b0]
        i = ids[off[b0]:off[b1]]
        so = orc.prepare(i, o)
        sd = gpu.prepare(torch.from_numpy(i).to(dev), torch.from_numpy(o.copy()).to(dev))
        compare_prepare(gpu, orc, sd.cpu().numpy(), so, k, deep=True)
        log(f"  micro-batch {k}: {gpu.stats()}")
    gpu.close()
