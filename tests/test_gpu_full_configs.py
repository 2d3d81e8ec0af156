"""`-m gpu`: configs 3, 4, 5 at their full sizes (17-51 GB pinned host tables, twice: one per side).

By default (when the box has the host memory): config 3 at all three cache ratios of its sweep, config 4 across the
first rotation of its hot set (plain and in the pipelined schedule), config 5 with Zipf and with uniform ids, the
second dataset shape and one column-sharded shape of config 2; FC_FULL_CONFIGS=1 adds the other transmitter for each,
FC_SKIP_FULL=1 skips them all.  Configs 1 and 2 run at full size in test_gpu_parity.py / test_gpu_edge.py.
"""
import os
import sys
import time

import numpy as np
import pytest

from tests.parity import report_worst, run_parity, run_parity_planned
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


_workloads = {}


def workload(name, ratio=0.015):
    """Full-size workloads are expensive to build (config 4: a 100M-entry permutation and its ranking); the tests of one
    configuration share one."""
    key = (name, ratio)
    if key not in _workloads:
        if len(_workloads) >= 2:
            _workloads.clear()
        t0 = time.time()
        _workloads[key] = make_workload(name, cache_ratio=ratio)
        w = _workloads[key]
        log(f"{name} ratio {ratio}: rows {w.num_rows} dim {w.dim} cache {w.cache_rows} bags/batch {w.bags_per_batch} "
            f"built in {time.time() - t0:.0f}s")
    return _workloads[key]


# Config 4's hot set moves every 100 batches (Workload.batch(t) is a pure function of t): a run that jumps from the
# first batches to 97..104 settles on the unshifted popularity, then crosses the first rotation at batch 100, where
# nearly every distinct row of the batch misses at once.
C4_BATCHES = [0, 1, 97, 98, 99, 100, 101, 102, 103, 104]

# name, cache ratio, batches, DMA evict transmitter, host GB needed
CASES = [("c3", 0.015, 4, True, 45), ("c3", 0.005, 3, False, 45), ("c3", 0.05, 3, True, 45),
         ("c4", 0.015, C4_BATCHES, False, 130), ("c5", 0.015, 3, False, 130), ("avz", 0.015, 3, True, 15),
         ("c2d32", 0.015, 4, True, 6)]
if EXTENDED:
    CASES += [("c3", 0.005, 4, True, 45), ("c3", 0.05, 3, False, 45), ("c4", 0.015, C4_BATCHES, True, 130), ("c5", 0.015, 3, True, 130)]


@pytest.mark.parametrize("name,ratio,batches,dma,host_gb", CASES)
def test_full_size(name, ratio, batches, dma, host_gb):
    need_host_gb(host_gb)
    t0 = time.time()
    w = workload(name, ratio)
    nb = batches if isinstance(batches, int) else len(batches)
    log(f"{name} ratio {ratio} dma {dma}: {nb} batches")
    tot = run_parity(w, batches, warm=True, deep_every=nb - 1, values_every=nb - 1, fwd_exact_every=nb - 1, log=log, dma_evict=dma)
    log(f"  totals {tot} in {time.time() - t0:.0f}s")
    report_worst(log)
    assert tot["miss"] > 0
    if name == "c4":
        assert tot["miss_of"][100] > 2 * tot["miss_of"][99]    # the rotation's burst of misses was really there


@pytest.mark.parametrize("name,batches,host_gb,free", [("c2", 10, 12, False), ("c2", 24, 12, True), ("c4", C4_BATCHES, 130, True),
                                                       ("c4", [99, 100, 101], 130, False), ("c5", 3, 130, True)])
def test_full_size_pipelined_schedule(name, batches, host_gb, free):
    """The launch configuration bench.py times: DMA evict transmitter, FC_INPUTS_READY, cache_plan_next(t+1) beside batch t's forward /
    backward, rows fetched ahead of time, cache_advance; `free`: no synchronisation inside the loop, as in the timed
    region (every slot array, pooled output and the final tables are compared afterwards).  Config 4 crosses the first
    rotation of its hot set."""
    need_host_gb(host_gb)
    w = workload(name)
    log(f"{name} pipelined, free-running {free}: batches {batches}")
    run_parity_planned(w, batches, warm=True, dma_evict=True, free_running=free, log=log, inputs_ready=True,
                       ahead_miss_pct=None)      # the library's own threshold: config 4 stops running ahead once its hot set has rotated
    report_worst(log)


def test_config5_uniform_ids_overflow_then_micro_batches():
    """Config 5's adversarial run: a full batch of uniform ids touches more distinct rows than the cache holds
    (an error, state unchanged); half batches fit."""
    need_host_gb(130)
    import torch
    from oracle import Oracle, OracleError
    from paper_2208_05321_amd import FreqCache, FreqCacheError
    from tests.parity import assert_close, check_forward, compare_prepare
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
    host_o = orc.host
    for k, (b0, b1) in enumerate(((0, nb // 2), (nb // 2, nb))):
        o = (off[b0:b1 + 1] - off[b0]).copy()
        i = ids[off[b0]:off[b1]]
        g = w.grad(k, b1 - b0)
        o_d = torch.from_numpy(o).to(dev)
        so = orc.prepare(i, o)
        sd = gpu.prepare(torch.from_numpy(i).to(dev), o_d)
        compare_prepare(gpu, orc, sd.cpu().numpy(), so, k, deep=True)
        log(f"  micro-batch {k}: {gpu.stats()}")
        rows_before = gpu.rows()
        out_d = gpu.embedding_bag_fwd(sd, o_d)
        check_forward(gpu, out_d, sd.cpu().numpy(), o, orc.embedding_bag_fwd(so, o), f"micro-batch {k}: pooled output",
                      rows_before, same_weights=k == 0)
        del rows_before
        gpu.embedding_bag_bwd_sgd(sd, o_d, torch.from_numpy(g).to(dev), w.lr)
        orc.embedding_bag_bwd_sgd(so, o, g, w.lr)
        assert_close(gpu.rows(), orc.cache, f"micro-batch {k}: cached rows after SGD")
    gpu.check()
    gpu.flush()
    orc.flush()
    assert_close(host, host_o, "host table after flush")
    report_worst(log)
    gpu.close()
    orc.close()
