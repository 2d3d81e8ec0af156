"""`-m gpu`: the HIP library against the CPU oracle, through the C ABI, on the same seeded inputs."""
import sys

import numpy as np
import pytest

from tests.parity import run_parity, run_parity_lookahead, run_parity_planned, assert_close
from workloads import make_workload, table_values

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2208_05321_amd import load_library
    load_library()          # fail loudly if the HIP library is not built
    return torch


@pytest.mark.parametrize("warm", [True, False])
def test_config1_full(torch_cuda, warm):
    log(f"config 1, warm={warm}")
    w = make_workload("c1")
    tot = run_parity(w, w.num_batches, warm=warm, exact_values=True)    # all-ones gradients: every sum is exact
    assert 0.5 < tot["hit_ids"] / tot["ids"] < 0.95


@pytest.mark.parametrize("name,scale,ratio,batches", [
    ("c2", 0.1, 0.015, 12), ("c3", 0.03, 0.03, 8), ("c4", 0.01, 0.03, 8), ("c5", 0.05, 0.015, 6),
    ("avz", 0.1, 0.03, 6), ("c2d64", 0.1, 0.015, 5), ("c2d32", 0.1, 0.015, 5), ("c2d16", 0.1, 0.015, 5),
])
def test_scaled_configs(torch_cuda, name, scale, ratio, batches):
    log(f"{name} at scale {scale}")
    w = make_workload(name, scale=scale, cache_ratio=ratio)
    tot = run_parity(w, batches, warm=True, deep_every=3, values_every=3, log=log)
    assert tot["miss"] > 0 and tot["evict"] > 0


def test_cold_start_scaled_c2(torch_cuda):
    w = make_workload("c2", scale=0.05, cache_ratio=0.05)
    tot = run_parity(w, 8, warm=False, deep_every=2, values_every=2, log=log)
    assert tot["evict"] > 0


@pytest.mark.parametrize("staging_rows", [1, 7, 100000])
def test_results_independent_of_staging_buffer(torch_cuda, staging_rows):
    """The transmitter's buffer bound changes the number of rounds, never the result (Section 4.3)."""
    w = make_workload("c2", scale=0.004, cache_ratio=0.05)
    run_parity(w, 6, warm=True, staging_rows=staging_rows)


@pytest.mark.parametrize("staging_rows", [0, 5])
def test_staged_block_transmitter(torch_cuda, staging_rows):
    """The paper's gather -> bulk copy -> scatter transmitter gives the same results as the direct one."""
    w = make_workload("c2", scale=0.02, cache_ratio=0.04)
    run_parity(w, 6, warm=True, staged=True, staging_rows=staging_rows)
    run_parity(w, 4, warm=False, staged=True, staging_rows=staging_rows)


@pytest.mark.parametrize("staging_rows", [0, 3000, 7])
def test_dma_evict_transmitter(torch_cuda, staging_rows):
    """Evicted blocks leave by DMA and are scattered by host threads; rows whose newest copy is still in transit are
    served from the device-side block.  staging_rows 3000: some batches fit one block, some fall back to the
    kernel store; 7: every batch falls back.  Results are identical to the oracle in all cases."""
    w = make_workload("c2", scale=0.1, cache_ratio=0.015)
    tot = run_parity(w, 14, warm=True, dma_evict=True, staging_rows=staging_rows, deep_every=2, values_every=2)
    assert tot["evict"] > 0
    run_parity(w, 6, warm=False, dma_evict=True, staging_rows=staging_rows)


def test_dma_evict_rows_come_back_quickly(torch_cuda):
    """A tiny cache thrashed by alternating id sets: rows evicted in one batch are missed in the next (served from
    the in-transit block) and evicted again two batches later."""
    import torch
    from tests.tiny_workload import TinyWorkload
    from tests.parity import compare_prepare
    from tests.test_gpu_edge import make_pair
    w = TinyWorkload(num_rows=600, dim=64, cache_rows=40, seed=11, multi_hot=False)
    gpu, orc = make_pair(w, warm=True, dma_evict=True)
    dev = torch.device("cuda:0")
    sets = [np.arange(0, 30), np.arange(30, 60), np.arange(15, 45), np.arange(100, 130)]
    for t in range(40):
        ids = sets[t % len(sets) if t % 7 else 0].astype(np.int64)
        off = np.arange(len(ids) + 1, dtype=np.int64)
        g = np.random.default_rng(t).standard_normal((len(ids), w.dim)).astype(np.float32)
        so = orc.prepare(ids, off)
        sd = gpu.prepare(torch.from_numpy(ids).to(dev), torch.from_numpy(off).to(dev))
        compare_prepare(gpu, orc, sd.cpu().numpy(), so, t)
        od = gpu.embedding_bag_fwd(sd, torch.from_numpy(off).to(dev))
        assert_close(od.cpu().numpy(), orc.embedding_bag_fwd(so, off), f"fwd {t}")
        gpu.embedding_bag_bwd_sgd(sd, torch.from_numpy(off).to(dev), torch.from_numpy(g).to(dev), 0.05)
        orc.embedding_bag_bwd_sgd(so, off, g, 0.05)
    gpu.check()
    gpu.flush()
    orc.flush()
    assert_close(gpu.host_weight(), orc.host, "host table")
    gpu.close()


@pytest.mark.parametrize("name,scale,ratio,dma", [("c2", 0.1, 0.03, True), ("c2", 0.1, 0.03, False), ("c5", 0.05, 0.03, True),
                                                  ("c4", 0.01, 0.03, True)])
def test_lookahead_prepare(torch_cuda, name, scale, ratio, dma):
    """cache_prepare_next: the next batch is prepared on the library's own stream while the current one trains."""
    w = make_workload(name, scale=scale, cache_ratio=ratio)
    tot = run_parity_lookahead(w, 10, warm=True, dma_evict=dma, deep_every=2)
    assert tot["lookahead"] == 9 and tot["fallback"] == 0 and tot["evict"] > 0


def test_lookahead_refused_when_two_batches_do_not_fit(torch_cuda):
    """1.5% cache at 1/10 scale: one batch fits (12.8k distinct rows of 15k), two do not: both sides refuse the
    look-ahead and prepare the plain way after the backward pass."""
    w = make_workload("c2", scale=0.1, cache_ratio=0.015)
    tot = run_parity_lookahead(w, 6, warm=True, dma_evict=True)
    assert tot["fallback"] > 0


def test_lookahead_cold_start(torch_cuda):
    w = make_workload("c2", scale=0.05, cache_ratio=0.08)
    run_parity_lookahead(w, 8, warm=False, dma_evict=True)


@pytest.mark.parametrize("dma", [True, False])
def test_lookahead_free_running(torch_cuda, dma):
    """No synchronisation inside the loop: the look-ahead stream, the auxiliary sort stream, the side stream and
    the host scatter threads all run beside the caller's stream; everything is compared after the loop."""
    w = make_workload("c2", scale=0.2, cache_ratio=0.03)
    tot = run_parity_lookahead(w, 24, warm=True, dma_evict=dma, free_running=True)
    assert tot["lookahead"] == 23


@pytest.mark.parametrize("name,scale,ratio,dma,free", [
    ("c2", 0.1, 0.015, True, False), ("c2", 0.1, 0.015, False, False), ("c5", 0.05, 0.015, True, False),
    ("c2", 0.2, 0.015, True, True), ("c2", 0.2, 0.015, False, True), ("c4", 0.02, 0.03, True, True),
])
@pytest.mark.parametrize("ready", [False, True])
def test_planned_prepare(torch_cuda, name, scale, ratio, dma, free, ready):
    """cache_plan_next + cache_advance: index work of batch t+1 beside the forward / backward of batch t; identical
    results to plain cache_prepare (same oracle, program order).  ready: FC_INPUTS_READY, the planned batch's decisions
    do not wait for the caller's stream at all."""
    w = make_workload(name, scale=scale, cache_ratio=ratio)
    run_parity_planned(w, 16 if free else 8, warm=True, dma_evict=dma, free_running=free, inputs_ready=ready)
    run_parity_planned(w, 6, warm=True, dma_evict=dma, free_running=free, plan_first=True, inputs_ready=ready)


@pytest.mark.parametrize("name,scale,ratio,dma,free,ready", [
    ("c2", 0.1, 0.015, True, False, False), ("c2", 0.2, 0.015, True, True, True), ("c2", 0.2, 0.015, False, True, False),
    ("c5", 0.05, 0.015, True, True, True), ("c4", 0.02, 0.03, True, True, True),
])
def test_planned_prepare_dma_miss_path(torch_cuda, name, scale, ratio, dma, free, ready):
    """FC_MISS_DMA: the planned batch's missing rows are gathered by host threads and cross the link by hipMemcpyAsync
    (the block transmitter of Section 4.3 for the host -> device direction); rows in transit come from the evicted-row
    blocks at cache_advance.  Identical results, with and without the DMA evict transmitter."""
    w = make_workload(name, scale=scale, cache_ratio=ratio)
    run_parity_planned(w, 16 if free else 8, warm=True, dma_evict=dma, free_running=free, inputs_ready=ready, miss_dma=True)
    run_parity_planned(w, 6, warm=False, dma_evict=dma, free_running=free, plan_first=True, inputs_ready=ready, miss_dma=True,
                       staging_rows=0 if free else 2500)        # some batches miss more rows than a block holds: kernel path


@pytest.mark.parametrize("dma", [True, False])
def test_dma_miss_path_tiny_cache_thrashing(torch_cuda, dma):
    """Rows evicted by one batch and missed by the next: with the DMA evict transmitter they are in transit and must come
    from the evicted-row block, not from the host table the gather threads read."""
    from tests.tiny_workload import TinyWorkload
    w = TinyWorkload(num_rows=900, dim=64, cache_rows=48, seed=23, multi_hot=True, bags=24, max_bag=3, distinct_cap=40)
    for free in (False, True):
        run_parity_planned(w, 40, warm=True, dma_evict=dma, free_running=free, inputs_ready=True, miss_dma=True)
    run_parity_planned(w, 24, warm=False, dma_evict=dma, free_running=True, miss_dma=True, staging_rows=16)


@pytest.mark.parametrize("dma", [True, False])
@pytest.mark.parametrize("free", [True, False])
def test_planned_inputs_ready_tiny_cache_thrashing(torch_cuda, dma, free):
    """FC_INPUTS_READY with a cache so small that rows evicted by one batch are missed by the next or the one after:
    the planned batch is indexed (and its rows fetched) while the evictions of the batch before are still to be
    carried out on the caller's stream."""
    from tests.tiny_workload import TinyWorkload
    w = TinyWorkload(num_rows=900, dim=64, cache_rows=48, seed=21, multi_hot=True, bags=24, max_bag=3, distinct_cap=40)
    run_parity_planned(w, 40, warm=True, dma_evict=dma, free_running=free, inputs_ready=True)
    run_parity_planned(w, 24, warm=False, dma_evict=dma, free_running=free, inputs_ready=True, staging_rows=16)


@pytest.mark.parametrize("dma", [True, False])
@pytest.mark.parametrize("free", [True, False])
def test_planned_run_ahead_switches_on_and_off(torch_cuda, dma, free):
    """FC_INPUTS_READY with the threshold at the median miss share of the very batches driven: about every other batch is
    planned ahead of the caller's stream (index kernels unordered against it, the sort's later passes on the side stream),
    the others behind it, and the two modes keep alternating."""
    w = make_workload("c2", scale=0.1, cache_ratio=0.015)
    run_parity_planned(w, 24, warm=True, dma_evict=dma, free_running=free, inputs_ready=True, ahead_miss_pct="median", log=log)
    w = make_workload("c4", scale=0.02, cache_ratio=0.015)
    run_parity_planned(w, 14, warm=True, dma_evict=dma, free_running=free, inputs_ready=True, ahead_miss_pct="median")


@pytest.mark.parametrize("ready", [False, True])
def test_planned_prepare_cold_and_small_blocks(torch_cuda, ready):
    w = make_workload("c2", scale=0.05, cache_ratio=0.05)
    run_parity_planned(w, 8, warm=False, dma_evict=True, staging_rows=900, inputs_ready=ready)     # some batches exceed one block
    run_parity_planned(w, 6, warm=False, dma_evict=False, staging_rows=5, inputs_ready=ready)


def test_planned_then_plain_prepare_and_flush(torch_cuda):
    """A planned batch that is never advanced explicitly: the next plain call (or flush) moves its rows first."""
    import torch
    from tests.test_gpu_edge import make_pair
    w = make_workload("c2", scale=0.05, cache_ratio=0.03)
    gpu, orc = make_pair(w, warm=True, dma_evict=True)
    dev = torch.device("cuda:0")
    dt = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    b = [w.batch(t) for t in range(4)]
    s0 = gpu.prepare(dt(b[0][0]), dt(b[0][1])); orc.prepare(*b[0])
    s1 = gpu.plan_next(dt(b[1][0]), dt(b[1][1]))                  # planned ...
    so1 = orc.prepare(*b[1])
    s2 = gpu.prepare(dt(b[2][0]), dt(b[2][1]))                    # ... and overtaken by a plain prepare
    so2 = orc.prepare(*b[2])
    assert np.array_equal(s1.cpu().numpy(), so1) and np.array_equal(s2.cpu().numpy(), so2)
    assert_close(gpu.rows(), orc.cache, "rows after plan + plain prepare")
    gpu.plan_next(dt(b[3][0]), dt(b[3][1]))
    orc.prepare(*b[3])
    gpu.flush(); orc.flush()                                       # flush completes the planned batch first
    assert_close(gpu.host_weight(), orc.host, "host table")
    assert_close(gpu.rows(), orc.cache, "rows")
    gpu.close()


# ---- FC_DIRTY_TRACK: only victims updated since they were loaded are written back (a variant beyond the paper) ----
@pytest.mark.gpu
@pytest.mark.parametrize("transmitter,staging_rows", [("direct", 0), ("direct", 9), ("dma", 0), ("dma", 700), ("staged", 0), ("staged", 5)])
@pytest.mark.parametrize("warm", [True, False])
def test_dirty_tracking(torch_cuda, transmitter, staging_rows, warm):
    """Mixed run: every third batch is forward-only, so part of the victims are clean.  Slots, lists, maps, bytes written
    (bit-exact) and all values equal the oracle's dirty-tracking variant; a flush in mid-run cleans every row."""
    w = make_workload("c2", scale=0.1, cache_ratio=0.015)
    tot = run_parity(w, 12, warm=warm, staged=transmitter == "staged", dma_evict=transmitter == "dma", staging_rows=staging_rows,
                     dirty_tracking=True, forward_only=lambda t: t % 3 == 1, flush_at=(6,))
    assert 0 < tot["bytes_d2h"] < tot["evict"] * w.dim * 4      # some victims were written, some were dropped


@pytest.mark.gpu
@pytest.mark.parametrize("dma", [True, False])
def test_dirty_tracking_forward_only_writes_nothing(torch_cuda, dma):
    w = make_workload("c3", scale=0.02, cache_ratio=0.015)
    tot = run_parity(w, 6, warm=True, dma_evict=dma, dirty_tracking=True, forward_only=lambda t: True)
    assert tot["evict"] > 0 and tot["bytes_d2h"] == 0


@pytest.mark.gpu
def test_dirty_tracking_always_trained_equals_plain_policy(torch_cuda):
    """Cold start and a backward pass after every batch: every resident row is dirty, the bytes are those of the paper's policy."""
    w = make_workload("c5", scale=0.02, cache_ratio=0.015)
    tot = run_parity(w, 6, warm=False, dma_evict=True, dirty_tracking=True)
    assert tot["bytes_d2h"] == tot["evict"] * w.dim * 4 > 0


@pytest.mark.gpu
@pytest.mark.parametrize("dma,free", [(True, False), (False, False), (True, True)])
def test_dirty_tracking_planned(torch_cuda, dma, free):
    """FC_DIRTY_TRACK with cache_plan_next / cache_advance: what is dirty is decided at cache_advance, after the current
    batch's backward pass; bytes written back, the host table and everything else equal the oracle in program order."""
    from tests.parity import run_parity_planned
    w = make_workload("c2", scale=0.1, cache_ratio=0.015)
    tot = run_parity_planned(w, 12, warm=True, dma_evict=dma, free_running=free, dirty_tracking=True,
                             forward_only=lambda t: t % 3 == 1)
    assert tot["bytes_d2h"] > 0
    run_parity_planned(w, 6, warm=False, dma_evict=dma, staging_rows=900, dirty_tracking=True, forward_only=lambda t: t % 2 == 0)


@pytest.mark.gpu
@pytest.mark.parametrize("dma", [True, False])
def test_dirty_tracking_lookahead(torch_cuda, dma):
    from tests.parity import run_parity_lookahead
    w = make_workload("c2", scale=0.1, cache_ratio=0.03)
    tot = run_parity_lookahead(w, 10, warm=True, dma_evict=dma, dirty_tracking=True, forward_only=lambda t: t % 3 == 1)
    assert tot["lookahead"] > 0 and 0 < tot["bytes_d2h"] < tot["evict"] * w.dim * 4


@pytest.mark.gpu
def test_planned_inputs_uploaded_one_step_ahead(torch_cuda):
    """The ordering contract of cache_plan_next: ids / offsets that are copied to the device on the caller's stream (no
    host synchronisation) before the previous cache_advance are seen complete by the library's streams."""
    torch = torch_cuda
    from oracle import Oracle
    from paper_2208_05321_amd import FreqCache
    w = make_workload("c2", scale=0.2, cache_ratio=0.015)
    dev = torch.device("cuda:0")
    T = 12
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        gpu = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, dma_evict=True, stream=st)
        host = gpu.host_weight()
        w.host_table(out=host)
        gpu.warm()
        orc = Oracle(w.freq_rank, host.copy(), w.cache_rows, warm=True)
        batches = [w.batch(t) for t in range(T + 2)]
        pinned = [(torch.from_numpy(i).pin_memory(), torch.from_numpy(o).pin_memory()) for i, o in batches]
        nmax = max(len(i) for i, _ in batches)
        ring = [(torch.empty(nmax, dtype=torch.int64, device=dev), torch.empty(len(batches[0][1]), dtype=torch.int64, device=dev)) for _ in range(3)]
        grads = [torch.from_numpy(w.grad(t, len(batches[t][1]) - 1)).to(dev) for t in range(T)]
        slots_buf = [torch.empty(nmax, dtype=torch.int32, device=dev) for _ in range(3)]
        dev_in = {}

        def upload(t):                                   # asynchronous, on the cache's stream
            bi, bo = ring[t % 3]
            n = len(batches[t][0])
            bi[:n].copy_(pinned[t][0], non_blocking=True)
            bo.copy_(pinned[t][1], non_blocking=True)
            dev_in[t] = (bi[:n], bo)

        torch.cuda.synchronize()
        upload(0); upload(1)
        cur = gpu.prepare(dev_in[0][0], dev_in[0][1], out=slots_buf[0][: len(batches[0][0])])
        got = [cur.clone()]
        for t in range(T):
            upload(t + 2)                                # before this step's advance(): ready for the next step's plan_next
            out = gpu.embedding_bag_fwd(cur, dev_in[t][1])
            gpu.embedding_bag_bwd_sgd(cur, dev_in[t][1], grads[t], w.lr)
            nxt = gpu.plan_next(dev_in[t + 1][0], dev_in[t + 1][1], out=slots_buf[(t + 1) % 3][: len(batches[t + 1][0])])
            gpu.advance()
            got.append(nxt.clone())                      # on the cache's stream, after advance
            cur = nxt
        torch.cuda.synchronize()
        for t in range(T + 1):
            so = orc.prepare(*batches[t])
            assert np.array_equal(got[t].cpu().numpy(), so), f"batch {t}: slots"
            if t < T:
                orc.embedding_bag_fwd(so, batches[t][1])
                orc.embedding_bag_bwd_sgd(so, batches[t][1], w.grad(t, len(batches[t][1]) - 1), w.lr)
        gpu.flush(); orc.flush()
        assert_close(host, orc.host, "host table")
        gpu.close()
