"""`-m gpu`: seeded random mixes of the three ways to prepare a batch (cache_prepare, cache_plan_next + cache_advance,
cache_prepare_next + cache_advance), forward-only batches, flushes and checks in between, on both transmitters, with
and without dirty tracking, against the oracle driven in program order.  Nothing here is special-cased: the point is
that any legal order of calls leaves the same state as the oracle."""
import numpy as np
import pytest

from tests.parity import assert_close, compare_prepare
from tests.tiny_workload import TinyWorkload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed,dma,dirty,staging_rows", [(0, True, False, 0), (1, False, False, 0), (2, True, True, 0), (3, False, True, 0),
                                                         (4, True, False, 40), (5, True, True, 40), (6, True, False, 0), (7, True, True, 0)])
def test_random_call_sequences(seed, dma, dirty, staging_rows):
    import torch
    from oracle import Oracle, OracleError
    from paper_2208_05321_amd import FreqCache, FreqCacheError

    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(1000 + seed)
    w = TinyWorkload(num_rows=6000, dim=20, cache_rows=260, seed=50 + seed, multi_hot=bool(seed % 2), distinct_cap=200, bags=96)
    gpu = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, host_weight=None, warm=False, dma_evict=dma,
                    dirty_tracking=dirty, staging_rows=staging_rows)
    host = gpu.host_weight()
    w.host_table(out=host)
    warm = bool(rng.integers(0, 2))
    if warm:
        gpu.warm()
    orc = Oracle(w.freq_rank, host.copy(), w.cache_rows, warm=warm, dirty_tracking=dirty)
    keep = []                                             # device inputs stay alive and untouched until the end

    def batch(t):
        ids, off = w.batch(t)
        grad = w.grad(t, len(off) - 1)
        d = (torch.from_numpy(ids).to(dev), torch.from_numpy(off).to(dev), torch.from_numpy(grad).to(dev))
        keep.append(d)
        torch.cuda.synchronize()
        return ids, off, grad, d

    def train(cur, so, sd, t, backward):
        ids, off, grad, (ids_d, off_d, grad_d) = cur
        if len(ids) == 0:
            return
        out_d = gpu.embedding_bag_fwd(sd, off_d)
        assert_close(out_d.cpu().numpy(), orc.embedding_bag_fwd(so, off), f"step {t}: pooled output")
        if backward:
            gpu.embedding_bag_bwd_sgd(sd, off_d, grad_d, w.lr)
            orc.embedding_bag_bwd_sgd(so, off, grad, w.lr)

    cur = batch(0)
    so = orc.prepare(cur[0], cur[1])
    sd = gpu.prepare(cur[3][0], cur[3][1])
    compare_prepare(gpu, orc, sd.cpu().numpy(), so, 0)
    counts = {"plain": 0, "planned": 0, "lookahead": 0, "refused": 0}
    for t in range(1, 41):
        nxt = batch(t)
        mode = ("plain", "planned", "lookahead")[int(rng.integers(0, 3))]
        backward = rng.random() < 0.75
        if mode == "plain":
            train(cur, so, sd, t, backward)
            r = rng.random()
            if r < 0.15:
                gpu.flush(); orc.flush()
                assert_close(host, orc.host, f"step {t}: host table after flush")
            elif r < 0.3:
                gpu.check()
            so_n = orc.prepare(nxt[0], nxt[1])
            sd_n = gpu.prepare(nxt[3][0], nxt[3][1])
            stats = gpu.stats()
        elif mode == "planned":
            ids, off, grad, (ids_d, off_d, grad_d) = cur
            first = rng.random() < 0.5                      # cache_plan_next before or after the current batch's work
            if first:
                sd_n = gpu.plan_next(nxt[3][0], nxt[3][1])
            train(cur, so, sd, t, backward)
            if not first:
                sd_n = gpu.plan_next(nxt[3][0], nxt[3][1])
            gpu.advance()
            stats = gpu.stats()
            so_n = orc.prepare(nxt[0], nxt[1])
        else:
            refused = False
            try:
                so_n = orc.prepare(nxt[0], nxt[1], lookahead=True)
            except OracleError as e:
                assert e.name == "BATCH_EXCEEDS_CACHE"
                refused = True
            try:
                sd_n = gpu.prepare_next(nxt[3][0], nxt[3][1])
                stats = gpu.stats()
                assert not refused
            except FreqCacheError as e:
                assert e.name == "BATCH_EXCEEDS_CACHE" and refused
            if not refused:
                ostats = orc.stats()
            train(cur, so, sd, t, backward)
            gpu.advance()
            if refused:
                counts["refused"] += 1
                so_n = orc.prepare(nxt[0], nxt[1])
                sd_n = gpu.prepare(nxt[3][0], nxt[3][1])
                stats = gpu.stats()
            else:
                assert stats == ostats, f"step {t} (lookahead): stats {stats} vs {ostats}"
        counts[mode] += 1
        if mode != "lookahead" or refused:
            assert stats == orc.stats(), f"step {t} ({mode}): stats {stats} vs {orc.stats()}"
        assert np.array_equal(sd_n.cpu().numpy(), so_n), f"step {t} ({mode}): slots"
        if t % 5 == 0:
            sr, rs = gpu.state()
            assert np.array_equal(sr, orc.slot_rank) and np.array_equal(rs, orc.rank_slot), f"step {t}: maps"
            assert_close(gpu.rows(), orc.cache, f"step {t}: cached rows")
        cur, so, sd = nxt, so_n, sd_n
    assert min(counts["plain"], counts["planned"], counts["lookahead"]) > 0
    gpu.check()
    gpu.flush(); orc.flush()
    assert_close(host, orc.host, "host table at the end")
    gpu.close()
    orc.close()
