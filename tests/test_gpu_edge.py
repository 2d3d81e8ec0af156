"""`-m gpu`: edge cases, error paths and odd shapes of the HIP library, against the oracle, through the C ABI."""
import ctypes
import sys

import numpy as np
import pytest

from tests.parity import run_parity, assert_close, compare_prepare
from tests.tiny_workload import TinyWorkload
from workloads import make_workload

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2208_05321_amd import load_library
    load_library()
    return torch


def make_pair(w, warm=True, **kw):
    from oracle import Oracle
    from paper_2208_05321_amd import FreqCache
    gpu = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, host_weight=None, warm=False, **kw)
    host = gpu.host_weight()
    w.host_table(out=host)
    if warm:
        gpu.warm()
    orc = Oracle(w.freq_rank, host.copy(), w.cache_rows, warm=warm)
    return gpu, orc


@pytest.mark.parametrize("dim", [1, 5, 6, 16, 64, 260])
@pytest.mark.parametrize("warm", [True, False])
def test_odd_dims_multi_hot_with_empty_bags(torch_cuda, dim, warm):
    """Every vector width (1, 2, 4 floats per lane), rows wider than one pass of 64 lanes, empty bags,
    ids repeated inside a bag."""
    log(f"dim {dim} warm {warm}")
    w = TinyWorkload(num_rows=3000, dim=dim, cache_rows=260, seed=dim, bags=97, max_bag=6, distinct_cap=200)
    run_parity(w, 12, warm=warm)


def test_hot_rows_long_runs(torch_cuda):
    """A few ids take most of 20k lookups: runs of one slot span hundreds of backward chunks."""
    w = TinyWorkload(num_rows=50000, dim=128, cache_rows=900, seed=3, bags=4000, max_bag=9, hot=[7, 11, 13],
                     distinct_cap=800, allow_empty=False)
    run_parity(w, 5, warm=True)


@pytest.mark.parametrize("multi_hot", [False, True])
@pytest.mark.parametrize("cache_rows", [300000, 1048581])
def test_large_cache_many_key_bits(torch_cuda, multi_hot, cache_rows):
    """Caches of more than 2^18 slots: the backward's sort then takes three or more passes without a scan kernel (the
    small caches of the other tests take the two-pass path with one).  One lookup per bag (values = positions, offsets
    not read) and multi-hot bags; several tiles, a ragged tail, hot rows whose runs cross tiles."""
    bags = 9000 if multi_hot else 23000
    w = TinyWorkload(num_rows=2 * cache_rows + 1000, dim=4, cache_rows=cache_rows, seed=41, multi_hot=multi_hot, bags=bags,
                     max_bag=5, hot=[3, 77, 4242], distinct_cap=6000, allow_empty=True)
    run_parity(w, 4, warm=False)
    run_parity(w, 3, warm=True)


@pytest.mark.parametrize("knobs", [{"FC_SORT_BITS": "4"}, {"FC_SORT_BITS": "6"}, {"FC_SORT_BITS": "9"}, {"FC_SORT_FUSED": "0"},
                                   {"FC_SORT_FUSED": "0", "FC_SORT_BITS": "5"}])
def test_sort_pass_shapes(torch_cuda, monkeypatch, knobs):
    """Every shape of the sort's passes on one cheap workload: 2 to 5 passes, digits of 4 to 11 bits, with and without the
    scan kernel (the knobs override the policy that picks among them by key width and batch size)."""
    for k, v in knobs.items():
        monkeypatch.setenv(k, v)
    w = TinyWorkload(num_rows=90000, dim=8, cache_rows=40000, seed=53, multi_hot=True, bags=5000, max_bag=6, hot=[1, 2, 3],
                     distinct_cap=3000)
    run_parity(w, 3, warm=True)
    w = TinyWorkload(num_rows=90000, dim=8, cache_rows=40000, seed=54, multi_hot=False, bags=21000, hot=[9], distinct_cap=3000)
    run_parity(w, 3, warm=False)


def test_large_cache_batches_of_very_different_sizes(torch_cuda):
    """Consecutive sorts of very different sizes on one handle (the tables of per-supertile counts alternate, and each
    sort clears what the one before it left behind): 70k lookups, then 5, then 23k, ..., trained and compared every time."""
    torch = torch_cuda
    w = TinyWorkload(num_rows=700000, dim=4, cache_rows=300000, seed=47, multi_hot=False)
    gpu, orc = make_pair(w, warm=True)
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(5)
    for t, n in enumerate([70000, 5, 23000, 2049, 70000, 1, 4096, 33000]):
        pool = rng.permutation(w.num_rows)[: min(n, 5000)]
        ids = pool[rng.integers(0, len(pool), size=n)].astype(np.int64)
        ids[: n // 10] = pool[0]                                  # one hot row: a run over several tiles
        off = np.arange(n + 1, dtype=np.int64)
        g = rng.standard_normal((n, w.dim)).astype(np.float32)
        so = orc.prepare(ids, off)
        sd = gpu.prepare(torch.from_numpy(ids).to(dev), torch.from_numpy(off).to(dev))
        compare_prepare(gpu, orc, sd.cpu().numpy(), so, t)
        od = gpu.embedding_bag_fwd(sd, torch.from_numpy(off).to(dev))
        assert_close(od.cpu().numpy(), orc.embedding_bag_fwd(so, off), f"batch {t}: pooled output")
        gpu.embedding_bag_bwd_sgd(sd, torch.from_numpy(off).to(dev), torch.from_numpy(g).to(dev), 0.05)
        orc.embedding_bag_bwd_sgd(so, off, g, 0.05)
        assert_close(gpu.rows(), orc.cache, f"batch {t} (n={n}): cached rows")
    gpu.check()
    gpu.close()


def test_large_cache_planned_schedule(torch_cuda):
    """The same sort path as started by cache_plan_next (slot write-out folded into its first kernel)."""
    from tests.parity import run_parity_planned
    w = TinyWorkload(num_rows=700000, dim=8, cache_rows=300000, seed=43, multi_hot=False, bags=30000, hot=[5, 9],
                     distinct_cap=8000)
    run_parity_planned(w, 5, warm=True, dma_evict=True, free_running=True, inputs_ready=True)


def test_single_id_batches(torch_cuda):
    """Degenerate: every lookup is the same row (one run over the whole batch), and a one-lookup batch."""
    torch = torch_cuda
    w = TinyWorkload(num_rows=500, dim=32, cache_rows=8, seed=5, multi_hot=False)
    gpu, orc = make_pair(w, warm=True)
    dev = torch.device("cuda:0")
    for n, the_id in ((1, 123), (10000, 77), (4097, 77), (33, 499)):
        ids = np.full(n, the_id, dtype=np.int64)
        off = np.arange(n + 1, dtype=np.int64)
        g = np.random.default_rng(n).standard_normal((n, w.dim)).astype(np.float32)
        so = orc.prepare(ids, off)
        sd = gpu.prepare(torch.from_numpy(ids).to(dev), torch.from_numpy(off).to(dev))
        compare_prepare(gpu, orc, sd.cpu().numpy(), so, n)
        od = gpu.embedding_bag_fwd(sd, torch.from_numpy(off).to(dev))
        assert_close(od.cpu().numpy(), orc.embedding_bag_fwd(so, off), "fwd")
        gpu.embedding_bag_bwd_sgd(sd, torch.from_numpy(off).to(dev), torch.from_numpy(g).to(dev), 0.01)
        orc.embedding_bag_bwd_sgd(so, off, g, 0.01)
        assert_close(gpu.rows(), orc.cache, f"rows after n={n}")
    gpu.check()
    gpu.close()


def test_whole_cache_needed_and_all_hits(torch_cuda):
    """|unique| == cache_rows (every other resident row is evicted), then a batch of pure hits."""
    torch = torch_cuda
    w = TinyWorkload(num_rows=4000, dim=16, cache_rows=300, seed=9, multi_hot=False)
    gpu, orc = make_pair(w, warm=True)
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(0)
    for t in range(6):
        if t % 2 == 0:
            ids = rng.permutation(w.num_rows)[: w.cache_rows].astype(np.int64)       # exactly C distinct rows
        else:
            res = np.nonzero(orc.rank_slot >= 0)[0]
            ids = w.inv_rank[res][rng.integers(0, len(res), size=500)].astype(np.int64)   # all resident
        off = np.arange(len(ids) + 1, dtype=np.int64)
        so = orc.prepare(ids, off)
        sd = gpu.prepare(torch.from_numpy(ids).to(dev), torch.from_numpy(off).to(dev))
        compare_prepare(gpu, orc, sd.cpu().numpy(), so, t)
        s = gpu.stats()
        if t % 2 == 0:
            assert s["n_unique"] == w.cache_rows
        else:
            assert s["n_miss"] == 0 and s["n_evict"] == 0 and s["n_hit_ids"] == 500
    gpu.close()


def test_error_paths_leave_state_unchanged(torch_cuda):
    torch = torch_cuda
    from paper_2208_05321_amd import FreqCacheError
    w = TinyWorkload(num_rows=2000, dim=8, cache_rows=50, seed=1, multi_hot=True, bags=20, max_bag=3, distinct_cap=40)
    gpu, orc = make_pair(w, warm=True)
    dev = torch.device("cuda:0")

    def dev_t(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    def step(t):
        ids, off = w.batch(t)
        so = orc.prepare(ids, off)
        sd = gpu.prepare(dev_t(ids), dev_t(off))
        compare_prepare(gpu, orc, sd.cpu().numpy(), so, t)
        g = w.grad(t, len(off) - 1)
        gpu.embedding_bag_bwd_sgd(sd, dev_t(off), dev_t(g), 0.1)
        orc.embedding_bag_bwd_sgd(so, off, g, 0.1)

    step(0)
    step(1)
    sr0, rs0 = gpu.state()
    rows0 = gpu.rows()
    host0 = gpu.host_weight().copy()
    stats0 = gpu.stats()

    def unchanged():
        sr, rs = gpu.state()
        return (np.array_equal(sr, sr0) and np.array_equal(rs, rs0) and np.array_equal(gpu.rows(), rows0)
                and np.array_equal(gpu.host_weight(), host0) and gpu.stats() == stats0)

    one = np.arange(4, dtype=np.int64)
    cases = [
        ("BATCH_EXCEEDS_CACHE", np.arange(51, dtype=np.int64), np.arange(52, dtype=np.int64)),
        ("ID_OUT_OF_RANGE", np.array([1, 2000, 3], dtype=np.int64), one),
        ("ID_OUT_OF_RANGE", np.array([1, -1, 3], dtype=np.int64), one),
        ("BAD_OFFSETS", np.array([1, 2, 3], dtype=np.int64), np.array([0, 2, 1, 3], dtype=np.int64)),
        ("BAD_OFFSETS", np.array([1, 2, 3], dtype=np.int64), np.array([1, 2, 3, 3], dtype=np.int64)),
        ("BAD_OFFSETS", np.array([1, 2, 3], dtype=np.int64), np.array([0, 1, 2, 2], dtype=np.int64)),
        # offsets are checked before ids (same precedence as the oracle)
        ("BAD_OFFSETS", np.array([1, 9999, 3], dtype=np.int64), np.array([0, 2, 1, 3], dtype=np.int64)),
    ]
    from oracle import OracleError
    for name, ids, off in cases:
        with pytest.raises(FreqCacheError) as e:
            gpu.prepare(dev_t(ids), dev_t(off))
        assert e.value.name == name, (name, e.value.name)
        with pytest.raises(OracleError) as eo:
            orc.prepare(ids, off)
        assert eo.value.name == name
        assert unchanged(), f"state changed by a failing call ({name})"
    # empty batch with three empty bags: fine, nothing moves
    sd = gpu.prepare(dev_t(np.empty(0, np.int64)), dev_t(np.zeros(4, np.int64)))
    assert sd.numel() == 0
    out = gpu.embedding_bag_fwd(sd, dev_t(np.zeros(4, np.int64)))
    assert out.shape == (3, 8) and float(out.abs().max()) == 0.0
    gpu.embedding_bag_bwd_sgd(sd, dev_t(np.zeros(4, np.int64)), dev_t(np.ones((3, 8), np.float32)), 0.1)
    orc.prepare(np.empty(0, np.int64), np.zeros(4, np.int64))
    sr, rs = gpu.state()
    assert np.array_equal(sr, sr0) and np.array_equal(gpu.rows(), rows0)
    # the cache still works and still agrees with the oracle afterwards
    step(2)
    step(3)
    gpu.check()
    gpu.flush()
    orc.flush()
    assert_close(gpu.host_weight(), orc.host, "host table")
    gpu.close()


def test_bad_slots_are_reported_not_followed(torch_cuda):
    torch = torch_cuda
    from paper_2208_05321_amd import FreqCacheError
    w = TinyWorkload(num_rows=500, dim=16, cache_rows=20, seed=2)
    gpu, _ = make_pair(w, warm=True)
    dev = torch.device("cuda:0")
    rows0 = gpu.rows()
    slots = torch.tensor([0, 5, 20, -3, 7], dtype=torch.int32, device=dev)
    off = torch.tensor([0, 2, 5], dtype=torch.int64, device=dev)
    out = gpu.embedding_bag_fwd(slots, off)
    with pytest.raises(FreqCacheError) as e:
        gpu.check()
    assert e.value.name == "BAD_SLOT"
    ref = np.stack([rows0[0] + rows0[5], rows0[7]])
    assert_close(out.cpu().numpy(), ref, "valid slots still pooled")
    gpu.check()                                     # the flag is cleared once reported
    g = torch.ones((2, 16), dtype=torch.float32, device=dev)
    gpu.embedding_bag_bwd_sgd(slots, off, g, 0.5)
    with pytest.raises(FreqCacheError):
        gpu.check()
    rows1 = gpu.rows()
    expect = rows0.copy()
    for s in (0, 5, 7):
        expect[s] = expect[s] - np.float32(0.5) * np.float32(1.0)
    assert_close(rows1, expect, "only valid slots updated")
    gpu.close()


def test_create_argument_errors(torch_cuda):
    torch = torch_cuda
    from paper_2208_05321_amd import FreqCache, FreqCacheError
    fr = np.arange(100, dtype=np.int32)
    for kw, name in ((dict(cache_rows=0), "INVALID_ARG"), (dict(cache_rows=101), "INVALID_ARG"),
                     (dict(dim=0), "INVALID_ARG")):
        args = dict(num_rows=100, dim=4, cache_rows=10)
        args.update(kw)
        with pytest.raises(FreqCacheError) as e:
            FreqCache(args["num_rows"], args["dim"], args["cache_rows"], fr)
        assert e.value.name == name
    bad = fr.copy()
    bad[3] = 4
    with pytest.raises(FreqCacheError) as e:
        FreqCache(100, 4, 10, bad)
    assert e.value.name == "NOT_PERMUTATION"
    # warm-up needs a table to load from
    with pytest.raises(FreqCacheError) as e:
        FreqCache(100, 4, 10, fr, host_weight=None, warm=True)
    assert e.value.name == "INVALID_ARG"
    # pageable memory is refused
    L = __import__("paper_2208_05321_amd").load_library()
    h = ctypes.c_void_p()
    pageable = np.zeros((100, 4), dtype=np.float32)
    rc = L.cache_create(100, 4, 10, fr.ctypes.data, pageable.ctypes.data, 0, 0, None, ctypes.byref(h))
    assert rc == -9
    # a pinned torch tensor is accepted and used in place
    host = torch.empty((100, 4), dtype=torch.float32, pin_memory=True)
    host.copy_(torch.arange(400, dtype=torch.float32).reshape(100, 4))
    c = FreqCache(100, 4, 10, fr, host_weight=host, warm=True)
    assert np.array_equal(c.rows(), host.numpy()[:10])
    assert c.host_weight().ctypes.data == host.data_ptr()
    c.close()


def test_backward_is_reproducible(torch_cuda):
    """No floating-point atomics: two runs over the same inputs give bit-identical cached rows."""
    torch = torch_cuda
    w = make_workload("c5", scale=0.02, cache_ratio=0.03)
    dev = torch.device("cuda:0")
    results = []
    for run in range(2):
        gpu, _ = make_pair(w, warm=True)
        for t in range(3):
            ids, off = w.batch(t)
            sd = gpu.prepare(torch.from_numpy(ids).to(dev), torch.from_numpy(off).to(dev))
            gpu.embedding_bag_bwd_sgd(sd, torch.from_numpy(off).to(dev), torch.from_numpy(w.grad(t, len(off) - 1)).to(dev), w.lr)
        results.append(gpu.rows())
        gpu.close()
    assert np.array_equal(results[0], results[1])


@pytest.mark.slow
def test_config2_full_size(torch_cuda):
    """Config 2 at its real size (10M x 128 table, 425,984 ids per batch, 150k-row cache), as bench.py runs it."""
    log("config 2, full size")
    w = make_workload("c2")
    tot = run_parity(w, 10, warm=True, deep_every=3, values_every=3, log=log)
    assert 0.85 < tot["hit_ids"] / tot["ids"] < 0.95


@pytest.mark.parametrize("dma", [True, False])
def test_planned_degenerate_batches(torch_cuda, dma):
    """cache_plan_next / cache_advance on the batches where some stage has nothing to do: an empty batch, pure hits
    (nothing fetched ahead), exactly cache_rows distinct rows (every other row evicted), a refused batch (too many
    distinct rows: nothing changes, training goes on), a single lookup."""
    torch = torch_cuda
    from paper_2208_05321_amd import FreqCacheError
    w = TinyWorkload(num_rows=3000, dim=24, cache_rows=200, seed=21, multi_hot=False)
    gpu, orc = make_pair(w, warm=True, dma_evict=dma)
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(3)

    def some(k, n):
        pool = rng.permutation(w.num_rows)[:k]
        return pool[rng.integers(0, k, size=n)].astype(np.int64)

    def resident(n):
        res = np.nonzero(orc.rank_slot >= 0)[0]
        return w.inv_rank[res][rng.integers(0, len(res), size=n)].astype(np.int64)

    kinds = ["some", "empty", "some", "hits", "whole", "too_many", "one", "some", "hits", "some"]
    ids0 = some(50, 300)
    off0 = np.arange(len(ids0) + 1, dtype=np.int64)
    so = orc.prepare(ids0, off0)
    sd = gpu.prepare(torch.from_numpy(ids0).to(dev), torch.from_numpy(off0).to(dev))
    compare_prepare(gpu, orc, sd.cpu().numpy(), so, -1)
    cur = (ids0, off0)
    keep = []                                        # device buffers stay alive while the library may read them
    for t, kind in enumerate(kinds):
        ids, off = cur
        off_d = torch.from_numpy(off).to(dev)
        g = rng.standard_normal((len(off) - 1, w.dim)).astype(np.float32)
        if len(ids):
            out_d = gpu.embedding_bag_fwd(sd, off_d)
            assert_close(out_d.cpu().numpy(), orc.embedding_bag_fwd(so, off), f"step {t}: pooled output")
            gpu.embedding_bag_bwd_sgd(sd, off_d, torch.from_numpy(g).to(dev), 0.05)
            orc.embedding_bag_bwd_sgd(so, off, g, 0.05)
        if kind == "some":
            nxt = some(120, 400)
        elif kind == "empty":
            nxt = np.empty(0, dtype=np.int64)
        elif kind == "hits":
            nxt = resident(256)
        elif kind == "whole":
            nxt = rng.permutation(w.num_rows)[: w.cache_rows].astype(np.int64)
        elif kind == "too_many":
            nxt = rng.permutation(w.num_rows)[: w.cache_rows + 1].astype(np.int64)
        else:
            nxt = some(1, 1)
        noff = np.arange(len(nxt) + 1, dtype=np.int64)
        nxt_d, noff_d = torch.from_numpy(nxt).to(dev), torch.from_numpy(noff).to(dev)
        keep.append((nxt_d, noff_d, off_d))
        torch.cuda.synchronize()
        if kind == "too_many":
            sr_before = orc.slot_rank
            with pytest.raises(FreqCacheError) as e:
                gpu.plan_next(nxt_d, noff_d)
            assert e.value.name == "BATCH_EXCEEDS_CACHE"
            gpu.advance()                            # nothing planned: a no-op
            sr, rs = gpu.state()
            assert np.array_equal(sr, sr_before) and np.array_equal(rs, orc.rank_slot)
            assert_close(gpu.rows(), orc.cache, f"step {t}: rows after a refused plan")
            nxt = nxt[: w.cache_rows // 2]           # the caller splits the batch and goes on
            noff = np.arange(len(nxt) + 1, dtype=np.int64)
            nxt_d, noff_d = torch.from_numpy(nxt).to(dev), torch.from_numpy(noff).to(dev)
            keep.append((nxt_d, noff_d))
            torch.cuda.synchronize()
        sd_next = gpu.plan_next(nxt_d, noff_d)
        gstats = gpu.stats()
        gpu.advance()
        so_next = orc.prepare(nxt, noff)
        assert gstats == orc.stats(), f"step {t} ({kind}): stats {gstats} vs {orc.stats()}"
        compare_prepare(gpu, orc, sd_next.cpu().numpy(), so_next, t)
        assert_close(gpu.rows(), orc.cache, f"step {t} ({kind}): cached rows after the rows moved")
        so, sd, cur = so_next, sd_next, (nxt, noff)
    gpu.check()
    gpu.flush(); orc.flush()
    assert_close(gpu.host_weight(), orc.host, "host table")
    gpu.close()


def test_two_tables_interleaved(torch_cuda):
    """Two caches (different shapes and transmitters) driven in turn on one stream: no state is shared between handles."""
    torch = torch_cuda
    dev = torch.device("cuda:0")
    wa = TinyWorkload(num_rows=5000, dim=32, cache_rows=300, seed=31, multi_hot=True)
    wb = TinyWorkload(num_rows=2000, dim=6, cache_rows=150, seed=32, multi_hot=False)
    ga, oa = make_pair(wa, warm=True, dma_evict=True)
    gb, ob = make_pair(wb, warm=False)
    sa = sb = None
    for t in range(8):
        for w, g, o in ((wa, ga, oa), (wb, gb, ob)):
            ids, off = w.batch(t)
            grad = w.grad(t, len(off) - 1)
            ids_d, off_d = torch.from_numpy(ids).to(dev), torch.from_numpy(off).to(dev)
            so = o.prepare(ids, off)
            sd = g.prepare(ids_d, off_d)
            compare_prepare(g, o, sd.cpu().numpy(), so, t)
            assert_close(g.embedding_bag_fwd(sd, off_d).cpu().numpy(), o.embedding_bag_fwd(so, off), f"batch {t}: pooled output")
            g.embedding_bag_bwd_sgd(sd, off_d, torch.from_numpy(grad).to(dev), w.lr)
            o.embedding_bag_bwd_sgd(so, off, grad, w.lr)
    for g, o in ((ga, oa), (gb, ob)):
        assert_close(g.rows(), o.cache, "cached rows")
        g.check(); g.flush(); o.flush()
        assert_close(g.host_weight(), o.host, "host table")
        g.close()


def test_profile_timeline_file(torch_cuda, tmp_path, monkeypatch):
    """FC_TIMELINE: every timed kernel of the profiled steps appears once with start <= end, and the per-kernel totals of
    cache_profile_get are the sums of those spans."""
    torch = torch_cuda
    from paper_2208_05321_amd import FreqCache
    from tests.timeline_file import load_first_collection
    w = make_workload("c1")
    dev = torch.device("cuda:0")
    path = tmp_path / "timeline.txt"
    monkeypatch.setenv("FC_TIMELINE", str(path))
    gpu = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, dma_evict=True)
    w.host_table(out=gpu.host_weight())
    gpu.warm()
    gpu.profile(True)
    steps = 3
    for t in range(steps):
        ids, off = w.batch(t)
        ids_d, off_d = torch.from_numpy(ids).to(dev), torch.from_numpy(off).to(dev)
        slots = gpu.prepare(ids_d, off_d)
        gpu.embedding_bag_fwd(slots, off_d)
        gpu.embedding_bag_bwd_sgd(slots, off_d, torch.from_numpy(w.grad(t, len(off) - 1)).to(dev), w.lr)
    rep = gpu.profile_report()
    gpu.profile(False)
    monkeypatch.delenv("FC_TIMELINE")
    gpu.profile(False)                                   # a collection without the variable closes the file
    gpu.close()
    spans = load_first_collection(str(path))
    assert spans and all(a <= b for a, b, _ in spans)
    for name in ("remap_mark", "bag_fwd", "bwd_reduce"):
        mine = [(a, b) for a, b, n in spans if n == name]
        assert len(mine) == steps == rep[name]["launches"]
        assert abs(sum(b - a for a, b in mine) * 1e-3 - rep[name]["ms"]) < 0.01 * steps
    fwd = sorted(a for a, b, n in spans if n == "bag_fwd")
    bwd = sorted(a for a, b, n in spans if n == "bwd_reduce")
    assert all(f < g for f, g in zip(fwd, bwd))           # same stream: forward before backward in every step


@pytest.mark.parametrize("dma", [False, True])
def test_batch_prepared_but_not_trained_leaves_no_sort_behind(torch_cuda, dma):
    """Static input / slot buffers reused by every batch (as a training loop with preallocated tensors does), and
    batches that are prepared and pooled but never trained on (evaluation steps): the backward pass of a later batch
    must use that batch's own sorted lookups, never the ones sorted ahead of time for an earlier batch that happened to
    live in the same buffers.  Also with reserved buffers (cache_reserve), so that nothing is allocated in the loop."""
    torch = torch_cuda
    w = make_workload("c2", scale=0.05, cache_ratio=0.03)
    gpu, orc = make_pair(w, warm=True, dma_evict=dma)
    dev = torch.device("cuda:0")
    n = len(w.batch(0)[0])
    gpu.reserve(n, pipelined=True)
    ids_d = torch.empty(n, dtype=torch.int64, device=dev)
    off_d = torch.empty(w.bags_per_batch + 1, dtype=torch.int64, device=dev)
    slots_d = torch.empty(n, dtype=torch.int32, device=dev)
    grad_d = torch.empty((w.bags_per_batch, w.dim), dtype=torch.float32, device=dev)
    for t in range(9):
        ids, off = w.batch(t)
        assert len(ids) == n
        torch.cuda.synchronize()
        ids_d.copy_(torch.from_numpy(ids)); off_d.copy_(torch.from_numpy(off))
        so = orc.prepare(ids, off)
        gpu.prepare(ids_d, off_d, out=slots_d)
        assert np.array_equal(slots_d.cpu().numpy(), so), f"batch {t}: slots"
        out = gpu.embedding_bag_fwd(slots_d, off_d)
        assert_close(out.cpu().numpy(), orc.embedding_bag_fwd(so, off), f"batch {t}: pooled output")
        if t % 3 != 1:                          # batches 1, 4, 7 are evaluation steps: no backward pass
            g = w.grad(t, w.bags_per_batch)
            grad_d.copy_(torch.from_numpy(g))
            gpu.embedding_bag_bwd_sgd(slots_d, off_d, grad_d, w.lr)
            orc.embedding_bag_bwd_sgd(so, off, g, w.lr)
        assert_close(gpu.rows(), orc.cache, f"batch {t}: cached rows")
    gpu.check()
    gpu.flush()
    orc.flush()
    assert_close(gpu.host_weight(), orc.host, "host table")
    gpu.close()
