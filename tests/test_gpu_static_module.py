"""`-m gpu`: the GPU build of the static module (id counts -> freq_rank -> re-ordered table) against the oracle."""
import numpy as np
import pytest

from workloads import make_workload, table_values

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    from paper_2208_05321_amd import load_library
    load_library()
    return torch


def build_both(torch, num_rows, batches):
    from oracle import count_ids, freq_rank_from_counts
    from paper_2208_05321_amd import FreqCounter
    dev = torch.device("cuda:0")
    fc = FreqCounter(num_rows)
    for ids in batches:
        fc.add(torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int64)).to(dev))
    fr, inv, cnt = fc.build(with_counts=True)
    fc.close()
    counts = count_ids(batches, num_rows)
    fr_o, inv_o = freq_rank_from_counts(counts)
    assert np.array_equal(cnt, counts)                      # integer work: bit-exact
    assert np.array_equal(inv, inv_o) and np.array_equal(fr, fr_o)
    return fr, inv


@pytest.mark.parametrize("name,scale", [("c1", 1.0), ("c2", 0.1), ("c5", 0.02)])
def test_freq_rank_from_trace(torch_cuda, name, scale):
    w = make_workload(name, scale=scale)
    batches = [w.batch(t)[0] for t in range(12)]
    fr, inv = build_both(torch_cuda, w.num_rows, batches)
    # the hot rows of the generator's own ranking come out on top
    top = inv[:50]
    assert np.median(w.freq_rank[top]) < 200


def test_freq_rank_edge_cases(torch_cuda):
    torch = torch_cuda
    rng = np.random.default_rng(0)
    # no ids at all: every count is 0 -> identity ranking
    build_both(torch, 1000, [])
    # one id only, many times (one 9-bit pass is not enough for the count); ragged tile sizes
    build_both(torch, 4097, [np.full(5000, 17), np.full(3, 4096)])
    # a count above 2^18 (5,000,000 needs 23 bits) takes three radix passes, the counts before one and two
    build_both(torch, 300, [np.concatenate([np.full(5_000_000, 7), rng.integers(0, 300, size=100_000)])])
    # a table larger than one sort tile with all-distinct counts
    ids = np.repeat(np.arange(3000), np.arange(3000) % 7 + 1)
    rng.shuffle(ids)
    build_both(torch, 20000, [ids])


def test_freq_add_rejects_out_of_range(torch_cuda):
    torch = torch_cuda
    from paper_2208_05321_amd import FreqCounter, FreqCacheError
    fc = FreqCounter(100)
    fc.add(torch.tensor([1, 2, 100], dtype=torch.int64, device="cuda:0"))
    with pytest.raises(FreqCacheError) as e:
        fc.build()
    assert e.value.name == "ID_OUT_OF_RANGE"
    fc.close()


def test_table_reorder_and_cache_on_built_ranks(torch_cuda):
    """End to end: ranks built on the GPU from a warm-up trace, table re-ordered on the GPU, cache run on them."""
    torch = torch_cuda
    from oracle import reorder_table
    from paper_2208_05321_amd import table_reorder, FreqCache
    from tests.parity import run_parity
    w = make_workload("c2", scale=0.05, cache_ratio=0.03)
    fr, inv = build_both(torch, w.num_rows, [w.batch(1000 + t)[0] for t in range(20)])
    src = torch.empty((w.num_rows, w.dim), dtype=torch.float32, pin_memory=True)
    src.numpy()[:] = table_values(0, np.arange(w.num_rows), w.dim)           # table in id order
    dst = torch.empty_like(src).pin_memory() if not torch.empty_like(src).is_pinned() else torch.empty_like(src)
    table_reorder(src, dst, inv)
    assert np.array_equal(dst.numpy(), reorder_table(src.numpy(), inv))
    # run the cache on the GPU-built ranking (the workload's table generator follows inv_rank)
    w.freq_rank, w.inv_rank = fr, inv
    run_parity(w, 6, warm=True)


@pytest.mark.slow
def test_config3_ranks_built_by_the_library_at_full_size(torch_cuda):
    """Config 3's frequency ranks (33.8M rows, counted on a 10M-sample warm-up trace of 26 ids per sample) built with
    freq_add / freq_build: identical to the ranking the input generator derives from the same trace on the CPU, and to
    the numpy oracle of the static module."""
    torch = torch_cuda
    import time
    from oracle import count_ids, freq_rank_from_counts
    from paper_2208_05321_amd import FreqCounter
    t0 = time.time()
    w = make_workload("c3")
    print(f"c3 built in {time.time() - t0:.0f}s", flush=True)
    dev = torch.device("cuda:0")
    fc = FreqCounter(w.num_rows)
    counts = np.zeros(w.num_rows, dtype=np.int64)
    n = 0
    for ids in w.warmup_trace():
        fc.add(torch.from_numpy(ids).to(dev))
        counts += np.bincount(ids, minlength=w.num_rows)
        n += len(ids)
    assert n == w.warm_samples * w.num_features
    fr, inv, cnt = fc.build(with_counts=True)
    fc.close()
    assert np.array_equal(cnt, counts)
    assert np.array_equal(fr, w.freq_rank) and np.array_equal(inv, w.inv_rank)       # the generator's empirical ranking
    fr_o, inv_o = freq_rank_from_counts(counts)
    assert np.array_equal(fr, fr_o) and np.array_equal(inv, inv_o)
    print(f"ranks of {w.num_rows} rows from {n} ids identical ({time.time() - t0:.0f}s)", flush=True)


@pytest.mark.slow
def test_table_reorder_at_config2_size(torch_cuda):
    """table_reorder on a 10M x 128 table (5.1 GB) between two pinned host tables against the oracle's re-ordering."""
    torch = torch_cuda
    from oracle import reorder_table
    from paper_2208_05321_amd import table_reorder
    from workloads.gen import fill_host_table
    w = make_workload("c2")
    src = torch.empty((w.num_rows, w.dim), dtype=torch.float32, pin_memory=True)
    fill_host_table(src.numpy(), 0, None)                                     # the table in id order
    dst = torch.empty((w.num_rows, w.dim), dtype=torch.float32, pin_memory=True)
    table_reorder(src, dst, w.inv_rank)
    ref = reorder_table(src.numpy(), w.inv_rank)
    assert np.array_equal(dst.numpy(), ref)
    # it is the table the input generator builds row by row for the cache
    probe = np.random.default_rng(0).integers(0, w.num_rows, size=1000)
    assert np.array_equal(dst.numpy()[probe], table_values(0, w.inv_rank[probe], w.dim))


def test_freq_add_refuses_what_would_overflow_its_counters(torch_cuda):
    torch = torch_cuda
    from paper_2208_05321_amd import FreqCounter, FreqCacheError
    fc = FreqCounter(50)
    ids = torch.arange(50, dtype=torch.int64, device="cuda:0")
    fc.add(ids)
    rc = fc._L.freq_add(fc._h, ids.data_ptr(), (1 << 31) - 50)               # refused on the host before any id is read
    assert rc == -12
    fr, inv, cnt = fc.build(with_counts=True)
    assert np.array_equal(cnt, np.ones(50, dtype=np.int32))                   # nothing was counted by the refused call
    fc.close()
