"""Pins for the CPU oracle (oracle/fc_oracle.c): everything here runs without a GPU.

P0  hand-worked traces of Algorithm 1 (tests/golden/alg1_handworked.json)
P1  brute-force statement of Algorithm 1 with Python sets and dicts (tests/alg1_bruteforce.py) on tiny tables, random traces
P2  cache transparency: flushed table == EmbeddingBag-sum + SGD on the whole table, no cache
    (Section 2.2: updates are synchronous, so the cache must be invisible)
P3  closed form for config 1 (all-ones gradient, one id per bag)
P4  special cases of the policy
I1-I6 invariants (maps inverse, residency, conservation, inclusion in cache size, ...)
"""
import json
import os

import numpy as np
import pytest
import torch

from oracle import Oracle, OracleError
from tests.alg1_bruteforce import BruteForceCache
from workloads import make_workload, table_values

HERE = os.path.dirname(os.path.abspath(__file__))


def one_hot_offsets(n):
    return np.arange(n + 1, dtype=np.int64)


def rand_table(N, D, seed=0):
    return table_values(seed, np.arange(N), D).copy()


def check_maps(o: Oracle):
    sr, rs = o.slot_rank, o.rank_slot
    res = sr[sr >= 0]
    assert len(np.unique(res)) == len(res), "I1: duplicate row in cache"
    assert (rs[res] == np.nonzero(sr >= 0)[0]).all(), "I1: rank_slot[slot_rank[s]] != s"
    on = np.nonzero(rs >= 0)[0]
    assert (sr[rs[on]] == on).all(), "I1: slot_rank[rank_slot[u]] != u"
    assert len(on) == len(res)
    assert ((sr >= 0) | (sr == -1)).all()


# ---------------------------------------------------------------- P0
def test_handworked_traces():
    g = json.load(open(os.path.join(HERE, "golden", "alg1_handworked.json")))
    N, C = g["num_rows"], g["cache_rows"]
    fr = np.array(g["freq_rank"], dtype=np.int32)
    for tr in g["traces"]:
        host = rand_table(N, 4)
        o = Oracle(fr, host, C, warm=tr["warm"])
        for b in tr["batches"]:
            ids = np.array(b["ids"], dtype=np.int64)
            assert list(fr[ids]) == b["ranks"]
            slots = o.prepare(ids, one_hot_offsets(len(ids)))
            L, s = o.last_lists(), o.stats()
            assert list(L["miss_ranks"]) == b["miss_ranks"]
            assert list(L["evict_ranks"]) == b["evict_ranks"]
            assert list(L["fill_slots"]) == b["fill_slots"]
            assert list(o.slot_rank) == b["slot_rank_after"]
            assert list(slots) == b["slots"]
            assert s["n_hit_ids"] == b["n_hit_ids"] and s["n_unique"] == b["n_unique"]
            assert s["bytes_h2d"] == len(b["miss_ranks"]) * 4 * 4
            assert s["bytes_d2h"] == len(b["evict_ranks"]) * 4 * 4
            check_maps(o)


# ---------------------------------------------------------------- P1
@pytest.mark.parametrize("seed", range(12))
def test_against_array_ops_algorithm1(seed):
    rng = np.random.default_rng(seed)
    N = int(rng.integers(6, 64))
    C = int(rng.integers(1, min(N, 9) + 1))
    D = 3
    warm = bool(seed % 2)
    fr = rng.permutation(N).astype(np.int32)
    host_a = rand_table(N, D, seed)
    host_b = host_a.copy()
    o = Oracle(fr, host_a, C, warm=warm)
    ref = BruteForceCache(fr, host_b, C, warm=warm)
    for t in range(40):
        kind = t % 5
        if kind == 0:      # exactly C distinct rows: the whole cache is needed
            ids = rng.permutation(N)[:C]
        elif kind == 1:    # all hits: rows currently resident (or a cold start)
            res = np.nonzero(o.rank_slot >= 0)[0]
            ids = np.argsort(fr)[res][: max(1, C // 2)] if len(res) else rng.integers(0, N, size=1)
        else:
            k = int(rng.integers(1, C + 1))
            ids = rng.permutation(N)[:k]
            ids = np.concatenate([ids, ids[rng.integers(0, k, size=int(rng.integers(0, 4)))]])  # duplicates
            rng.shuffle(ids)
        ids = ids.astype(np.int64)
        # perturb resident rows so that write-back moves distinguishable data
        slots_ref = ref.prepare_cache(ids)
        slots = o.prepare(ids, one_hot_offsets(len(ids)))
        L, s = o.last_lists(), o.stats()
        assert np.array_equal(slots, slots_ref)
        assert np.array_equal(o.slot_rank, ref.cache_idx_map)
        assert np.array_equal(L["miss_ranks"], ref.missed)
        assert np.array_equal(L["evict_ranks"], ref.evicted)
        assert np.array_equal(L["fill_slots"], ref.targets)
        assert s["n_hit_ids"] == ref.hit_ids
        assert s["n_miss"] == len(ref.missed) and s["n_evict"] == len(ref.evicted)
        assert s["n_hit_unique"] == s["n_unique"] - s["n_miss"]
        check_maps(o)
        # update cached rows identically on both sides (same slots): a fake optimizer step
        g = rng.standard_normal((len(ids), D)).astype(np.float32)
        o.embedding_bag_bwd_sgd(slots, one_hot_offsets(len(ids)), g, 0.5)
        acc = np.zeros_like(ref.cuda_weight)
        for i, sl in enumerate(slots_ref):
            acc[sl] = acc[sl] + g[i]
        for sl in np.unique(slots_ref):
            ref.cuda_weight[sl] = ref.cuda_weight[sl] - np.float32(0.5) * acc[sl]
        assert np.array_equal(o.cache, ref.cuda_weight)
        assert np.array_equal(host_a, host_b)


# ---------------------------------------------------------------- P2
def no_cache_training(W, batches, lr):
    """EmbeddingBag(sum) + SGD on the full table in id space, lookups accumulated in position order."""
    outs = []
    for ids, offsets, grad in batches:
        B = len(offsets) - 1
        out = np.zeros((B, W.shape[1]), dtype=np.float32)
        g = {}
        for b in range(B):
            for i in range(offsets[b], offsets[b + 1]):
                out[b] = out[b] + W[ids[i]]
        for b in range(B):
            for i in range(offsets[b], offsets[b + 1]):
                k = int(ids[i])
                g[k] = (g[k] + grad[b]) if k in g else (np.zeros(W.shape[1], np.float32) + grad[b])
        for k, gk in g.items():
            W[k] = W[k] - np.float32(lr) * gk
        outs.append(out)
    return outs


def random_bags(rng, N, C, multi):
    if multi:
        B = int(rng.integers(1, 6))
        sizes = rng.integers(0, 4, size=B)
        n = int(sizes.sum())
        offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    else:
        n = int(rng.integers(1, C + 3))
        offsets = one_hot_offsets(n)
    pool = rng.permutation(N)[: max(1, min(C, n))]
    ids = pool[rng.integers(0, len(pool), size=n)].astype(np.int64)
    return ids, offsets


@pytest.mark.parametrize("seed,warm,multi", [(s, w, m) for s in range(4) for w in (0, 1) for m in (0, 1)])
def test_cache_is_transparent(seed, warm, multi):
    rng = np.random.default_rng(100 + seed)
    N, D = 50, 5
    C = int(rng.integers(3, 12))
    fr = rng.permutation(N).astype(np.int32)
    inv = np.argsort(fr)
    W = rand_table(N, D, seed)                 # id space
    host = W[inv].copy()                       # rank space: row rho = W[id with rank rho]
    o = Oracle(fr, host, C, warm=bool(warm))
    batches = []
    for t in range(30):
        ids, offsets = random_bags(rng, N, C, multi)
        grad = rng.standard_normal((len(offsets) - 1, D)).astype(np.float32)
        batches.append((ids, offsets, grad))
    W_ref = W.copy()
    outs_ref = no_cache_training(W_ref, batches, 0.1)
    for (ids, offsets, grad), out_ref in zip(batches, outs_ref):
        slots = o.prepare(ids, offsets)
        out = o.embedding_bag_fwd(slots, offsets)
        assert np.array_equal(out, out_ref)          # same fp32 operations in the same order
        o.embedding_bag_bwd_sgd(slots, offsets, grad, 0.1)
        check_maps(o)
    o.flush()
    assert np.array_equal(host, W_ref[inv])          # I3: host + cache == full table after flush


def test_values_against_torch_embedding_bag_autograd():
    """Same as P2 but the reference is the library routine: torch EmbeddingBag(sum) + autograd + SGD."""
    rng = np.random.default_rng(7)
    N, D, C = 200, 8, 20
    fr = rng.permutation(N).astype(np.int32)
    inv = np.argsort(fr)
    W = rand_table(N, D, 3)
    host = W[inv].copy()
    o = Oracle(fr, host, C, warm=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    for t in range(25):
        B = 12
        sizes = rng.integers(0, 5, size=B)
        offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        pool = rng.permutation(N)[:C]
        ids = pool[rng.integers(0, C, size=int(sizes.sum()))].astype(np.int64)
        grad = rng.standard_normal((B, D)).astype(np.float32)
        slots = o.prepare(ids, offsets)
        out = o.embedding_bag_fwd(slots, offsets)
        o.embedding_bag_bwd_sgd(slots, offsets, grad, 0.05)
        out_t = torch.nn.functional.embedding_bag(torch.tensor(ids), Wt, torch.tensor(offsets[:-1]), mode="sum")
        np.testing.assert_allclose(out, out_t.detach().numpy(), rtol=1e-5, atol=1e-7)
        out_t.backward(torch.tensor(grad, dtype=torch.float64))
        with torch.no_grad():
            Wt -= 0.05 * Wt.grad
            Wt.grad.zero_()
    o.flush()
    np.testing.assert_allclose(host, Wt.detach().numpy()[inv], rtol=1e-5, atol=1e-6)


# ---------------------------------------------------------------- P3
@pytest.mark.parametrize("warm", [True, False])
def test_config1_closed_form(warm):
    w = make_workload("c1")
    host = w.host_table()
    W0 = host.copy()
    o = Oracle(w.freq_rank, host, w.cache_rows, warm=warm)
    count = np.zeros(w.num_rows, dtype=np.int64)
    hits = tot = 0
    for t in range(w.num_batches):
        ids, offsets = w.batch(t)
        slots = o.prepare(ids, offsets)
        s = o.stats()
        hits += s["n_hit_ids"]
        tot += s["n_ids"]
        o.embedding_bag_fwd(slots, offsets)
        o.embedding_bag_bwd_sgd(slots, offsets, w.grad(t, len(offsets) - 1), w.lr)
        np.add.at(count, w.freq_rank[ids], 1)
    o.flush()
    expect = W0.astype(np.float64) - 0.01 * count[:, None]
    np.testing.assert_allclose(host, expect, rtol=1e-4, atol=1e-6)
    assert 0.5 < hits / tot < 0.95        # skewed ids: most lookups hit a 1.5% cache (Section 3)


# ---------------------------------------------------------------- P4
def test_full_size_cache_never_misses():
    N, D = 40, 2
    rng = np.random.default_rng(1)
    fr = rng.permutation(N).astype(np.int32)
    host = rand_table(N, D)
    o = Oracle(fr, host, N, warm=True)
    for t in range(5):
        ids = rng.integers(0, N, size=30).astype(np.int64)
        slots = o.prepare(ids, one_hot_offsets(30))
        s = o.stats()
        assert s["n_miss"] == 0 and s["n_evict"] == 0 and s["n_hit_ids"] == 30
        assert np.array_equal(slots, fr[ids])      # warm-up puts cpu_row_idx s into slot s


def test_cold_cache_large_enough_only_first_touch_misses():
    N, D, C = 100, 2, 60
    rng = np.random.default_rng(2)
    fr = rng.permutation(N).astype(np.int32)
    o = Oracle(fr, rand_table(N, D), C, warm=False)
    pool = rng.permutation(N)[:C]
    seen = set()
    for t in range(20):
        ids = pool[rng.integers(0, C, size=25)].astype(np.int64)
        o.prepare(ids, one_hot_offsets(25))
        s = o.stats()
        new = set(ids.tolist()) - seen
        assert s["n_miss"] == len(new) and s["n_evict"] == 0
        seen |= new


def test_first_warm_batch_hits_are_top_ranks():
    w = make_workload("c2", scale=0.01, cache_ratio=0.05)
    o = Oracle(w.freq_rank, w.host_table(), w.cache_rows, warm=True)
    ids, offsets = w.batch(0)
    o.prepare(ids, offsets)
    r = np.unique(w.freq_rank[ids])
    L = o.last_lists()
    assert np.array_equal(L["miss_ranks"], r[r >= w.cache_rows])
    # LFU by static rank: victims are exactly the largest resident ranks not used by the batch
    resident_unused = np.setdiff1d(np.arange(w.cache_rows), r)
    assert np.array_equal(L["evict_ranks"], resident_unused[len(resident_unused) - len(L["evict_ranks"]):])


def test_victims_have_largest_rank_and_batch_rows_protected():
    rng = np.random.default_rng(5)
    N, C = 300, 40
    fr = rng.permutation(N).astype(np.int32)
    o = Oracle(fr, rand_table(N, 2), C, warm=True)
    for t in range(50):
        ids = rng.integers(0, N, size=int(rng.integers(1, C))).astype(np.int64)
        before = o.slot_rank
        o.prepare(ids, one_hot_offsets(len(ids)))
        U = np.unique(fr[ids])
        L, s = o.last_lists(), o.stats()
        ev = L["evict_ranks"]
        free_before = int((before == -1).sum())
        assert len(ev) == max(0, s["n_miss"] - free_before)          # I2: |V| = need
        assert len(np.intersect1d(ev, U)) == 0                       # protected
        still = np.setdiff1d(before[before >= 0], np.concatenate([ev, U]))
        if len(ev) and len(still):
            assert ev.min() > still.max()                            # every victim ranks below every survivor
        assert (o.rank_slot[fr[ids]] >= 0).all()                     # I2: all rows of the batch resident
        res_before, res_after = int((before >= 0).sum()), int((o.slot_rank >= 0).sum())
        assert res_after == res_before + s["n_miss"] - s["n_evict"]  # I5
        assert s["bytes_h2d"] + s["bytes_d2h"] == (s["n_miss"] + s["n_evict"]) * 2 * 4


# ---------------------------------------------------------------- I4
@pytest.mark.parametrize("warm", [True, False])
def test_resident_set_inclusion_in_cache_size(warm):
    """Priority (in current batch, then static rank) does not depend on C, so the resident set at C is a
    subset of the resident set at C' > C after every batch; hit counts are therefore monotone in C."""
    w = make_workload("c2", scale=0.003)
    sizes = sorted([w.samples * 26 + 8, w.samples * 26 * 2, w.samples * 26 * 4, w.num_rows // 3])
    host = w.host_table()
    orcs = [Oracle(w.freq_rank, host.copy(), c, warm=warm) for c in sizes]
    hits = [0] * len(sizes)
    for t in range(25):
        ids, offsets = w.batch(t)
        prev = None
        for k, o in enumerate(orcs):
            o.prepare(ids, offsets)
            hits[k] += o.stats()["n_hit_ids"]
            res = set(np.nonzero(o.rank_slot >= 0)[0].tolist())
            if prev is not None:
                assert prev <= res
            prev = res
    assert hits == sorted(hits)


# ---------------------------------------------------------------- error paths
def test_error_paths_leave_state_unchanged():
    rng = np.random.default_rng(3)
    N, C, D = 30, 5, 2
    fr = rng.permutation(N).astype(np.int32)
    host = rand_table(N, D)
    o = Oracle(fr, host, C, warm=True)
    o.prepare(np.array([3, 4, 5], dtype=np.int64), one_hot_offsets(3))
    sr, rs, ca, ho = o.slot_rank, o.rank_slot, o.cache, host.copy()

    def unchanged():
        return (np.array_equal(sr, o.slot_rank) and np.array_equal(rs, o.rank_slot)
                and np.array_equal(ca, o.cache) and np.array_equal(ho, host))

    with pytest.raises(OracleError) as e:
        o.prepare(np.arange(C + 1, dtype=np.int64), one_hot_offsets(C + 1))
    assert e.value.name == "BATCH_EXCEEDS_CACHE" and unchanged()
    with pytest.raises(OracleError) as e:
        o.prepare(np.array([1, N], dtype=np.int64), one_hot_offsets(2))
    assert e.value.name == "ID_OUT_OF_RANGE" and unchanged()
    with pytest.raises(OracleError) as e:
        o.prepare(np.array([1, -1], dtype=np.int64), one_hot_offsets(2))
    assert e.value.name == "ID_OUT_OF_RANGE" and unchanged()
    for bad in ([0, 2, 1, 3], [1, 2, 3], [0, 1, 2]):
        with pytest.raises(OracleError) as e:
            o.prepare(np.array([1, 2, 3], dtype=np.int64), np.array(bad, dtype=np.int64))
        assert e.value.name == "BAD_OFFSETS" and unchanged()
    with pytest.raises(OracleError) as e:
        Oracle(np.zeros(N, dtype=np.int32), host, C)
    assert e.value.name == "NOT_PERMUTATION"
    for c in (0, N + 1):
        with pytest.raises(OracleError):
            Oracle(fr, host, c)
    # empty batch and empty bags are fine
    slots = o.prepare(np.empty(0, dtype=np.int64), np.zeros(4, dtype=np.int64))
    assert len(slots) == 0 and unchanged()
    out = o.embedding_bag_fwd(slots, np.zeros(4, dtype=np.int64))
    assert out.shape == (3, D) and (out == 0).all()


# ---------------------------------------------------------------- static module (Section 4.2)
def test_static_module_hand_example():
    from oracle import count_ids, freq_rank_from_counts, reorder_table
    # ids 0..5; occurrences: id3 x4, id1 x2, id5 x2, id0 x1, id2 x0, id4 x0
    trace = [np.array([3, 1, 3, 5]), np.array([3, 0, 5, 1, 3])]
    counts = count_ids(trace, 6)
    assert counts.tolist() == [1, 2, 0, 4, 0, 2]
    fr, inv = freq_rank_from_counts(counts)
    assert inv.tolist() == [3, 1, 5, 0, 2, 4]          # high to low; equal counts: lower id first
    assert fr.tolist() == [3, 1, 4, 0, 5, 2]
    T = np.arange(12, dtype=np.float32).reshape(6, 2)
    assert np.array_equal(reorder_table(T, inv), T[[3, 1, 5, 0, 2, 4]])


@pytest.mark.parametrize("seed", range(5))
def test_static_module_against_python_sort(seed):
    from oracle import count_ids, freq_rank_from_counts
    rng = np.random.default_rng(seed)
    N = int(rng.integers(5, 400))
    trace = [rng.zipf(1.3, size=300) % N for _ in range(3)]
    counts = count_ids(trace, N)
    brute = np.zeros(N, dtype=np.int64)
    for t in trace:
        for i in t:
            brute[i] += 1
    assert np.array_equal(counts, brute)
    fr, inv = freq_rank_from_counts(counts)
    expect = sorted(range(N), key=lambda i: (-int(counts[i]), i))
    assert inv.tolist() == expect
    assert np.array_equal(np.sort(fr), np.arange(N)) and np.array_equal(fr[inv], np.arange(N))
    c = counts[inv]
    assert (np.diff(c) <= 0).all()                               # high to low
    same = np.diff(c) == 0
    assert (np.diff(inv)[same] > 0).all()                        # ties by ascending id
    with pytest.raises(ValueError):
        count_ids([np.array([0, N])], N)


# ---------------------------------------------------------------- look-ahead variant (Future Work section)
@pytest.mark.parametrize("seed", range(8))
def test_lookahead_against_array_ops_algorithm1(seed):
    """Backlist = rows of this batch and of the previously prepared one."""
    rng = np.random.default_rng(500 + seed)
    N = int(rng.integers(20, 80))
    C = int(rng.integers(6, 14))
    fr = rng.permutation(N).astype(np.int32)
    host_a = rand_table(N, 2, seed)
    host_b = host_a.copy()
    o = Oracle(fr, host_a, C, warm=bool(seed % 2))
    ref = BruteForceCache(fr, host_b, C, warm=bool(seed % 2))
    prev = None
    for t in range(40):
        k = int(rng.integers(1, C // 2 + 1))          # two batches always fit together
        ids = rng.permutation(N)[:k].astype(np.int64)
        look = prev is not None and t % 3 != 0       # mix plain and look-ahead calls
        slots_ref = ref.prepare_cache(ids, also_protect=prev if look else None)
        slots = o.prepare(ids, one_hot_offsets(k), lookahead=look)
        L = o.last_lists()
        assert np.array_equal(slots, slots_ref) and np.array_equal(o.slot_rank, ref.cache_idx_map)
        assert np.array_equal(L["evict_ranks"], ref.evicted) and np.array_equal(L["fill_slots"], ref.targets)
        if look:
            assert len(np.intersect1d(L["evict_ranks"], prev)) == 0      # previous batch's rows stay
            assert (o.rank_slot[prev] >= 0).all()
        prev = np.unique(fr[ids])
        check_maps(o)


def test_lookahead_schedule_is_transparent():
    """The schedule the look-ahead is for: batch t+1 is prepared BEFORE batch t's forward/backward run.
    Because batch t's rows are protected, the result still equals no-cache training."""
    rng = np.random.default_rng(77)
    N, D, C = 120, 4, 30
    fr = rng.permutation(N).astype(np.int32)
    inv = np.argsort(fr)
    W = rand_table(N, D, 5)
    host = W[inv].copy()
    o = Oracle(fr, host, C, warm=True)
    batches = []
    for t in range(40):
        n = int(rng.integers(1, 14))
        ids = rng.permutation(N)[:n][rng.integers(0, n, size=n + 2)].astype(np.int64)
        batches.append((ids, one_hot_offsets(len(ids)), rng.standard_normal((len(ids), D)).astype(np.float32)))
    W_ref = W.copy()
    outs_ref = no_cache_training(W_ref, batches, 0.1)
    slots_cur = o.prepare(batches[0][0], batches[0][1])
    for t, (ids, offsets, grad) in enumerate(batches):
        slots_next = o.prepare(batches[t + 1][0], batches[t + 1][1], lookahead=True) if t + 1 < len(batches) else None
        out = o.embedding_bag_fwd(slots_cur, offsets)
        assert np.array_equal(out, outs_ref[t])
        o.embedding_bag_bwd_sgd(slots_cur, offsets, grad, 0.1)
        slots_cur = slots_next
    o.flush()
    assert np.array_equal(host, W_ref[inv])


def test_lookahead_fails_cleanly_when_two_batches_do_not_fit():
    rng = np.random.default_rng(9)
    N, C = 60, 10
    fr = rng.permutation(N).astype(np.int32)
    o = Oracle(fr, rand_table(N, 2), C, warm=True)
    a = np.argsort(fr)[20:28].astype(np.int64)        # 8 rows, none resident
    b = np.argsort(fr)[30:38].astype(np.int64)        # 8 other rows: 16 > 10 together
    o.prepare(a, one_hot_offsets(8))
    sr, rs = o.slot_rank, o.rank_slot
    with pytest.raises(OracleError) as e:
        o.prepare(b, one_hot_offsets(8), lookahead=True)
    assert e.value.name == "BATCH_EXCEEDS_CACHE"
    assert np.array_equal(sr, o.slot_rank) and np.array_equal(rs, o.rank_slot)
    o.prepare(b, one_hot_offsets(8))                  # the plain call fits


def test_bag_sum_on_supplied_rows_is_the_forward_definition():
    """oracle.bag_sum (the forward's arithmetic applied to rows the caller supplies; the GPU tests use it to check the
    forward kernel bit for bit on the GPU's own rows): against a direct fp32 loop, torch's embedding_bag in fp64, and
    Oracle.embedding_bag_fwd on the oracle's own cached rows."""
    import torch
    from oracle import bag_sum
    rng = np.random.default_rng(5)
    C, D = 37, 6
    rows = rng.standard_normal((C, D)).astype(np.float32)
    sizes = rng.integers(0, 5, size=23)                     # empty bags included
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    slots = rng.integers(0, C, size=int(offsets[-1])).astype(np.int32)
    got = bag_sum(rows, slots, offsets)
    ref = np.zeros((len(sizes), D), dtype=np.float32)
    for b in range(len(sizes)):
        for i in range(offsets[b], offsets[b + 1]):
            ref[b] = ref[b] + rows[slots[i]]                # one row after the other, fp32
    assert np.array_equal(got, ref)
    t = torch.nn.functional.embedding_bag(torch.from_numpy(slots.astype(np.int64)), torch.from_numpy(rows.astype(np.float64)),
                                          torch.from_numpy(offsets[:-1]), mode="sum")
    assert np.allclose(got, t.numpy(), rtol=1e-6, atol=1e-6)
    assert np.array_equal(got[sizes == 0], np.zeros((int((sizes == 0).sum()), D), dtype=np.float32))
    # same routine as the oracle's forward on its own rows
    N = 200
    fr = rng.permutation(N).astype(np.int32)
    host = rng.standard_normal((N, D)).astype(np.float32)
    o = Oracle(fr, host, C, warm=True)
    assert np.array_equal(o.embedding_bag_fwd(slots, offsets), bag_sum(o.cache, slots, offsets))
    o.close()
