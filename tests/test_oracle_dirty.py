"""Pins of the oracle's dirty-tracking variant (not in the paper: only victims that a backward pass has updated since they
were loaded are written back; Algorithm 1 itself always calls move_to_cpu).  What fixes it: values never change, the
write-back set is the set a model independent of the oracle predicts, a trace small enough to work out by hand."""
import numpy as np
import pytest

from oracle import Oracle
from tests.alg1_bruteforce import BruteForceCache
from workloads import table_values


def offs(n):
    return np.arange(n + 1, dtype=np.int64)


def default_mk(fr, host, C, warm, dirty):
    return Oracle(fr, host, C, warm=warm, dirty_tracking=dirty)


def pin_handworked(mk):
    """6 rows, identity ranks, 2 slots, cold, rows of 4 floats (16 bytes).
    b0 ids 0,1 trained    -> both loaded, then dirty;                      nothing evicted
    b1 id 2, forward only -> victim rank 1 (largest not in batch), dirty:  16 bytes written; rank 2 sits clean in slot 1
    b2 id 3, trained      -> victim rank 2, clean:                          0 bytes;          rank 3 in slot 1, then dirty
    b3 ids 4,5, forward   -> victims ranks 0 and 3, both dirty:             32 bytes"""
    fr = np.arange(6, dtype=np.int32)
    host = table_values(1, np.arange(6), 4).copy()
    o = mk(fr, host, 2, False, True)
    plan = [([0, 1], True, 0, [0, 0]), ([2], False, 16, [1, 0]), ([3], True, 0, [1, 0]), ([4, 5], False, 32, [0, 0])]
    for ids, train, bytes_d2h, dirty_before_bwd in plan:
        ids = np.array(ids, dtype=np.int64)
        slots = o.prepare(ids, offs(len(ids)))
        assert o.stats()["bytes_d2h"] == bytes_d2h, (ids, o.stats())
        assert list(o.dirty) == dirty_before_bwd, (ids, o.dirty)
        if train:
            o.embedding_bag_bwd_sgd(slots, offs(len(ids)), np.ones((len(ids), 4), np.float32), 0.5)
            assert all(o.dirty[s] == 1 for s in slots)


def pin_values_identical(mk):
    """Same trace (a mix of trained and forward-only batches) with and without tracking: every output, the maps and
    lists, and the flushed table are bit-identical; the tracked run never writes more."""
    for seed in range(3):
        rng = np.random.default_rng(70 + seed)
        N, D, C = 60, 3, 8
        fr = rng.permutation(N).astype(np.int32)
        h_plain = table_values(seed, np.argsort(fr), D).copy()
        h_track = h_plain.copy()
        warm = bool(seed % 2)
        a, b = mk(fr, h_plain, C, warm, False), mk(fr, h_track, C, warm, True)
        for t in range(40):
            k = int(rng.integers(1, C + 1))
            ids = rng.permutation(N)[:k]
            ids = np.concatenate([ids, ids[:2]]).astype(np.int64)
            sa, sb = a.prepare(ids, offs(len(ids))), b.prepare(ids, offs(len(ids)))
            assert np.array_equal(sa, sb) and np.array_equal(a.slot_rank, b.slot_rank)
            la, lb = a.last_lists(), b.last_lists()
            assert all(np.array_equal(la[key], lb[key]) for key in la)
            assert b.stats()["bytes_d2h"] <= a.stats()["bytes_d2h"]
            assert {k_: v for k_, v in a.stats().items() if k_ != "bytes_d2h"} == {k_: v for k_, v in b.stats().items() if k_ != "bytes_d2h"}
            assert np.array_equal(a.embedding_bag_fwd(sa, offs(len(ids))), b.embedding_bag_fwd(sb, offs(len(ids))))
            if rng.random() < 0.6:
                g = rng.standard_normal((len(ids), D)).astype(np.float32)
                a.embedding_bag_bwd_sgd(sa, offs(len(ids)), g, 0.3)
                b.embedding_bag_bwd_sgd(sb, offs(len(ids)), g, 0.3)
            assert np.array_equal(a.cache, b.cache)
            if t == 20:                       # a flush in the middle leaves every resident row clean
                a.flush(); b.flush()
                assert np.array_equal(h_plain, h_track) and not b.dirty.any()
        a.flush(); b.flush()
        assert np.array_equal(h_plain, h_track)


def pin_writeback_set_against_model(mk):
    """The write-back set predicted without the oracle: a brute-force statement of Algorithm 1 (Python sets) gives the victims; a Python set
    of rows updated since they were loaded says which of them are dirty."""
    for seed in range(3):
        rng = np.random.default_rng(90 + seed)
        N, D, C = 40, 2, 6
        fr = rng.permutation(N).astype(np.int32)
        ha = table_values(seed, np.arange(N), D).copy()
        warm = bool(seed % 2)
        o = mk(fr, ha, C, warm, True)
        ref = BruteForceCache(fr, ha.copy(), C, warm=warm)
        updated = set()
        for t in range(50):
            k = int(rng.integers(1, C + 1))
            ids = rng.permutation(N)[:k].astype(np.int64)
            ref.prepare_cache(ids)
            slots = o.prepare(ids, offs(k))
            written = [r for r in ref.evicted if int(r) in updated]
            assert o.stats()["bytes_d2h"] == len(written) * D * 4
            updated -= {int(r) for r in ref.evicted}
            if t % 3 != 2:
                o.embedding_bag_bwd_sgd(slots, offs(k), np.ones((k, D), np.float32), 0.1)
                updated |= {int(r) for r in fr[ids]}
            sr = o.slot_rank
            assert [bool(d) for d in o.dirty] == [int(r) in updated for r in sr]


def pin_forward_only_never_writes(mk):
    rng = np.random.default_rng(5)
    N, D, C = 30, 2, 5
    fr = rng.permutation(N).astype(np.int32)
    host = table_values(2, np.arange(N), D).copy()
    before = host.copy()
    o = mk(fr, host, C, True, True)
    for t in range(30):
        ids = rng.permutation(N)[:C].astype(np.int64)
        o.prepare(ids, offs(C))
        assert o.stats()["bytes_d2h"] == 0 and o.stats()["n_evict"] > 0
    o.flush()
    assert np.array_equal(host, before)


def pin_cold_and_always_trained_equals_plain_policy(mk):
    """From a cold start with a backward pass after every batch every resident row is dirty: same bytes as always writing."""
    rng = np.random.default_rng(6)
    N, D, C = 30, 2, 5
    fr = rng.permutation(N).astype(np.int32)
    a = mk(fr, table_values(2, np.arange(N), D).copy(), C, False, False)
    b = mk(fr, table_values(2, np.arange(N), D).copy(), C, False, True)
    for t in range(30):
        ids = rng.permutation(N)[: int(rng.integers(1, C + 1))].astype(np.int64)
        sa, sb = a.prepare(ids, offs(len(ids))), b.prepare(ids, offs(len(ids)))
        assert a.stats() == b.stats()
        g = np.ones((len(ids), D), np.float32)
        a.embedding_bag_bwd_sgd(sa, offs(len(ids)), g, 0.1)
        b.embedding_bag_bwd_sgd(sb, offs(len(ids)), g, 0.1)


DIRTY_PINS = [pin_handworked, pin_values_identical, pin_writeback_set_against_model, pin_forward_only_never_writes,
              pin_cold_and_always_trained_equals_plain_policy]


@pytest.mark.parametrize("pin", DIRTY_PINS, ids=[p.__name__ for p in DIRTY_PINS])
def test_dirty_tracking_pin(pin):
    pin(default_mk)
