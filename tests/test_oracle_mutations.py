"""Are the oracle's pins strong enough?  Plant one plausible mistake at a time in a COPY of oracle/fc_oracle.c (on the
CPU, never in the GPU path), build it, and check that the pin battery below rejects every such mutant while it
accepts the real oracle.  The battery is a compact version of tests/test_oracle_pins.py."""
import ctypes
import json
import os
import subprocess
import tempfile

import numpy as np
import pytest

from oracle.wrapper import Oracle, OracleError, _load, _SRC
from tests.alg1_bruteforce import BruteForceCache
from tests.test_oracle_dirty import DIRTY_PINS
from workloads import table_values

HERE = os.path.dirname(os.path.abspath(__file__))


def offs(n):
    return np.arange(n + 1, dtype=np.int64)


def battery(lib):
    """Raises AssertionError (or OracleError) if the oracle build `lib` violates a pin."""
    mk = lambda fr, host, C, warm: Oracle(fr, host, C, warm=warm, lib=lib)
    # the dirty-tracking variant (values unchanged, write-back set against an independent model, hand-worked bytes)
    for pin in DIRTY_PINS:
        pin(lambda fr, host, C, warm, dirty: Oracle(fr, host, C, warm=warm, lib=lib, dirty_tracking=dirty))
    # P0 hand-worked traces
    g = json.load(open(os.path.join(HERE, "golden", "alg1_handworked.json")))
    fr = np.array(g["freq_rank"], dtype=np.int32)
    for tr in g["traces"]:
        o = mk(fr, table_values(0, np.arange(8), 4).copy(), g["cache_rows"], tr["warm"])
        for b in tr["batches"]:
            ids = np.array(b["ids"], dtype=np.int64)
            slots = o.prepare(ids, offs(len(ids)))
            L, s = o.last_lists(), o.stats()
            assert list(L["miss_ranks"]) == b["miss_ranks"] and list(L["evict_ranks"]) == b["evict_ranks"]
            assert list(L["fill_slots"]) == b["fill_slots"] and list(o.slot_rank) == b["slot_rank_after"]
            assert list(slots) == b["slots"] and s["n_hit_ids"] == b["n_hit_ids"] and s["n_unique"] == b["n_unique"]
    # P1 brute-force Algorithm 1 (plain and look-ahead), with row values travelling through evictions
    for seed in range(4):
        rng = np.random.default_rng(seed)
        N, C, D = 40, 7, 3
        fr = rng.permutation(N).astype(np.int32)
        ha = table_values(seed, np.arange(N), D).copy()
        hb = ha.copy()
        o = mk(fr, ha, C, bool(seed % 2))
        ref = BruteForceCache(fr, hb, C, warm=bool(seed % 2))
        prev = None
        for t in range(30):
            k = int(rng.integers(1, C // 2 + 1))
            ids = rng.permutation(N)[:k]
            ids = np.concatenate([ids, ids[:1]]).astype(np.int64)
            look = prev is not None and t % 2 == 1
            s_ref = ref.prepare_cache(ids, also_protect=prev if look else None)
            s_o = o.prepare(ids, offs(len(ids)), lookahead=look)
            L, st = o.last_lists(), o.stats()
            assert np.array_equal(s_o, s_ref) and np.array_equal(o.slot_rank, ref.cache_idx_map)
            assert np.array_equal(L["miss_ranks"], ref.missed) and np.array_equal(L["evict_ranks"], ref.evicted)
            assert st["n_hit_ids"] == ref.hit_ids and st["bytes_h2d"] == len(ref.missed) * D * 4
            assert st["bytes_d2h"] == len(ref.evicted) * D * 4
            sr, rs = o.slot_rank, o.rank_slot
            res = np.nonzero(sr >= 0)[0]
            assert (rs[sr[res]] == res).all() and (rs >= 0).sum() == len(res)
            grad = rng.standard_normal((len(ids), D)).astype(np.float32)
            o.embedding_bag_bwd_sgd(s_o, offs(len(ids)), grad, 0.5)
            acc = np.zeros_like(ref.cuda_weight)
            for i, sl in enumerate(s_ref):
                acc[sl] = acc[sl] + grad[i]
            for sl in np.unique(s_ref):
                ref.cuda_weight[sl] = ref.cuda_weight[sl] - np.float32(0.5) * acc[sl]
            assert np.array_equal(o.cache, ref.cuda_weight) and np.array_equal(ha, hb)
            prev = np.unique(fr[ids])
    # P2 transparency against no-cache training, multi-hot bags with empty bags and repeated ids
    rng = np.random.default_rng(11)
    N, D, C = 50, 4, 9
    fr = rng.permutation(N).astype(np.int32)
    inv = np.argsort(fr)
    W = table_values(3, np.arange(N), D).copy()
    host = W[inv].copy()
    for warm in (True, False):
        Wr = W.copy()
        host = W[inv].copy()
        o = mk(fr, host, C, warm)
        for t in range(25):
            B = 5
            sizes = rng.integers(0, 4, size=B)
            offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
            pool = rng.permutation(N)[:C]
            ids = pool[rng.integers(0, C, size=int(sizes.sum()))].astype(np.int64)
            grad = rng.standard_normal((B, D)).astype(np.float32)
            slots = o.prepare(ids, offsets)
            out = o.embedding_bag_fwd(slots, offsets)
            o.embedding_bag_bwd_sgd(slots, offsets, grad, 0.1)
            ref_out = np.zeros((B, D), np.float32)
            gsum = {}
            for b in range(B):
                for i in range(offsets[b], offsets[b + 1]):
                    ref_out[b] = ref_out[b] + Wr[ids[i]]
                    gsum[int(ids[i])] = gsum.get(int(ids[i]), np.zeros(D, np.float32)) + grad[b]
            assert np.array_equal(out, ref_out)
            for k_, g_ in gsum.items():
                Wr[k_] = Wr[k_] - np.float32(0.1) * g_
        o.flush()
        assert np.array_equal(host, Wr[inv])
    # error paths leave the state alone
    o = mk(fr, W[inv].copy(), C, True)
    sr = o.slot_rank
    for bad_ids, bad_off, name in ((np.arange(C + 1), offs(C + 1), "BATCH_EXCEEDS_CACHE"), (np.array([N]), offs(1), "ID_OUT_OF_RANGE"),
                                   (np.array([1, 2]), np.array([0, 2, 1]), "BAD_OFFSETS")):
        try:
            o.prepare(bad_ids.astype(np.int64), bad_off.astype(np.int64))
            raise AssertionError("no error")
        except OracleError as e:
            assert e.name == name
        assert np.array_equal(sr, o.slot_rank)


MUTANTS = [
    ("evicts the most frequent rows", "if (x->rank != y->rank) return (x->rank < y->rank) - (x->rank > y->rank);",
     "if (x->rank != y->rank) return (x->rank > y->rank) - (x->rank < y->rank);"),
    ("batch rows not protected", "if (k < 0 || contains_sorted(U, nU, k)) continue;", "if (k < 0) continue;"),
    ("look-ahead protection ignored", "if (protect_prev && contains_sorted(o->prev_U, o->n_prev, k)) continue;", ""),
    ("evicts one row too many", "int64_t evict_num = nM - empty;", "int64_t evict_num = nM - empty + 1;"),
    ("evicts against total capacity", "int64_t evict_num = nM - empty;", "int64_t evict_num = nM - C;"),
    ("no write-back", "memcpy(o->host + (size_t)k * D, o->cache + (size_t)s * D, (size_t)D * 4);\n                ++n_written;",
     "++n_written;"),
    ("inverse map not reset on eviction", "            o->rank_slot[k] = -1;\n            o->slot_rank[s] = -1;", "            o->slot_rank[s] = -1;"),
    ("misses take the highest empty slots", "for (int64_t s = 0; s < C && j < nM; ++s) {", "for (int64_t s = C - 1; s >= 0 && j < nM; --s) {"),
    ("missed row not loaded", "memcpy(o->cache + (size_t)s * D, o->host + (size_t)k * D, (size_t)D * 4);\n            o->slot_rank[s] = k;",
     "o->slot_rank[s] = k;"),
    ("hit count per unique row", "for (int64_t i = 0; i < n; ++i) if (o->rank_slot[r[i]] >= 0) ++hit_ids;", "hit_ids = nH;"),
    ("forward drops the last lookup of a bag", "for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {\n            if (i >= n || slots[i] < 0 || slots[i] >= rows) return FCO_INVALID_ARG;\n            const float* row",
     "for (int64_t i = offsets[b]; i < offsets[b + 1] - 1; ++i) {\n            if (i >= n || slots[i] < 0 || slots[i] >= rows) return FCO_INVALID_ARG;\n            const float* row"),
    ("SGD step with the wrong sign", "row[c] = row[c] - step;", "row[c] = row[c] + step;"),
    ("gradient of the wrong bag", "const float* gb = grad_out + (size_t)b * D;", "const float* gb = grad_out + (size_t)(b > 0 ? b - 1 : 0) * D;"),
    ("warm-up in reverse order", "o->slot_rank[s] = (int32_t)s;\n            o->rank_slot[s] = (int32_t)s;\n            memcpy(o->cache + (size_t)s * D, host + (size_t)s * D, (size_t)D * 4);",
     "o->slot_rank[s] = (int32_t)(C - 1 - s);\n            o->rank_slot[C - 1 - s] = (int32_t)s;\n            memcpy(o->cache + (size_t)s * D, host + (size_t)(C - 1 - s) * D, (size_t)D * 4);"),
    ("flush skips a slot", "for (int64_t s = 0; s < o->C; ++s) {\n        int32_t k = o->slot_rank[s];\n        if (k >= 0 &&",
     "for (int64_t s = 1; s < o->C; ++s) {\n        int32_t k = o->slot_rank[s];\n        if (k >= 0 &&"),
    ("bytes counted per float", "o->bytes_h2d = nM * (int64_t)D * 4;", "o->bytes_h2d = nM * (int64_t)D;"),
    ("duplicate ids counted as distinct rows", "if (i == 0 || U[i] != U[i - 1]) U[nU++] = U[i];", "U[nU++] = U[i];"),
    ("dirty tracking: backward does not mark rows", "        o->dirty[s] = 1;\n", ""),
    ("dirty tracking: an evicted slot stays dirty", "            o->dirty[s] = 0;                   /* the slot is empty; whatever is loaded next equals its CPU copy */\n", ""),
    ("dirty tracking: clean rows written, dirty rows dropped", "if (!o->dirty_track || o->dirty[s]) {", "if (!o->dirty_track || !o->dirty[s]) {"),
    ("dirty tracking: bytes still count every victim", "o->bytes_d2h = n_written * (int64_t)D * 4;", "o->bytes_d2h = nV * (int64_t)D * 4;"),
    ("dirty tracking: flush leaves rows dirty", "        o->dirty[s] = 0;                       /* the CPU Weight is current for every resident row now */\n", ""),
    ("dirty tracking: flush writes clean rows only", "if (k >= 0 && (!o->dirty_track || o->dirty[s]))", "if (k >= 0 && (!o->dirty_track || !o->dirty[s]))"),
    ("rank lookup skipped", "for (int64_t i = 0; i < n; ++i) r[i] = o->rank[ids[i]];", "for (int64_t i = 0; i < n; ++i) r[i] = (int32_t)ids[i];"),
]


def build_variant(src_text, tmpdir, name):
    c = os.path.join(tmpdir, name + ".c")
    so = os.path.join(tmpdir, name + ".so")
    open(c, "w").write(src_text)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-ffp-contract=off", "-shared", "-fPIC", c, "-o", so])
    return _load(so)


def test_battery_accepts_the_real_oracle():
    battery(_load())


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(what, old, new):
    src = open(_SRC).read()
    assert src.count(old) == 1, f"mutation site for '{what}' not found exactly once"
    with tempfile.TemporaryDirectory() as d:
        lib = build_variant(src.replace(old, new), d, "mutant")
        try:
            battery(lib)
        except (AssertionError, OracleError, IndexError):
            return
        raise AssertionError(f"the pins did not notice: {what}")
