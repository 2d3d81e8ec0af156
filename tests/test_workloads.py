"""The seeded input generators (workloads/): shapes, determinism, numpy == native fill."""
import numpy as np

from workloads import make_workload, table_values, fill_host_table, zipf_positions, log_uniform_cardinalities


def test_table_values_native_matches_numpy_and_range():
    ids = np.array([0, 1, 5, 99999, 2**31 - 1], dtype=np.int32)
    out = np.empty((5, 24), dtype=np.float32)
    fill_host_table(out, 3, ids)
    ref = table_values(3, ids, 24)
    assert np.array_equal(out, ref)
    assert (np.abs(ref) < 0.05).all() and ref.std() > 0.02


def test_zipf_positions_bounds_and_skew():
    rng = np.random.default_rng(0)
    k = zipf_positions(rng.random(200000), 1000, 1.05)
    assert k.min() == 1 and k.max() <= 1000
    c = np.bincount(k, minlength=1001)[1:]
    assert c[0] > c[9] > c[99] > 0
    # P(1) = (1 - 2^(1-a)) / (1 - (K+1)^(1-a))
    p1 = (1 - 2 ** -0.05) / (1 - 1001 ** -0.05)
    assert abs(c[0] / 200000 - p1) < 0.01


def test_cardinalities_sum_exactly():
    for total in (2600, 100000, 10_000_000):
        c = log_uniform_cardinalities(26, total, 10, total // 5, 1)
        assert c.sum() == total and (c >= 1).all()


def test_workloads_are_deterministic_and_well_formed():
    for name in ("c1", "c2", "c3", "c4", "c5", "c5u", "avz", "c2d32"):
        a = make_workload(name, scale=0.002)
        b = make_workload(name, scale=0.002)
        assert np.array_equal(np.sort(a.freq_rank), np.arange(a.num_rows))       # a permutation
        assert np.array_equal(a.freq_rank[a.inv_rank], np.arange(a.num_rows))
        assert np.array_equal(a.freq_rank, b.freq_rank)
        for t in (0, 3):
            ia, oa = a.batch(t)
            ib, ob = b.batch(t)
            assert np.array_equal(ia, ib) and np.array_equal(oa, ob)
            assert ia.min() >= 0 and ia.max() < a.num_rows
            assert oa[0] == 0 and oa[-1] == len(ia) and (np.diff(oa) >= 0).all()
            assert len(oa) - 1 == a.bags_per_batch
        assert not np.array_equal(a.batch(0)[0], a.batch(1)[0])
        g = a.grad(1, a.bags_per_batch)
        assert g.shape == (a.bags_per_batch, a.dim) and g.dtype == np.float32


def test_host_table_is_rank_ordered():
    w = make_workload("c2", scale=0.002)
    T = w.host_table()
    ids = np.array([0, 17, w.num_rows - 1])
    assert np.array_equal(T[w.freq_rank[ids]], table_values(w.seed, ids, w.dim))


def test_analytic_rank_follows_popularity():
    w = make_workload("c1")
    ids = np.concatenate([w.batch(t)[0] for t in range(50)])
    counts = np.bincount(ids, minlength=w.num_rows)
    top = np.argsort(-counts, kind="stable")[:20]
    assert (w.freq_rank[top] < 60).all()


def test_drift_rotates_hot_set():
    w = make_workload("c4", scale=0.001)
    r0 = w.freq_rank[w.batch(0)[0]]
    r1 = w.freq_rank[w.batch(100)[0]]
    assert np.median(r1) > np.median(r0)
