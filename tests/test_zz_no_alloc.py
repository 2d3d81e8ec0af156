"""`-m gpu`: embedding_bag_bwd_sgd_noalloc (the backward pass for callers that cannot allocate) against the existing
embedding_bag_bwd_sgd, through the C ABI: same kernels, scratch in the library's fixed device array instead of
allocated buffers, so the updated rows must be bit-identical; and against the oracle within the usual tolerance."""
import numpy as np
import pytest

from tests.parity import assert_close, assert_same
from workloads import make_workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,scale", [("c2", 0.1), ("c5", 0.02)])
def test_noalloc_backward_matches_allocating_backward(name, scale):
    import torch
    from oracle import Oracle
    from paper_2208_05321_amd import FreqCache, FreqCacheError
    from paper_2208_05321_amd.binding import NOALLOC_MAX_IDS

    assert torch.cuda.is_available()
    w = make_workload(name, scale=scale, cache_ratio=0.03)
    dev = torch.device("cuda:0")
    a = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, warm=False)
    b = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, warm=False, presort=False)
    for c in (a, b):
        w.host_table(out=c.host_weight())
        c.warm()
    orc = Oracle(w.freq_rank, a.host_weight().copy(), w.cache_rows, warm=True)
    # two calls in a row, the second with a smaller input (the first bags of the next batch only)
    for t, frac in ((0, 1.0), (1, 0.37), (2, 1.0)):
        ids, off = w.batch(t)
        nb = max(1, int((len(off) - 1) * frac))
        off = off[: nb + 1].copy()
        ids = ids[: off[-1]].copy()
        assert len(ids) <= NOALLOC_MAX_IDS
        g = w.grad(t, len(w.batch(t)[1]) - 1)[:nb].copy()
        ids_d, off_d, g_d = torch.from_numpy(ids).to(dev), torch.from_numpy(off).to(dev), torch.from_numpy(g).to(dev)
        so = orc.prepare(ids, off)
        sa = a.prepare(ids_d, off_d)
        sb = b.prepare(ids_d, off_d)
        assert np.array_equal(sa.cpu().numpy(), so) and np.array_equal(sb.cpu().numpy(), so)
        a.embedding_bag_bwd_sgd(sa, off_d, g_d, w.lr)
        b.embedding_bag_bwd_sgd_noalloc(sb, off_d, g_d, w.lr)
        orc.embedding_bag_bwd_sgd(so, off, g, w.lr)
        ra, rb = a.rows(), b.rows()
        assert_same(rb, ra, f"call {t} ({len(ids)} lookups): rows after the no-allocation backward vs the allocating one")
        assert_close(rb, orc.cache, f"call {t}: rows after the no-allocation backward vs the oracle")
    a.check(); b.check()
    # beyond the fixed scratch: refused before anything is touched
    with pytest.raises(FreqCacheError) as e:
        b._check(b._L.embedding_bag_bwd_sgd_noalloc(b._h, sb.data_ptr(), NOALLOC_MAX_IDS + 1, off_d.data_ptr(), 1, g_d.data_ptr(), 0.1), "noalloc")
    assert e.value.name == "SCRATCH_EXCEEDED"
    assert np.array_equal(b.rows(), rb)
    a.close(); b.close(); orc.close()
