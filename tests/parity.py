"""GPU-vs-oracle parity harness (used by the `-m gpu` tests and by __graft_entry__.smoke).

Both sides get the same seeded inputs from workloads/.  Index decisions (slots, hit / miss / victim lists,
slot assignment, both maps, byte counts) and the pooled outputs of the forward pass are compared bit-for-bit;
cached rows after the SGD step and the flushed host table within RTOL (see assert_close).
"""
from __future__ import annotations

import numpy as np

# Pooled outputs: both sides add a bag's rows one by one in position order in fp32, so they are compared bit for bit
# (assert_same).
#
# Updated rows: the task's bar is 1e-5 relative in fp32.  The only arithmetic difference between the two sides is the
# association order of the backward pass's gradient sum (the GPU adds fixed blocks of consecutive lookups, then
# the blocks; the oracle adds one by one), so an element differs by a few ulp OF THE PARTIAL SUMS, not of the result:
# a weight that cancels to nearly zero is off by the same absolute amount as its large neighbours, and a row that
# received K gradient terms carries a rounding error that grows with K on both sides (about u * K * |term| for a
# sequential fp32 sum of K terms of similar size, u = 2^-24).  Two bounds are asserted:
#   row-wise      |gpu[r, c] - oracle[r, c]| <= RTOL * max_c(|gpu[r, :]|, |oracle[r, :]|) + ATOL       for every element;
#   element-wise  |gpu[r, c] - oracle[r, c]| <= RTOL * |oracle[r, c]| + TERM_ULPS * u * K[r] * term_scale
#                 where K[r] is the number of gradient terms row r has received so far and term_scale = lr * max|grad|
#                 (callers that track K pass `terms`): a row never trained on, or trained by single lookups, has to
#                 agree to 1e-5 of each element (in fact it agrees bit for bit); the allowance only opens with K.
# Reported, not asserted (it fails for sound reasons on rows with thousands of terms): the largest relative error
# among elements of at least ELEM_FLOOR of their row's largest magnitude.  `worst` keeps the largest error / bound
# ratios seen in a process; the tests print them.
RTOL = 1e-5
ATOL = 1e-9
ELEM_FLOOR = 1e-2
TERM_ULPS = 4.0
U32 = 2.0 ** -24
worst = {"rowwise": 0.0, "elementwise_bound": 0.0, "elementwise_rel_at_floor": 0.0}

STAT_FIELDS = ("n_ids", "n_unique", "n_hit_unique", "n_hit_ids", "n_miss", "n_evict", "bytes_h2d", "bytes_d2h")


def assert_same(a, b, what):
    """Bit-for-bit equality of two fp32 arrays (signed zeros compare equal)."""
    a = np.asarray(a)
    b = np.asarray(b)
    assert a.shape == b.shape, f"{what}: shape {a.shape} vs {b.shape}"
    if np.array_equal(a, b):
        return
    bad = np.argwhere(a != b)
    i = tuple(bad[0])
    raise AssertionError(f"{what}: {len(bad)} elements differ, first at {i}: gpu {a[i]!r} oracle {b[i]!r}")


def assert_close(a, b, what, terms=None, term_scale=0.0, chunk=1 << 16):
    """terms: per row, the number of gradient terms it has received (enables the element-wise bound above)."""
    a = np.asarray(a)
    b = np.asarray(b)
    assert a.shape == b.shape and a.ndim == 2, f"{what}: shape {a.shape} vs {b.shape}"
    for r0 in range(0, a.shape[0], chunk):
        x, y = a[r0:r0 + chunk], b[r0:r0 + chunk]
        if np.array_equal(x, y):
            continue
        err = np.abs(x.astype(np.float64) - y.astype(np.float64))
        scale = np.maximum(np.abs(x).max(axis=1), np.abs(y).max(axis=1)).astype(np.float64)
        lim = (ATOL + RTOL * scale)[:, None]
        ratio = err / lim
        worst["rowwise"] = max(worst["rowwise"], float(ratio.max()))
        if not (err <= lim).all():
            r, c = np.unravel_index(int(np.argmax(ratio)), err.shape)
            raise AssertionError(f"{what}: row {r0 + r} col {c}: |diff| {err[r, c]:.3e} > limit {lim[r, 0]:.3e} "
                                 f"(gpu {x[r, c]!r}, oracle {y[r, c]!r}, row scale {scale[r]:.3e}); "
                                 f"{int((err > lim).sum())} elements over the limit")
        ay = np.abs(y).astype(np.float64)
        big = (ay >= ELEM_FLOOR * scale[:, None]) & (ay > 0)
        if big.any():
            worst["elementwise_rel_at_floor"] = max(worst["elementwise_rel_at_floor"], float((err[big] / ay[big]).max()) / RTOL)
        if terms is not None:
            k = np.asarray(terms[r0:r0 + chunk], dtype=np.float64)
            elim = RTOL * ay + (TERM_ULPS * U32 * term_scale) * k[:, None] + 1e-30
            eratio = err / elim
            worst["elementwise_bound"] = max(worst["elementwise_bound"], float(eratio.max()))
            if eratio.max() > 1.0:
                r, c = np.unravel_index(int(np.argmax(eratio)), err.shape)
                raise AssertionError(f"{what}: row {r0 + r} col {c}: |diff| {err[r, c]:.3e} > element-wise limit {elim[r, c]:.3e} "
                                     f"(gpu {x[r, c]!r}, oracle {y[r, c]!r}, {int(k[r])} gradient terms so far); "
                                     f"{int((eratio > 1).sum())} elements over the limit")


class TermCount:
    """Number of gradient terms every row of the table (by frequency rank) has received so far, and the largest
    lr * |gradient element| seen: what the element-wise bound of assert_close needs."""

    def __init__(self, w):
        self.freq_rank = w.freq_rank
        self.by_rank = np.zeros(w.num_rows, dtype=np.int32)
        self.term_scale = 0.0

    def add(self, ids, grad, lr):
        np.add.at(self.by_rank, self.freq_rank[ids], 1)
        self.term_scale = max(self.term_scale, float(lr) * float(np.abs(grad).max()))

    def of_slots(self, slot_rank):
        return np.where(slot_rank >= 0, self.by_rank[np.maximum(slot_rank, 0)], 0)


def report_worst(log=print):
    log(f"  worst error / bound so far: row-wise {worst['rowwise']:.3f}, element-wise (with the per-row term allowance) "
        f"{worst['elementwise_bound']:.3f}; largest plain relative error among elements >= {ELEM_FLOOR:g} of their row's "
        f"maximum: {worst['elementwise_rel_at_floor'] * RTOL:.2e}")


def compare_prepare(gpu, orc, slots_gpu, slots_orc, t, deep=True):
    sg, so = gpu.stats(), orc.stats()
    for f in STAT_FIELDS:
        assert sg[f] == so[f], f"batch {t}: stat {f}: gpu {sg[f]} oracle {so[f]}"
    assert np.array_equal(slots_gpu, slots_orc), f"batch {t}: slots differ"
    lg, lo = gpu.last_lists(), orc.last_lists()
    assert np.array_equal(lg["miss_ranks"], lo["miss_ranks"]), f"batch {t}: miss set"
    assert np.array_equal(lg["fill_slots"], lo["fill_slots"]), f"batch {t}: slot assignment of misses"
    og, oo = np.argsort(lg["evict_ranks"], kind="stable"), np.argsort(lo["evict_ranks"], kind="stable")
    assert np.array_equal(lg["evict_ranks"][og], lo["evict_ranks"][oo]), f"batch {t}: evicted ids"
    assert np.array_equal(lg["evict_slots"][og], lo["evict_slots"][oo]), f"batch {t}: evicted slots"
    if deep:
        sr, rs = gpu.state()
        assert np.array_equal(sr, orc.slot_rank), f"batch {t}: slot->rank map"
        assert np.array_equal(rs, orc.rank_slot), f"batch {t}: rank->slot map"


def check_forward(gpu, out_d, slots_np, offsets, out_o, what, rows_before=None, same_weights=False):
    """Pooled output of the GPU against the oracle.  The forward pass adds a bag's rows in position order on both sides:
    given the same weights the results are bit-identical.  same_weights: the two sides' cached rows are known to be
    bit-identical (no backward pass yet, or exact gradient sums) -> compared bit for bit with the oracle's output.
    rows_before: the GPU's cached rows as they were when the forward ran -> the oracle's bag sum over THOSE rows must
    equal the GPU's output bit for bit (whatever rounding the earlier backward passes left in them).  Always: within
    tolerance of the oracle's output."""
    from oracle import bag_sum
    out_np = out_d.cpu().numpy()
    if same_weights:
        assert_same(out_np, out_o, what + " (bit-exact)")
    if rows_before is not None:
        assert_same(out_np, bag_sum(rows_before, slots_np, offsets), what + " (bit-exact on the GPU's own rows)")
    assert_close(out_np, out_o, what)
    return out_np


def run_parity(w, batches, warm=True, staged=False, staging_rows=0, deep_every=1, values_every=1, log=None,
               dma_evict=False, dirty_tracking=False, forward_only=lambda t: False, flush_at=(), exact_values=False,
               fwd_exact_every=1):
    """Drive the GPU library and the oracle over batches of workload `w`: the first `batches` ones, or the batch numbers
    listed in `batches` (Workload.batch(t) is a pure function of t, so a run can jump to the batches of interest).
    forward_only(t): no backward pass after batch t (matters with dirty_tracking: its rows stay clean);
    flush_at: batches after which both sides flush;
    exact_values: gradient sums are exact in fp32 (config 1: all-ones gradients), so cached rows, pooled outputs and the
    flushed table are compared bit for bit;
    fwd_exact_every: on every k-th compared batch the GPU's pooled output is also checked bit for bit against the
    oracle's bag sum over a copy of the GPU's own cached rows (0 = never)."""
    import torch
    from oracle import Oracle
    from paper_2208_05321_amd import FreqCache

    order = list(range(batches)) if isinstance(batches, int) else list(batches)
    dev = torch.device("cuda:0")
    gpu = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, host_weight=None, staging_rows=staging_rows,
                    warm=False, staged=staged, dma_evict=dma_evict, dirty_tracking=dirty_tracking)
    host_gpu = gpu.host_weight()
    w.host_table(out=host_gpu)
    host_orc = host_gpu.copy()
    if warm:
        gpu.warm()
    orc = Oracle(w.freq_rank, host_orc, w.cache_rows, warm=warm, dirty_tracking=dirty_tracking)
    tot = {"ids": 0, "hit_ids": 0, "miss": 0, "evict": 0, "bytes_d2h": 0, "miss_of": {}}
    terms = TermCount(w)
    if exact_values:
        close = lambda a, b, what, by_slot: assert_same(a, b, what)
    else:
        close = lambda a, b, what, by_slot: assert_close(a, b, what, terms=terms.of_slots(orc.slot_rank) if by_slot else terms.by_rank,
                                                         term_scale=terms.term_scale)
    trained = False
    for k, t in enumerate(order):
        last = k == len(order) - 1
        ids, offsets = w.batch(t)
        nb = len(offsets) - 1
        grad = w.grad(t, nb)
        ids_d = torch.from_numpy(ids).to(dev)
        off_d = torch.from_numpy(offsets).to(dev)
        grad_d = torch.from_numpy(grad).to(dev)
        slots_o = orc.prepare(ids, offsets)
        slots_d = gpu.prepare(ids_d, off_d)
        deep = deep_every and (k % deep_every == 0 or last)
        slots_np = slots_d.cpu().numpy()
        compare_prepare(gpu, orc, slots_np, slots_o, t, deep=bool(deep))
        rows_before = gpu.rows() if fwd_exact_every and (k % fwd_exact_every == 0 or last) else None
        out_d = gpu.embedding_bag_fwd(slots_d, off_d)
        out_o = orc.embedding_bag_fwd(slots_o, offsets)
        check_forward(gpu, out_d, slots_np, offsets, out_o, f"batch {t}: pooled output", rows_before,
                      same_weights=exact_values or not trained)
        del rows_before
        if not forward_only(t):
            gpu.embedding_bag_bwd_sgd(slots_d, off_d, grad_d, w.lr)
            orc.embedding_bag_bwd_sgd(slots_o, offsets, grad, w.lr)
            terms.add(ids, grad, w.lr)
            trained = True
        if values_every and (k % values_every == 0 or last):
            close(gpu.rows(), orc.cache, f"batch {t}: cached rows after SGD", True)
        if t in flush_at:
            gpu.flush()
            orc.flush()
            close(host_gpu, host_orc, f"batch {t}: host table after a flush in mid-run", False)
        s = orc.stats()
        tot["ids"] += s["n_ids"]; tot["hit_ids"] += s["n_hit_ids"]; tot["miss"] += s["n_miss"]; tot["evict"] += s["n_evict"]
        tot["bytes_d2h"] += s["bytes_d2h"]
        tot["miss_of"][t] = s["n_miss"]
        if log:
            log(f"  batch {t}: n={s['n_ids']} unique={s['n_unique']} hit_ids={s['n_hit_ids']} miss={s['n_miss']} evict={s['n_evict']} ok")
    gpu.check()
    gpu.flush()
    orc.flush()
    close(host_gpu, host_orc, "host table after flush", False)
    sr, rs = gpu.state()
    assert np.array_equal(sr, orc.slot_rank) and np.array_equal(rs, orc.rank_slot)
    gpu.close()
    orc.close()
    return tot


def run_parity_lookahead(w, num_batches, warm=True, dma_evict=True, staging_rows=0, deep_every=1, log=None,
                         free_running=False, dirty_tracking=False, forward_only=lambda t: False):
    """The look-ahead schedule on both sides: batch t+1 is prepared (protecting batch t's rows) before batch t's
    forward / backward run.  When the two batches do not fit together both sides must refuse, and the batch is then
    prepared the plain way after the backward pass.
    free_running: no device synchronisation inside the loop (the look-ahead stream really runs beside the caller's
    stream); slots and pooled outputs are kept and compared after the loop."""
    import torch
    from oracle import Oracle, OracleError
    from paper_2208_05321_amd import FreqCache, FreqCacheError

    dev = torch.device("cuda:0")
    gpu = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, host_weight=None, staging_rows=staging_rows,
                    warm=False, dma_evict=dma_evict, dirty_tracking=dirty_tracking)
    host_gpu = gpu.host_weight()
    w.host_table(out=host_gpu)
    host_orc = host_gpu.copy()
    if warm:
        gpu.warm()
    orc = Oracle(w.freq_rank, host_orc, w.cache_rows, warm=warm, dirty_tracking=dirty_tracking)
    data = []
    for t in range(num_batches):
        ids, offsets = w.batch(t)
        grad = w.grad(t, len(offsets) - 1)
        data.append((ids, offsets, grad, torch.from_numpy(ids).to(dev), torch.from_numpy(offsets).to(dev),
                     torch.from_numpy(grad).to(dev)))
    torch.cuda.synchronize()
    so = orc.prepare(data[0][0], data[0][1])
    sd = gpu.prepare(data[0][3], data[0][4])
    compare_prepare(gpu, orc, sd.cpu().numpy(), so, 0)
    tot = {"lookahead": 0, "fallback": 0, "ids": 0, "hit_ids": orc.stats()["n_hit_ids"], "evict": 0, "bytes_d2h": 0}
    later = []
    for t in range(num_batches):
        ids, offsets, grad, ids_d, off_d, grad_d = data[t]
        so_next = sd_next = None
        refused = False
        if t + 1 < num_batches:
            nids, noff, _, nids_d, noff_d, _ = data[t + 1]
            try:
                so_next = orc.prepare(nids, noff, lookahead=True)
            except OracleError as e:
                assert e.name == "BATCH_EXCEEDS_CACHE"
                refused = True
            try:
                sd_next = gpu.prepare_next(nids_d, noff_d)
                assert not refused, f"batch {t + 1}: oracle refused the look-ahead, GPU accepted it"
            except FreqCacheError as e:
                assert e.name == "BATCH_EXCEEDS_CACHE" and refused, f"batch {t + 1}: GPU refused ({e.name}), oracle did not"
            if not refused:
                if free_running:
                    assert gpu.stats() == orc.stats(), f"batch {t + 1}: stats"
                    later.append((f"batch {t + 1}: slots", sd_next, so_next))
                else:
                    deep = deep_every and ((t + 1) % deep_every == 0 or t + 2 == num_batches)
                    compare_prepare(gpu, orc, sd_next.cpu().numpy(), so_next, t + 1, deep=bool(deep))
                tot["lookahead"] += 1
        out_d = gpu.embedding_bag_fwd(sd, off_d)
        out_o = orc.embedding_bag_fwd(so, offsets)
        if free_running:
            later.append((f"batch {t}: pooled output", out_d, out_o))
        else:
            assert_close(out_d.cpu().numpy(), out_o, f"batch {t}: pooled output")
        if not forward_only(t):
            gpu.embedding_bag_bwd_sgd(sd, off_d, grad_d, w.lr)
            orc.embedding_bag_bwd_sgd(so, offsets, grad, w.lr)
        gpu.advance()
        if refused:
            so_next = orc.prepare(nids, noff)
            sd_next = gpu.prepare(nids_d, noff_d)
            compare_prepare(gpu, orc, sd_next.cpu().numpy(), so_next, t + 1)
            tot["fallback"] += 1
        if t + 1 < num_batches:
            s = orc.stats()
            tot["hit_ids"] += s["n_hit_ids"]; tot["evict"] += s["n_evict"]; tot["bytes_d2h"] += s["bytes_d2h"]
        tot["ids"] += len(ids)
        if log:
            log(f"  batch {t} ok ({'refused, plain prepare' if refused else 'look-ahead'})")
        so, sd = so_next, sd_next
    for what, a, b in later:
        if a.dtype == torch.int32:
            assert np.array_equal(a.cpu().numpy(), b), what
        else:
            assert_close(a.cpu().numpy(), b, what)
    assert_close(gpu.rows(), orc.cache, "cached rows at the end")
    gpu.check()
    gpu.flush()
    orc.flush()
    assert_close(host_gpu, host_orc, "host table after flush")
    sr, rs = gpu.state()
    assert np.array_equal(sr, orc.slot_rank) and np.array_equal(rs, orc.rank_slot)
    gpu.close()
    orc.close()
    return tot


def run_parity_planned(w, batches, warm=True, dma_evict=True, staging_rows=0, free_running=False, plan_first=False,
                       dirty_tracking=False, forward_only=lambda t: False, log=None, inputs_ready=False, miss_dma=False,
                       ahead_miss_pct=100.0):
    """cache_plan_next: the index half of the next batch's prepare runs beside the current batch's forward / backward,
    rows move at cache_advance.  Same policy as plain cache_prepare, so the oracle is simply driven in program order.
    batches: a count (the first ones) or a list of batch numbers, as for run_parity.
    ahead_miss_pct: with inputs_ready the library runs ahead of the caller's stream while the previous batch's miss
    share is below this (FC_AHEAD_MISS_PCT); 100 = always (the small test workloads miss far more than the library's
    default of 2 in 100), None = the library's default, "median" = the median share of these very batches, so that
    about every other batch runs ahead and the two modes keep alternating."""
    import os
    import torch
    from oracle import Oracle
    from paper_2208_05321_amd import FreqCache

    dev = torch.device("cuda:0")
    if ahead_miss_pct == "median":
        probe = Oracle(w.freq_rank, w.host_table(), w.cache_rows, warm=warm)
        shares = []
        for t in (range(batches) if isinstance(batches, int) else batches):
            ids, offsets = w.batch(t)
            probe.prepare(ids, offsets)
            shares.append(100.0 * probe.stats()["n_miss"] / max(1.0, 0.5 * (len(ids) + len(offsets) - 1)))
        probe.close()
        ahead_miss_pct = float(np.median(shares[1:] or shares))
        if log:
            log(f"  miss shares {min(shares):.2f}..{max(shares):.2f} per 100, threshold {ahead_miss_pct:.2f}")
    saved = os.environ.get("FC_AHEAD_MISS_PCT")
    if ahead_miss_pct is not None:
        os.environ["FC_AHEAD_MISS_PCT"] = repr(float(ahead_miss_pct))
    try:                                             # the knob is read by cache_create
        gpu = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, host_weight=None, staging_rows=staging_rows,
                        warm=False, dma_evict=dma_evict, dirty_tracking=dirty_tracking, inputs_ready=inputs_ready, miss_dma=miss_dma)
    finally:
        if saved is None:
            os.environ.pop("FC_AHEAD_MISS_PCT", None)
        else:
            os.environ["FC_AHEAD_MISS_PCT"] = saved
    host_gpu = gpu.host_weight()
    w.host_table(out=host_gpu)
    host_orc = host_gpu.copy()
    if warm:
        gpu.warm()
    orc = Oracle(w.freq_rank, host_orc, w.cache_rows, warm=warm, dirty_tracking=dirty_tracking)
    order = list(range(batches)) if isinstance(batches, int) else list(batches)
    num_batches = len(order)
    data = []
    for t in order:
        ids, offsets = w.batch(t)
        grad = w.grad(t, len(offsets) - 1)
        data.append((ids, offsets, grad, torch.from_numpy(ids).to(dev), torch.from_numpy(offsets).to(dev),
                     torch.from_numpy(grad).to(dev)))
    torch.cuda.synchronize()
    so = orc.prepare(data[0][0], data[0][1])
    sd = gpu.prepare(data[0][3], data[0][4])
    compare_prepare(gpu, orc, sd.cpu().numpy(), so, order[0])
    later = []
    bytes_d2h = 0
    trained = False
    terms = TermCount(w)
    for t in range(num_batches):                  # t: position in `order` from here on
        ids, offsets, grad, ids_d, off_d, grad_d = data[t]
        rows_before = None if free_running else gpu.rows()
        def plan():
            nxt = gpu.plan_next(data[t + 1][3], data[t + 1][4]) if t + 1 < num_batches else None
            return nxt, gpu.stats(), (None if free_running or nxt is None else gpu.last_lists())
        if plan_first:          # both call orders are legal
            sd_next, gstats, glists = plan()
        out_d = gpu.embedding_bag_fwd(sd, off_d)
        if not forward_only(t):
            gpu.embedding_bag_bwd_sgd(sd, off_d, grad_d, w.lr)
        if not plan_first:
            sd_next, gstats, glists = plan()
        gpu.advance()
        if dirty_tracking and sd_next is not None:
            gstats = gpu.stats()             # the bytes written back are known once the rows have moved
        out_o = orc.embedding_bag_fwd(so, offsets)
        if not forward_only(t):
            orc.embedding_bag_bwd_sgd(so, offsets, grad, w.lr)
            terms.add(ids, grad, w.lr)
        if free_running:
            later.append((f"batch {order[t]}: pooled output", out_d, out_o, not trained))
        else:
            check_forward(gpu, out_d, sd.cpu().numpy(), offsets, out_o, f"batch {order[t]}: pooled output", rows_before,
                          same_weights=not trained)
        del rows_before
        trained = trained or not forward_only(t)
        if log:
            log(f"  batch {order[t]}: {orc.stats()} ok")
        if sd_next is not None:
            so_next = orc.prepare(data[t + 1][0], data[t + 1][1])
            assert gstats == orc.stats(), f"batch {t + 1}: stats {gstats} vs {orc.stats()}"
            bytes_d2h += gstats["bytes_d2h"]
            if free_running:
                later.append((f"batch {order[t + 1]}: slots", sd_next, so_next, True))
            else:
                lo = orc.last_lists()
                assert np.array_equal(glists["miss_ranks"], lo["miss_ranks"]) and np.array_equal(glists["fill_slots"], lo["fill_slots"])
                assert np.array_equal(np.sort(glists["evict_ranks"]), np.sort(lo["evict_ranks"]))
                compare_prepare(gpu, orc, sd_next.cpu().numpy(), so_next, t + 1)
                assert_close(gpu.rows(), orc.cache, f"batch {order[t + 1]}: cached rows after the rows moved",
                             terms=terms.of_slots(orc.slot_rank), term_scale=terms.term_scale)
            so, sd = so_next, sd_next
    for what, a, b, exact in later:
        if a.dtype == torch.int32:
            assert np.array_equal(a.cpu().numpy(), b), what
        else:
            if exact:
                assert_same(a.cpu().numpy(), b, what + " (bit-exact)")
            assert_close(a.cpu().numpy(), b, what)
    assert_close(gpu.rows(), orc.cache, "cached rows at the end", terms=terms.of_slots(orc.slot_rank), term_scale=terms.term_scale)
    gpu.check()
    gpu.flush()
    orc.flush()
    assert_close(host_gpu, host_orc, "host table after flush", terms=terms.by_rank, term_scale=terms.term_scale)
    sr, rs = gpu.state()
    assert np.array_equal(sr, orc.slot_rank) and np.array_equal(rs, orc.rank_slot)
    gpu.close()
    orc.close()
    return {"bytes_d2h": bytes_d2h}
