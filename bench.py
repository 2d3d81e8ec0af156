#!/usr/bin/env python3
"""Benchmark of the cache step + EmbeddingBag forward/backward on one MI355X.

A step = cache_prepare + embedding_bag_fwd + embedding_bag_bwd_sgd on one batch of synthetic ids.  Default workload:
config 4, the largest configuration that fits one GPU (26 features in one 100M x 128 fp32 table of 51.2 GB in pinned
host memory, batch 65,536 x 26 one-hot ids, cache 1.5%, hot set rotating every 100 batches); `--config c2` etc. select
the others.  Prints ONE JSON line.  The byte model behind `roofline` (what one launch of each kernel has to move) is the `model`
table in profile_pass below.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# HBM bytes per launch from rocprofv3 --pmc (2 x FETCH_SIZE + WRITE_SIZE, scale factors from a plain copy;
# profiles/c2_pmc_fetch_write_size.md, profiles/c4_pmc_fetch_write_size.md); only quoted when the workload is exactly
# the configuration the counters were collected on.
PMC_TRAFFIC = {"c2": {"bwd_reduce": 313.7e6, "bag_fwd": 269.4e6},
               "c4": {"bwd_reduce": 1085.2e6, "bag_fwd": 990.0e6}}
HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published
LINK_PEAK_GBS = 64.0       # PCIe Gen5 x16, per direction, nominal


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def bench_static_module(args, w, torch, dev):
    """Section 4.2 on the GPU: count the ids of `steps` batches, then rank all rows by descending count."""
    from paper_2208_05321_amd import FreqCounter
    ids_d = [torch.from_numpy(w.batch(1000 + t)[0]).to(dev) for t in range(args.warmup + args.steps)]
    fc = FreqCounter(w.num_rows, stream=torch.cuda.current_stream())
    for t in range(args.warmup):
        fc.add(ids_d[t])
    torch.cuda.synchronize()
    a = time.perf_counter()
    for t in range(args.warmup, args.warmup + args.steps):
        fc.add(ids_d[t])
    torch.cuda.synchronize()
    t_count = time.perf_counter() - a
    n_ids = sum(x.numel() for x in ids_d[args.warmup:])
    fc.build()                                   # first call allocates its scratch
    a = time.perf_counter()
    fr, inv, cnt = fc.build(with_counts=True)
    t_build = time.perf_counter() - a
    from oracle import count_ids, freq_rank_from_counts
    a = time.perf_counter()
    counts_o = count_ids([x.cpu().numpy() for x in ids_d], w.num_rows)
    fr_o, inv_o = freq_rank_from_counts(counts_o)
    t_cpu = time.perf_counter() - a
    ok = bool(np.array_equal(cnt, counts_o) and np.array_equal(fr, fr_o))
    # algorithmic bytes of the build: max scan + per radix pass (read key, read pair, write pair) + rank scatter + copies out
    bits = max(1, int(cnt.max()).bit_length())
    passes = -(-bits // 9) if bits <= 18 else -(-bits // 8)      # the library's rule: two passes up to 18 key bits
    build_bytes = w.num_rows * (4 + passes * (4 + 8 + 8) + 8 + 12)
    res = {"metric": "static module on the GPU: ids counted per second; rows ranked per second",
           "value": round(n_ids / t_count, 1), "unit": "ids/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "higher_is_better": True, "dtype": "i32", "data": "synthetic",
           "config": {"workload": f"{w.name}: {w.num_rows} rows, {n_ids // args.steps} ids per batch"},
           "rank_build": {"ms": round(t_build * 1e3, 3), "rows_per_s": round(w.num_rows / t_build, 1), "radix_passes": passes,
                          "alg_bytes": build_bytes, "alg_GBps": round(build_bytes / t_build / 1e9, 1),
                          "includes": "3 device-to-host copies of 4*rows bytes"},
           "cpu_baseline": {"value": round(w.num_rows / t_cpu, 1), "unit": "rows/s (count + rank, numpy oracle)", "cores": 1,
                            "kind": "oracle", "sample": "same ids"},
           "identical_to_oracle": ok}
    fc.close()
    print(json.dumps(res), flush=True)


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c4")
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--cache-ratio", type=float, default=0.015)
    ap.add_argument("--transmitter", choices=("dma", "direct", "staged"), default="dma",
                    help="dma: misses read by kernels from the mapped host table, evicted blocks leave by DMA and are "
                         "scattered by host threads (default); direct: kernels both ways, no host threads; "
                         "staged: the paper's gather / bulk copy / scatter both ways")
    ap.add_argument("--schedule", choices=("pipelined", "plain", "lookahead"), default=None,
                    help="pipelined (default with the dma transmitter): fwd(t), bwd(t), cache_plan_next(t+1), cache_advance - Algorithm 1 as printed, the "
                         "index kernels and the row fetch of batch t+1 run on library streams beside batch t (identical results); "
                         "plain (default with the other transmitters): cache_prepare(t), fwd(t), bwd(t), everything on one stream; "
                         "lookahead: cache_prepare_next(t+1) before fwd(t), bwd(t) - a different cache policy (the previous "
                         "batch's rows are protected too), not the headline configuration")
    ap.add_argument("--miss-path", choices=("kernel", "dma"), default="kernel",
                    help="pipelined schedule: how the planned batch's missing rows cross the link: kernel = read by a kernel from "
                         "the mapped host table (default); dma = gathered by host threads into a pinned block and carried by "
                         "hipMemcpyAsync (FC_MISS_DMA)")
    ap.add_argument("--inputs-ready", choices=("auto", "on", "off"), default="auto",
                    help="FC_INPUTS_READY (the batches are resident before they are handed over, so the planned batch's index "
                         "work need not wait for the caller's stream): 10%% faster at config 4 while HBM binds its step; the library "
                         "itself stops running ahead while the host link binds (configs 2, 3, config 4 after its hot set has rotated), "
                         "where it would cost 7-10%%; auto = on unless the ids come from host memory inside the timed region")
    ap.add_argument("--dirty-tracking", action="store_true",
                    help="FC_DIRTY_TRACK: only victims updated since they were loaded are written back (a variant beyond the "
                         "paper)")
    ap.add_argument("--forward-only", action="store_true",
                    help="no backward pass (inference): a different metric, ids/s through cache prepare + EmbeddingBag forward")
    ap.add_argument("--ids-from-host", action="store_true",
                    help="side measurement, never the headline: every step also uploads its batch's ids and offsets from "
                         "pinned host memory inside the timed region (plain and pipelined schedules)")
    ap.add_argument("--static-module", action="store_true",
                    help="instead of the per-batch path, time the GPU build of the static module (id counting + ranking)")
    ap.add_argument("--staging-rows", type=int, default=0)
    ap.add_argument("--profile-steps", type=int, default=50, help="steps of the per-kernel HIP-event pass (0 = skip)")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="issue one plain device copy of this many MiB first (reference point for rocprofv3 --pmc byte counters)")
    ap.add_argument("--cpu-batches", type=int, default=200, help="most batches of the oracle (CPU baseline) leg (0 = skip)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="the oracle leg stops after the batch that passes this much CPU time")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2208_05321_amd import FreqCache
    from workloads import make_workload

    assert torch.cuda.is_available(), "bench.py needs the GPU; there is no CPU path"
    dev = torch.device("cuda:0")
    t0 = time.time()
    w = make_workload(args.config, scale=args.scale, cache_ratio=args.cache_ratio)
    total_steps = args.warmup + args.steps
    P = max(0, args.profile_steps)
    log(f"[bench] workload {w.name}: rows {w.num_rows} dim {w.dim} cache {w.cache_rows} bags/batch {w.bags_per_batch} "
        f"({time.time() - t0:.1f}s)")

    # a stream of our own (default priority): the library's side stream must not share a hardware queue with it
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)
    if args.static_module:
        return bench_static_module(args, w, torch, dev)

    inputs_ready = args.inputs_ready != "off" and not args.ids_from_host
    cache = FreqCache(w.num_rows, w.dim, w.cache_rows, w.freq_rank, host_weight=None, staging_rows=args.staging_rows,
                      warm=False, staged=args.transmitter == "staged", stream=stream,
                      dma_evict=args.transmitter == "dma", dirty_tracking=args.dirty_tracking, presort=not args.forward_only,
                      inputs_ready=inputs_ready,      
                      miss_dma=args.miss_path == "dma")
    host = cache.host_weight()
    w.host_table(out=host)
    cache.warm()
    log(f"[bench] host table {host.nbytes / 1e9:.2f} GB pinned, filled and warmed ({time.time() - t0:.1f}s)")

    # inputs resident in HBM before the timed region
    ids_d, off_d, n_ids = [], [], []
    for t in range(total_steps + 2 * P + 1):
        ids, offsets = w.batch(t)
        ids_d.append(torch.from_numpy(ids).to(dev))
        off_d.append(torch.from_numpy(offsets).to(dev))
        n_ids.append(len(ids))
    nb = w.bags_per_batch
    grads = [torch.from_numpy(w.grad(k, nb)).to(dev) for k in range(w.grad_pool)]
    max_n = max(n_ids)
    slots = torch.empty(max_n, dtype=torch.int32, device=dev)
    out = torch.empty((nb, w.dim), dtype=torch.float32, device=dev)
    log(f"[bench] {total_steps + 2 * P + 1} batches on device ({time.time() - t0:.1f}s)")
    cache.reserve(max_n, pipelined=True)          # nothing is allocated inside the loop

    if args.calib_copy_mb > 0:
        a = torch.ones(args.calib_copy_mb << 18, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                      # reads and writes exactly calib_copy_mb MiB each
        torch.cuda.synchronize()
        del a, b

    stats = []
    if args.ids_from_host:
        # pinned copies of every batch; three device buffers in rotation (a batch is uploaded two steps ahead of its use
        # in the pipelined schedule, where cache_plan_next reads what was enqueued before the previous cache_advance)
        ids_h = [x.cpu().pin_memory() for x in ids_d]
        off_h = [x.cpu().pin_memory() for x in off_d]
        ring = [(torch.empty(max_n, dtype=torch.int64, device=dev), torch.empty(nb + 1, dtype=torch.int64, device=dev)) for _ in range(3)]

        def upload(t):
            if t >= len(ids_h):
                return
            bi, bo = ring[t % 3]
            bi[: n_ids[t]].copy_(ids_h[t], non_blocking=True)
            bo.copy_(off_h[t], non_blocking=True)
            ids_d[t], off_d[t] = bi[: n_ids[t]], bo
    else:
        def upload(t):
            pass
    slots2 = [slots, torch.empty(max_n, dtype=torch.int32, device=dev)]
    fallbacks = [0]

    def step_plain(t):
        s = slots[: n_ids[t]]
        upload(t)
        cache.prepare(ids_d[t], off_d[t], out=s)
        stats.append(cache.stats())
        cache.embedding_bag_fwd(s, off_d[t], out=out)
        if not args.forward_only:
            cache.embedding_bag_bwd_sgd(s, off_d[t], grads[t % len(grads)], w.lr)

    def step_lookahead(t):
        # batch t was prepared by the previous step (or just below for the very first one)
        from paper_2208_05321_amd import FreqCacheError
        cur = slots2[t & 1][: n_ids[t]]
        if t == 0:
            cache.prepare(ids_d[0], off_d[0], out=cur)
            stats.append(cache.stats())
        nxt = slots2[(t + 1) & 1][: n_ids[t + 1]]
        refused = False
        try:
            cache.prepare_next(ids_d[t + 1], off_d[t + 1], out=nxt)
            stats.append(cache.stats())
        except FreqCacheError as e:
            if e.name != "BATCH_EXCEEDS_CACHE":
                raise
            refused = True
        cache.embedding_bag_fwd(cur, off_d[t], out=out)
        if not args.forward_only:
            cache.embedding_bag_bwd_sgd(cur, off_d[t], grads[t % len(grads)], w.lr)
        cache.advance()
        if refused:
            fallbacks[0] += 1
            cache.prepare(ids_d[t + 1], off_d[t + 1], out=nxt)
            stats.append(cache.stats())

    def step_planned(t):
        # same policy and results as step_plain; the index half of batch t+1's prepare is issued before batch t's
        # forward / backward and runs beside them on the library's stream, its rows move at cache_advance
        cur = slots2[t & 1][: n_ids[t]]
        if t == 0:
            upload(0); upload(1)
            cache.prepare(ids_d[0], off_d[0], out=cur)
            stats.append(cache.stats())
        nxt = slots2[(t + 1) & 1][: n_ids[t + 1]]
        upload(t + 2)
        cache.embedding_bag_fwd(cur, off_d[t], out=out)           # enqueued first: they wait on the GPU for batch t's rows
        if not args.forward_only:
            cache.embedding_bag_bwd_sgd(cur, off_d[t], grads[t % len(grads)], w.lr)
        cache.plan_next(ids_d[t + 1], off_d[t + 1], out=nxt)      # index kernels and row fetch of batch t+1 run beside all that
        if not args.dirty_tracking:
            stats.append(cache.stats())
        cache.advance()
        if args.dirty_tracking:
            stats.append(cache.stats())                           # bytes written back are known after the rows moved

    if args.schedule is None:
        args.schedule = "pipelined" if args.transmitter == "dma" else "plain"
    if args.schedule == "pipelined" and args.transmitter == "staged":
        args.schedule = "plain"          # cache_plan_next is not available with the staged transmitter
    pipelined, lookahead = args.schedule == "pipelined", args.schedule == "lookahead"
    step = step_lookahead if lookahead else (step_planned if pipelined else step_plain)

    # no collector pause inside the timed region (the loop allocates a few small Python objects per step)
    gc.collect()
    gc.disable()
    for t in range(args.warmup):
        step(t)
    torch.cuda.synchronize()
    cache.check()                        # nothing of the warm-up is still on its way (host scatter threads included)
    marks = [0.0] * (args.steps + 1)
    t_start = marks[0] = time.perf_counter()
    for t in range(args.warmup, total_steps):
        step(t)
        marks[t - args.warmup + 1] = time.perf_counter()
    torch.cuda.synchronize()
    t_sync = time.perf_counter()
    cache.check()                        # the clock stops once every evicted row of the timed steps is in the host table
    elapsed = time.perf_counter() - t_start
    gc.enable()
    # where the host spent the timed region (diagnostic: a stall of the host loop shows up as one long interval)
    host_steps = [(b - a) * 1e3 for a, b in zip(marks, marks[1:])]
    host_loop = {"max_ms": round(max(host_steps), 3), "median_ms": round(sorted(host_steps)[len(host_steps) // 2], 3),
                 "drain_ms": round((t_sync - marks[-1]) * 1e3, 3), "check_ms": round((t_start + elapsed - t_sync) * 1e3, 3)}
    # one entry per prepared batch; the pipelined schedules have prepared one batch beyond the last timed step
    timed = stats[args.warmup:total_steps]
    assert len(timed) == args.steps
    tot_ids = sum(n_ids[args.warmup:total_steps])
    hit_ratio = sum(s["n_hit_ids"] for s in timed) / max(1, tot_ids)
    uniq_hit_ratio = sum(s["n_hit_unique"] for s in timed) / max(1, sum(s["n_unique"] for s in timed))
    warm_in = stats[:args.warmup]
    warm_in_hit = sum(s["n_hit_ids"] for s in warm_in) / max(1, sum(s["n_ids"] for s in warm_in))
    value = tot_ids / elapsed
    ms_per_step = elapsed / args.steps * 1e3
    # workloads whose hot set moves (config 4): hit ratio of the timed steps before and after every rotation they cross
    phases = None
    if w.drift_every:
        phases = []
        for ph in sorted({t // w.drift_every for t in range(args.warmup, total_steps)}):
            sel = [stats[t] for t in range(args.warmup, total_steps) if t // w.drift_every == ph]
            hs = [host_steps[t - args.warmup] for t in range(args.warmup, total_steps) if t // w.drift_every == ph]
            phases.append({"host_ms_per_step": round(float(np.mean(hs)), 4),     # the host loop is paced by the GPU (it waits for every planning kernel)
                           "batches": [ph * w.drift_every if ph * w.drift_every > args.warmup else args.warmup,
                                       min((ph + 1) * w.drift_every, total_steps) - 1],
                           "rotations_so_far": ph,
                           "hit_ratio": round(sum(x["n_hit_ids"] for x in sel) / max(1, sum(x["n_ids"] for x in sel)), 5),
                           "miss_per_step": round(float(np.mean([x["n_miss"] for x in sel])), 1)})
    mean = {k: float(np.mean([s[k] for s in timed])) for k in ("n_ids", "n_unique", "n_miss", "n_evict")}
    log(f"[bench] {args.steps} steps in {elapsed:.4f}s: {value / 1e6:.1f} M ids/s, {ms_per_step:.3f} ms/step, "
        f"hit ratio {hit_ratio:.4f}, per batch unique {mean['n_unique']:.0f} miss {mean['n_miss']:.0f}")
    if phases and len(phases) > 1:
        log("[bench] by phase: " + "; ".join(f"batches {p['batches'][0]}-{p['batches'][1]}: {p['host_ms_per_step']:.3f} ms/step, hit ratio {p['hit_ratio']:.4f}, "
                                             f"{p['miss_per_step']:.0f} misses" for p in phases))
    log(f"[bench] host loop per step: median {host_loop['median_ms']} ms, max {host_loop['max_ms']} ms; drain {host_loop['drain_ms']} ms, "
        f"check {host_loop['check_ms']} ms")

    # ---- per-kernel pass: HIP events on the library's own streams ----
    kernels = {}
    roofline = None
    host_link = None
    if args.profile_steps > 0:
        R = w.dim * 4
        nw = -(-w.num_rows // 32)

        def profile_pass(step_fn, first):
            """P further batches of the same trace, each kernel / copy bracketed by HIP events on its own stream."""
            cache.profile(True)
            pstats = []
            for t in range(first, first + P):
                step_fn(t)
                pstats.append(stats[-1])
            rep = cache.profile_report()
            cache.profile(False)
            n_m = float(np.mean([s["n_ids"] for s in pstats]))
            u_m = float(np.mean([s["n_unique"] for s in pstats]))
            m_m = float(np.mean([s["n_miss"] for s in pstats]))
            e_m = float(np.mean([s["n_evict"] for s in pstats]))
            # algorithmic bytes per launch: what the step must move whatever the implementation (R = bytes per row)
            model = {
                "remap_mark": n_m * (8 + 4 + 4 + 4) + (nb + 1) * 8,            # id, idx_map entry, resident bit word, rank out
                "rank_count": nw * 4 * 2,
                "rank_emit": nw * 4 * 2 + m_m * 4 + e_m * (8 + 4 + 4),
                "evict_gather": e_m * (2 * R + 4),
                "evict_store": e_m * (2 * R + 4),
                "free_count": w.cache_rows * 4, "free_assign": w.cache_rows * 4 + m_m * 16,
                "miss_fill": m_m * (2 * R + 8),
                "rows_in": m_m * (2 * R + 4),
                "slots_out": n_m * 12,
                # forward: every DISTINCT row once (a row looked up again is served by the caches), slots, offsets, outputs
                "bag_fwd": u_m * R + n_m * 4 + nb * (R + 8),
                # backward: sorted pairs, every gradient row once, every distinct row read and written
                "bwd_reduce": n_m * 8 + nb * R + 2 * u_m * R,
                "sort_hist": n_m * 4, "sort_scatter": n_m * 16,
            }
            ks = {}
            for name, r in rep.items():
                avg_us = r["ms"] / r["launches"] * 1e3
                launches_per_step = r["launches"] / P
                k = {"avg_us": round(avg_us, 2), "launches_per_step": round(launches_per_step, 2),
                     "us_per_step": round(avg_us * launches_per_step, 2)}
                if name in model:
                    per_launch = model[name] / max(launches_per_step, 1e-9)
                    k["alg_bytes_per_launch"] = int(per_launch)
                    k["alg_GBps"] = round(per_launch / (avg_us * 1e-6) / 1e9, 1)
                ks[name] = k
            step_bytes = sum(model[name] for name in model if name in ks)       # all launches of a step together
            return ks, m_m, e_m, step_bytes

        kernels, m_m, e_m, step_bytes = profile_pass(step, total_steps)
        # HBM-bound kernels on the caller's stream (the sort runs on the auxiliary stream under the miss fill, where
        # its event-bracketed time says more about the fill than about the sort)
        # candidates: the kernels that stream rows through HBM; the index kernels are bound by latency, and beside a
        # copy kernel (as under a tracer) they can wait longer than any of these run
        hbm_kernels = [k for k in ("bag_fwd", "bwd_reduce", "evict_gather", "rows_in") if k in kernels and "alg_GBps" in kernels[k]]
        if pipelined:
            # In the pipelined schedule this kernel shares compute units with the host-link row fetch of the next batch
            # (its waves wait on host reads).  Two more measurements of the same kernels on the same data:
            # "serial": a pass in the plain schedule (one stream; the DMA copy of the evicted block still runs beside the
            # forward / backward kernels), and "alone": forward and backward launched again and again on the last batch
            # with a device synchronisation in between, nothing else on the GPU.
            serial, _, _, _ = profile_pass(step_plain, total_steps + P)
            for name, k in serial.items():
                if name in kernels:
                    kernels[name]["serial_avg_us"] = k["avg_us"]
            t_last = total_steps + 2 * P - 1
            s_last = slots[: n_ids[t_last]]
            torch.cuda.synchronize()
            cache.profile(True)
            for rep in range(12):
                cache.embedding_bag_fwd(s_last, off_d[t_last], out=out)
                torch.cuda.synchronize()
                if not args.forward_only:
                    cache.embedding_bag_bwd_sgd(s_last, off_d[t_last], grads[rep % len(grads)], w.lr)
                    torch.cuda.synchronize()
            rep_alone = cache.profile_report()
            cache.profile(False)
            for name in ("bag_fwd", "bwd_reduce", "bwd_fixup"):
                if name in rep_alone and name in kernels:
                    kernels[name]["alone_avg_us"] = round(rep_alone[name]["ms"] / rep_alone[name]["launches"] * 1e3, 2)
        # the one that takes longest per step on the caller's stream (the critical path) in the timed schedule
        dom = max(hbm_kernels, key=lambda k: kernels[k]["avg_us"] * kernels[k]["launches_per_step"])
        ach = kernels[dom]["alg_GBps"]
        roofline = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4),
                    "traffic": PMC_TRAFFIC.get(w.name, {}).get(dom) if (args.scale == 1.0 and args.cache_ratio == 0.015) else None,
                    "alg_bytes_per_launch": kernels[dom]["alg_bytes_per_launch"], "avg_us": kernels[dom]["avg_us"],
                    "measured": "HIP events around every launch, in the timed schedule (%s)" % args.schedule}
        if "alone_avg_us" in kernels[dom]:
            gbs = kernels[dom]["alg_bytes_per_launch"] / (kernels[dom]["alone_avg_us"] * 1e-6) / 1e9
            roofline["alone"] = {"avg_us": kernels[dom]["alone_avg_us"], "achieved": round(gbs, 1),
                                 "frac": round(gbs / HBM_PEAK_GBS, 4),
                                 "measured": "HIP events, the kernel relaunched on the last batch with nothing else running "
                                             "(a best case: that batch's rows are still warm in the caches)"}
        if "serial_avg_us" in kernels[dom]:
            gbs = kernels[dom]["alg_bytes_per_launch"] / (kernels[dom]["serial_avg_us"] * 1e-6) / 1e9
            roofline["serial"] = {"avg_us": kernels[dom]["serial_avg_us"], "achieved": round(gbs, 1),
                                  "frac": round(gbs / HBM_PEAK_GBS, 4),
                                  "measured": "HIP events, plain schedule (only the DMA copy of the evicted block beside it)"}
        # which roofline binds the whole step: the time the step's HBM bytes need at the HBM peak against the time its
        # link bytes (the larger direction; the link is full duplex) need at the link's nominal rate
        t_hbm = step_bytes / (HBM_PEAK_GBS * 1e9)
        t_link = max(m_m, e_m) * R / (LINK_PEAK_GBS * 1e9)
        roofline["step"] = {"hbm_bytes": int(step_bytes), "hbm_frac": round(t_hbm / (ms_per_step * 1e-3), 4),
                            "link_bytes_each_way": int(max(m_m, e_m) * R), "link_frac": round(t_link / (ms_per_step * 1e-3), 4),
                            "binding": "host_link" if t_link > t_hbm else "hbm",
                            "note": "fractions of the timed step that its bytes would need at the HBM peak (8 TB/s) and at the "
                                    "link's nominal rate (64 GB/s per direction); the larger one names the roofline that binds the step"}
        roofline["model"] = ("bytes that must move per launch: every distinct row once (rows looked up again are served by the "
                             "caches), every pooled output / gradient row once, the index arrays once")
        link = {}
        for name, direction, rows in (("miss_fill", "h2d", m_m), ("evict_store", "d2h", e_m),
                                      ("h2d_block", "h2d", m_m), ("d2h_block", "d2h", e_m)):
            if name in kernels and rows > 0:
                k = kernels[name]
                gbs = rows * R / max(k["launches_per_step"], 1e-9) / (k["avg_us"] * 1e-6) / 1e9
                link[name] = {"direction": direction, "achieved": round(gbs, 1), "peak": LINK_PEAK_GBS, "unit": "GB/s",
                              "frac": round(gbs / LINK_PEAK_GBS, 4), "bytes_per_step": int(rows * R),
                              "us_per_step": k["us_per_step"]}
        host_link = link
        for name in sorted(kernels, key=lambda k: -kernels[k]["us_per_step"]):
            log(f"[bench]   {name:14s} {kernels[name]}")

    # ---- CPU baseline: the oracle as it stands, one core, a bounded sample of the same trace ----
    cpu_baseline = None
    if args.cpu_batches > 0:
        from oracle import Oracle
        S = min(args.cpu_batches, total_steps)
        host_o = np.empty_like(host)
        w.host_table(out=host_o)
        orc = Oracle(w.freq_rank, host_o, w.cache_rows, warm=True, dirty_tracking=args.dirty_tracking)
        gpool = [w.grad(k, nb).copy() for k in range(w.grad_pool)]
        t_cpu = 0.0
        same = True
        done = ids_done = 0
        for t in range(S):
            if t_cpu >= args.cpu_seconds:
                break
            ids, offsets = w.batch(t)
            done, ids_done = done + 1, ids_done + len(ids)
            a = time.perf_counter()
            so = orc.prepare(ids, offsets)
            orc.embedding_bag_fwd(so, offsets)
            if not args.forward_only:
                orc.embedding_bag_bwd_sgd(so, offsets, gpool[t % len(gpool)], w.lr)
            t_cpu += time.perf_counter() - a
            same &= lookahead or orc.stats() == stats[t]
        S = done
        cpu_baseline = {"value": round(ids_done / t_cpu, 1), "unit": "ids/s", "cores": 1,
                        "kind": "oracle", "sample": f"first {S} batches of the same trace (prepare+fwd+bwd, warm start), {t_cpu:.1f} s of CPU time",
                        "host_cores_available": os.cpu_count(), "cpu_model": cpu_model(),
                        "gpu_stats_identical_on_sample": bool(same)}
        log(f"[bench] oracle: {cpu_baseline['value'] / 1e6:.2f} M ids/s on 1 core over {S} batches; stats identical: {same}")
        orc.close()

    result = {
        "metric": "ids/sec through cache prepare + EmbeddingBag fwd/bwd at 1.5% cache" if not args.forward_only else
                  "ids/sec through cache prepare + EmbeddingBag fwd (no backward pass) at 1.5% cache",
        "value": round(value, 1), "unit": "ids/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.num_features} features in one {w.num_rows} x {w.dim} fp32 table, "
                               f"batch {w.samples} x {w.num_features} {'multi-hot' if w.multi_hot else 'one-hot'} ids, "
                               f"Zipf({w.alpha}), cache {w.cache_rows} rows ({args.cache_ratio:.3%}), SGD lr {w.lr}",
                   "schedule": "fwd(t), bwd(t) | cache_plan_next(t+1): index + early row fetch on library streams | cache_advance" if pipelined else
                               ("cache_prepare_next(t+1) | fwd(t), bwd(t) | cache_advance" if lookahead else "cache_prepare(t), fwd(t), bwd(t)"),
                   "policy": "look-ahead (previous batch protected), %d refused" % fallbacks[0] if lookahead else
                             ("Algorithm 1, clean victims not written back" if args.dirty_tracking else "Algorithm 1 as printed"),
                   "transmitter": {"dma": ("kernel miss fill" if args.miss_path == "kernel" else "DMA miss path (host gather threads + hipMemcpyAsync)") +
                                          " + DMA evict with %s host scatter threads" % os.environ.get("FC_SCATTER_THREADS", "8"),
                                   "direct": "kernels both ways", "staged": "block transmitter both ways"}[args.transmitter],
                   "inputs_ready": bool(inputs_ready),
                   "ids_per_step": int(mean["n_ids"]), "unique_per_step": round(mean["n_unique"], 1),
                   "miss_per_step": round(mean["n_miss"], 1), "evict_per_step": round(mean["n_evict"], 1)},
        "ids_from_host": bool(args.ids_from_host),
        "hit_ratio": round(hit_ratio, 5), "unique_hit_ratio": round(uniq_hit_ratio, 5), "hit_ratio_by_phase": phases, "host_loop": host_loop,
        "warm_in": {"batches": args.warmup, "hit_ratio": round(warm_in_hit, 5), "timed": False},
        "roofline": roofline, "host_link": host_link, "kernels": kernels, "cpu_baseline": cpu_baseline,
    }
    cache.close()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
