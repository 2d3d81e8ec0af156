/* freqcache -- C ABI of the MI355X (gfx950) frequency-aware software cache for large
 * embedding tables, after arXiv:2208.05321 ("A Frequency-aware Software Cache for Large
 * Recommendation System Embeddings").
 *
 * The library keeps the whole embedding table in pinned host memory, re-ordered by
 * descending id frequency ("CPU Weight", paper Section 4.2), and `cache_rows` of its rows
 * in HBM ("CUDA Cached Weight", Section 4.3).  Once per training iteration the caller
 * turns the batch's ids into row indices of the cached weight (Algorithm 1,
 * PrepareCache), runs the EmbeddingBag-sum forward on the cached rows and applies the
 * sparse SGD update to them (Section 4.3, last step of the workflow; synchronous
 * updates, Section 2.2).  Every step runs in hand-written HIP kernels, on the caller's
 * stream unless stated otherwise: three library-owned streams carry the write-back of
 * evicted rows, the sort the backward pass needs, and -- with cache_plan_next or
 * cache_prepare_next -- the next batch's index work and row fetch beside the current batch.
 *
 * Conventions
 *   - every function returns FC_OK (0) or a negative FC_ERR_* code; nothing throws or aborts;
 *   - pointers named *_dev are device pointers owned by the caller (e.g. PyTorch tensors),
 *     pointers named *_host are ordinary host pointers owned by the caller;
 *   - one handle = one table = one GPU (the device current at cache_create); a handle is
 *     not thread-safe and calls on one handle must not overlap;
 *   - ids are already offset into the single concatenated table (Section 5.1);
 *   - int32 row indices internally: num_rows < 2^31 - 2^16, n < 2^31 - 2^16.
 *
 * There is no CPU fallback: if no HIP device is usable the calls fail with FC_ERR_HIP.
 */
#ifndef FREQCACHE_H
#define FREQCACHE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fc_cache fc_cache; /* opaque, owned by the library */

/* Observables of the most recent successful cache_prepare (Algorithm 1). */
typedef struct fc_stats {
    int64_t n_ids;        /* ids in the batch                                            */
    int64_t n_unique;     /* distinct rows the batch touches (|unique(idx_map[ids])|)    */
    int64_t n_hit_unique; /* of those, already resident                                  */
    int64_t n_hit_ids;    /* ids whose row was already resident (access-level hits)      */
    int64_t n_miss;       /* rows moved host -> HBM                                      */
    int64_t n_evict;      /* rows evicted (all written to the host table unless FC_DIRTY_TRACK) */
    int64_t bytes_h2d;    /* n_miss  * dim * 4                                           */
    int64_t bytes_d2h;    /* n_evict * dim * 4 (FC_DIRTY_TRACK: dirty victims * dim * 4)  */
} fc_stats;

enum {
    FC_OK = 0,
    FC_ERR_INVALID_ARG = -1,
    FC_ERR_ID_OUT_OF_RANGE = -2,     /* an id outside [0, num_rows)                               */
    FC_ERR_BAD_OFFSETS = -3,         /* offsets[0] != 0, offsets[num_bags] != n, or not monotone  */
    FC_ERR_BATCH_EXCEEDS_CACHE = -4, /* more distinct rows in the batch than cache_rows           */
    FC_ERR_NOT_PERMUTATION = -5,     /* freq_rank is not a permutation of [0, num_rows)           */
    FC_ERR_OOM_DEVICE = -6,
    FC_ERR_OOM_PINNED = -7,
    FC_ERR_HIP = -8,                 /* a HIP runtime call failed, or no usable device            */
    FC_ERR_NOT_PINNED = -9,          /* host_weight given but not page-locked, GPU-mapped memory  */
    FC_ERR_BAD_SLOT = -10,           /* a slot index outside [0, cache_rows) reached fwd / bwd     */
    FC_ERR_SCRATCH_EXCEEDED = -11,   /* embedding_bag_bwd_sgd_noalloc: the batch needs more than its fixed scratch */
    FC_ERR_COUNT_OVERFLOW = -12      /* freq_add: more than 2^31 - 1 ids in all would overflow the 32-bit counters */
};

/* Limits of embedding_bag_bwd_sgd_noalloc (below). */
#define FC_NOALLOC_MAX_IDS 524288                 /* lookups per call                                     */
#define FC_NOALLOC_SCRATCH_BYTES (20 * 1048576)   /* size of the library's fixed scratch array, per GPU   */

/* cache_create flags */
enum {
    FC_WARM = 1,            /* preload the cache_rows highest-frequency rows (Section 4.3, "cache warm-up") */
    FC_TRANSMIT_STAGED = 2, /* move rows the way the paper's data transmitter does (Section 4.3):
                               gather into a contiguous block on the source side, one bulk
                               hipMemcpyAsync over the host link, scatter on the target side.
                               Default (flag clear): kernels read / write the mapped pinned table
                               directly, one row-group of lanes per row.  Results are identical. */
    FC_EVICT_DMA = 4,       /* evicted rows only: the block leaves HBM by hipMemcpyAsync on the side stream (DMA
                               engine, full duplex with the miss fill, no compute units involved) and library-owned
                               host threads scatter it into the host table in the background (block transmitter of
                               Section 4.3 for the device -> host direction).  Misses are still read by kernels.
                               The host table is complete after cache_flush (or cache_check).  Number of threads:
                               environment variable FC_SCATTER_THREADS (default 8).  Not with FC_TRANSMIT_STAGED.
                               Results are identical. */
    FC_NO_PRESORT = 8,      /* By default cache_prepare also starts, on a library-owned stream, the sort of the
                               batch's (slot, bag) pairs that embedding_bag_bwd_sgd needs, so that it overlaps the
                               miss fill; it reads slots_dev and offsets_dev until it is done.  Set this flag when
                               no backward pass follows (inference) or those buffers are reused at once. */
    FC_INPUTS_READY = 32,   /* A promise about cache_plan_next's inputs: ids_dev / offsets_dev are complete when the call is made
                               (resident batches, or uploads the caller has waited for), not merely enqueued on the caller's
                               stream.  The library then starts the index work of the planned batch without waiting for the
                               caller's stream at all (only the slot write-out and the sort still wait for the backward pass
                               that last read those buffers), which puts the planned batch's index decisions and row fetch a
                               whole step ahead of cache_advance, and lets the sort's later passes run on the stream of the
                               evicted-row block instead of holding up the next batch's index kernels.  That pays where HBM
                               binds the step (large batches, high hit ratio); where the host link binds it, the extra overlap
                               slows the link transfers down, so the library runs ahead only while the previous batch missed
                               at most FC_AHEAD_MISS_PCT (default 2) rows per 100 of (lookups + bags) / 2, the point where
                               the link's bytes take as long as HBM's.  Results are unchanged.  Ignored with FC_DIRTY_TRACK. */
    FC_MISS_DMA = 64,       /* cache_plan_next only, with FC_EVICT_DMA or the default transmitter: the planned batch's missing rows
                               cross the link the way the paper's transmitter moves them (Section 4.3), pipelined: their list
                               is copied to the host, library-owned host threads (FC_GATHER_THREADS, default 6) gather the
                               rows from the host table into a pinned block chunk by chunk, and each chunk goes into the
                               arrival block in HBM by hipMemcpyAsync (DMA engine) on the fetch stream; no compute unit reads
                               host memory.  cache_advance waits on the host until the last chunk has been handed over.
                               Memory: two more pinned blocks of staging_rows * dim * 4 bytes.  Results are identical.
                               Ignored with FC_DIRTY_TRACK. */
    FC_DIRTY_TRACK = 16     /* Variant beyond the paper (Algorithm 1 always calls move_to_cpu): a resident row is
                               dirty once embedding_bag_bwd_sgd has updated it since it was loaded; only dirty
                               victims are written back, clean ones are dropped (their copy in the host table is
                               current), and cache_flush writes dirty rows only.  bytes_d2h counts the rows written.
                               Every other result is unchanged.  The call that moves the rows (cache_prepare,
                               cache_prepare_next, or cache_advance after cache_plan_next: what is dirty is only
                               known after the current batch's backward pass) then waits on the host once more, for
                               the number of dirty victims; after cache_plan_next, bytes_d2h of cache_last_stats is
                               final only once cache_advance has returned. */
};

/* Static module + dynamic module set-up (Sections 4.2, 4.3).
 *   num_rows, dim   table shape; fp32; 1 <= dim <= 1024.
 *   cache_rows      rows of the cached weight, 0 < cache_rows <= num_rows (the paper's cache ratio
 *                   times num_rows; 1.5% by default there).
 *   freq_rank_host  "idx_map": id -> row of the frequency-ordered table (0 = most frequent).
 *                   Host pointer, length num_rows, must be a permutation; copied.
 *   host_weight     the frequency-ordered table, num_rows*dim fp32, row r = embedding of the id with
 *                   rank r.  Either NULL -- the library allocates pinned memory, the caller fills it
 *                   through cache_host_weight() BEFORE the first cache_prepare (and before
 *                   cache_create's warm-up if FC_WARM is wanted: then create cold, fill, and call
 *                   cache_warm) -- or a pointer to page-locked, GPU-mapped memory
 *                   (hipHostMalloc / a pinned torch tensor) that outlives the handle.  The table is
 *                   the store of record: evictions and cache_flush write into it.
 *   staging_rows    bound, in rows, of the transmitter's block buffers (Section 4.3 keeps the transmitter's
 *                   memory footprint bounded); larger transfers are
 *                   done in several rounds.  0 = default (min(cache_rows, 524288)).  Memory, in blocks of
 *                   staging_rows * dim * 4 bytes: one in HBM by default; with FC_TRANSMIT_STAGED two in
 *                   HBM and one pinned; with FC_EVICT_DMA four in HBM and four pinned; cache_plan_next
 *                   adds two in HBM on first use.
 *   flags           any of FC_WARM, FC_TRANSMIT_STAGED, FC_EVICT_DMA, FC_NO_PRESORT, FC_DIRTY_TRACK, FC_INPUTS_READY, FC_MISS_DMA.
 *   hip_stream      hipStream_t on which all per-batch work is enqueued (NULL = default stream).
 *   out             receives the handle.
 * Errors: INVALID_ARG, NOT_PERMUTATION, NOT_PINNED, OOM_DEVICE, OOM_PINNED, HIP.  Synchronous (it also runs a few
 * sub-millisecond test kernels on hip_stream to find library streams that run beside it).
 * Tuning knobs, read from the environment at this call (defaults suit an MI355X on a PCIe Gen5 x16 link):
 *   FC_FILL_BLOCKS        workgroups of the miss fill (40 with FC_EVICT_DMA, else 1024)
 *   FC_FILL_BLOCKS_EARLY  workgroups of cache_plan_next's early row fetch, fixed (default: starts at 32 and follows the
 *                         measured fetch / block-copy durations); FC_FILL_BLOCKS_EARLY_START only moves the start
 *   FC_EVICT_BLOCKS, FC_EVICT_EARLY   width and start of the host-table store kernel (transmitter without FC_EVICT_DMA)
 *   FC_SCATTER_THREADS    host threads of FC_EVICT_DMA (8)
 *   FC_GATHER_THREADS     host threads of FC_MISS_DMA (6)
 *   FC_AHEAD_MISS_PCT     threshold of FC_INPUTS_READY (see there); 0 = never run ahead, 100 = always
 *   FC_SORT_TAIL          0: with FC_INPUTS_READY the whole sort stays on the index stream (default 1: passes after the first
 *                         on the side stream)
 *   FC_FWD_SORTED         0: batches with one lookup per bag are always pooled in bag order (default 1: in slot order, from
 *                         the pairs cache_prepare has sorted ahead of time for the backward pass, when those are at hand)
 *   FC_FWD_BAGS           bags per row-group of the bag-order forward kernel for one-lookup bags: 1, 2 or 4 (4)
 *   FC_SORT_BITS          most key bits per pass of the backward's sort (4..11; default: two passes of up to 9 bits up to 18 key
 *                         bits, beyond that passes of up to 9 bits without a scan kernel); FC_SORT_FUSED=0 keeps the scan kernel
 *   FC_FETCH_CU_MASK      experiment: number of compute units the early fetch's stream may use (default: all)
 *   FC_MARK_IPT           ids per thread of the marking kernel (2)
 *   FC_TUNE_REPORT        if set, cache_destroy prints where the early-fetch workgroup count settled
 *   FC_TIMELINE           file that receives, whenever profiling totals are collected, one line "name start_us end_us"
 *                         per timed kernel or copy (read at every collection, not here) */
int cache_create(int64_t num_rows, int32_t dim, int64_t cache_rows, const int32_t* freq_rank_host,
                 float* host_weight, int64_t staging_rows, int32_t flags, void* hip_stream, fc_cache** out);

/* Allocate now everything the per-batch calls would otherwise allocate when they first meet a batch of that size:
 * the per-id rank buffer of cache_prepare, the sort scratch and partial-sum rows of embedding_bag_bwd_sgd for batches
 * of up to max_ids lookups (three sort sets of 16 * max_ids bytes), and, if pipelined != 0, the two arrival blocks of
 * cache_plan_next (staging_rows * dim * 4 bytes each).  The transmitter's memory stays bounded by staging_rows
 * (Section 4.3); this call only moves the allocations out of the training loop.  Optional: without it (or for a larger
 * batch later) the buffers grow on demand, which costs a hipMalloc and a device-wide synchronisation in that step.
 * Synchronous.  Errors: INVALID_ARG, OOM_DEVICE, HIP. */
int cache_reserve(fc_cache* c, int64_t max_ids, int32_t pipelined);

/* Cache warm-up (Section 4.3): empty the cache and load rows 0..cache_rows-1 of the host table into
 * slots 0..cache_rows-1.  cache_create(FC_WARM) calls this.  Synchronous.  Does not write back
 * resident rows first (call cache_flush if they carry updates). */
int cache_warm(fc_cache* c);

/* Algorithm 1 (PrepareCache + PrepareCPURowIdxOnGPU): make every row the batch needs resident and
 * return, per input id, its row index in the cached weight.
 *   ids_dev      int64[n], device.           offsets_dev  int64[num_bags+1], device, bag b = ids
 *   slots_dev    int32[n], device, output.                [offsets[b], offsets[b+1]) (EmbeddingBag).
 * Steps, all on the GPU: ids -> frequency rank; distinct ranks; split into resident / missing; if the
 * missing rows outnumber the empty slots, evict that many resident rows not used by this batch,
 * largest rank (least frequent) first, writing them back to the host table; assign the i-th smallest
 * missing rank to the i-th smallest empty slot and load it from the host table.
 * On return the index decisions are final and the error code is known (the call waits for the
 * planning kernels, a few microseconds of GPU work); row movement and the slot write-out are enqueued
 * on the stream, so later work on the same stream sees every needed row resident.
 * Errors: INVALID_ARG, BAD_OFFSETS, ID_OUT_OF_RANGE, BATCH_EXCEEDS_CACHE (in this order of precedence),
 * OOM_DEVICE, HIP.  On any error the cache state is unchanged and slots_dev is unspecified. */
int cache_prepare(fc_cache* c, const int64_t* ids_dev, int64_t n, const int64_t* offsets_dev, int64_t num_bags,
                  int32_t* slots_dev);

/* Look-ahead (the paper's Future Work section proposes prefetching on the ids of coming batches): Algorithm 1 for the
 * NEXT batch, issued while the batch of the latest cache_prepare / cache_prepare_next is still being trained on.
 * Same arguments, results and errors as cache_prepare, with two differences:
 *   - the rows of that previous batch are protected from eviction as well (the backlist of Algorithm 1 is the union
 *     of both batches), so the forward / backward calls of the previous batch may be enqueued after this call; if too
 *     few evictable rows remain the call fails with FC_ERR_BATCH_EXCEEDS_CACHE and changes nothing (the caller then
 *     finishes the current batch and uses cache_prepare);
 *   - the work is enqueued on a library-owned stream and overlaps the caller's stream; ids_dev / offsets_dev must be
 *     complete on the caller's stream at the time of the call and stay untouched until cache_advance.
 * Usage:  cache_prepare(batch 0);  loop { cache_prepare_next(batch t+1, slots_next); fwd(t); bwd(t); cache_advance(); } */
int cache_prepare_next(fc_cache* c, const int64_t* ids_dev, int64_t n, const int64_t* offsets_dev, int64_t num_bags,
                       int32_t* slots_dev);
/* Software pipelining WITHOUT a change of policy: the index half of cache_prepare for the NEXT batch (ids -> ranks,
 * unique rows, misses, victims, slot assignment, the slots of the batch, the sort for its backward pass), enqueued on
 * a library-owned stream beside whatever the caller's stream still runs for the current batch: the arrival of its
 * missing rows, its forward and its backward pass.  None of these decisions depends on embedding values, so the
 * results (slots, statistics, lists, maps) are exactly those of cache_prepare called after the current batch's
 * backward pass.  No row is moved: cache_advance does that, on the caller's stream, i.e. after the backward pass the
 * caller enqueued in between.
 * Same arguments and errors as cache_prepare; not available with FC_TRANSMIT_STAGED.
 * Ordering (without FC_INPUTS_READY): the index work is ordered behind the caller's stream as of the ENTRY of the latest
 * cache_prepare / cache_advance call, not as of this call.  ids_dev / offsets_dev must therefore be complete by then (written by work
 * enqueued on the caller's stream before that call, or finished altogether) and stay untouched until cache_advance;
 * slots_dev must not be the buffer the current batch's forward / backward read.  cache_copy_rows / cache_host_weight
 * reflect the planned batch only after cache_advance.
 * Usage:  cache_prepare(batch 0);  loop { fwd(t); bwd(t); cache_plan_next(batch t+1, slots_next); cache_advance(); }
 * (forward / backward are asynchronous and best enqueued first, since this call waits on the host for its planning
 * kernels; those do not wait for them.  Calling it before them is equally correct.)
 * The call also starts fetching the planned batch's missing rows, on another library-owned stream, into a block in
 * device memory (allocated on first use, staging_rows rows per list set); cache_advance then writes the evicted
 * rows out and copies the fetched rows into their slots. */
int cache_plan_next(fc_cache* c, const int64_t* ids_dev, int64_t n, const int64_t* offsets_dev, int64_t num_bags,
                    int32_t* slots_dev);
/* Makes the batch of the latest cache_prepare_next / cache_plan_next the current one (for cache_plan_next this is
 * where its evicted rows leave and its missing rows arrive): work enqueued on the caller's stream after this
 * call sees its rows resident and its slots written.  Asynchronous (a stream-to-stream dependency). */
int cache_advance(fc_cache* c);

/* EmbeddingBag, mode "sum", on the cached weight (Section 4.3: the framework's embedding op runs on the
 * cached weight after the cache step):  out[b, :] = sum_{i in bag b} cached_weight[slots[i], :], summed
 * in position order; an empty bag gives zeros.
 *   slots_dev int32[n] as returned by the latest cache_prepare; out_dev fp32[num_bags*dim], device.
 * Asynchronous on the stream.  A slot outside [0, cache_rows) contributes nothing and raises a sticky
 * FC_ERR_BAD_SLOT reported by cache_check. */
int embedding_bag_fwd(fc_cache* c, const int32_t* slots_dev, int64_t n, const int64_t* offsets_dev,
                      int64_t num_bags, float* out_dev);

/* Backward of the sum-bag fused with the SGD step (synchronous update, Section 2.2): for every distinct
 * slot s, g = sum over the lookups i with slots[i] == s of grad_out[bag(i), :] (a row looked up k times
 * receives k gradients), then cached_weight[s, :] -= lr * g.  Deterministic: no floating-point atomics;
 * lookups of a slot are summed in position order within fixed blocks of consecutive lookups.
 *   grad_out_dev fp32[num_bags*dim], device.  Asynchronous on the stream; BAD_SLOT as above. */
int embedding_bag_bwd_sgd(fc_cache* c, const int32_t* slots_dev, int64_t n, const int64_t* offsets_dev,
                          int64_t num_bags, const float* grad_out_dev, float lr);

/* embedding_bag_bwd_sgd for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * or training loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results, but the
 * call allocates nothing (no hipMalloc / hipFree, no event creation): the sort buffers, radix histograms and partial
 * rows it needs live in a fixed array of FC_NOALLOC_SCRATCH_BYTES bytes of device memory that is part of the library's
 * code object (every GPU the library runs on holds one copy until the process ends; cache_create looks its address up).
 * Limits: n <= FC_NOALLOC_MAX_IDS lookups, and 10.5 MB + blocks * (16 + 8 * dim) bytes <= FC_NOALLOC_SCRATCH_BYTES, where
 * blocks = ceil(n / 256) for dim <= 128 and ceil(n * lanes / 8192) with lanes = min(64, dim / 4) for wider rows (dim 256:
 * n <= 524288; dim 1024: n <= 150000 or so); beyond them the call returns FC_ERR_SCRATCH_EXCEEDED and does nothing.
 * It never uses a sort started ahead of time by cache_prepare (create the handle with FC_NO_PRESORT to spare that work)
 * and is not covered by cache_profile_*.  All calls on one GPU, from any handle, share the one array: calls that overlap
 * on a GPU (two handles on different streams) race; the array keeps the previous call's contents, none of which the
 * next call reads before writing.  Errors: INVALID_ARG, SCRATCH_EXCEEDED, HIP; BAD_SLOT as embedding_bag_bwd_sgd. */
int embedding_bag_bwd_sgd_noalloc(fc_cache* c, const int32_t* slots_dev, int64_t n, const int64_t* offsets_dev,
                                  int64_t num_bags, const float* grad_out_dev, float lr);

/* Write every resident row back to the host table (the host table is the store of record, Section 3);
 * residency is unchanged.  Returns after the host table is complete. */
int cache_flush(fc_cache* c);

/* Wait for all enqueued work of this handle and return the sticky asynchronous error, if any
 * (then clears it). */
int cache_check(fc_cache* c);

/* Waits for outstanding work, frees everything the library allocated.  Does NOT flush. */
int cache_destroy(fc_cache* c);

/* ---- introspection (parity checks, reports) ---- */
int cache_last_stats(const fc_cache* c, fc_stats* out);
/* Copies of the two index maps (paper's cache_idx_map in both directions): slot_rank_host int32[cache_rows]
 * (-1 = empty slot), rank_slot_host int32[num_rows] (-1 = not resident); either may be NULL. Synchronous. */
int cache_copy_state(fc_cache* c, int32_t* slot_rank_host, int32_t* rank_slot_host);
/* Lists of the latest cache_prepare, each may be NULL: missing ranks (ascending, n_miss), evicted ranks
 * (ascending, n_evict) with the slots they left, and fill_slots[j] = slot that received miss_ranks[j]. */
int cache_last_lists(fc_cache* c, int32_t* miss_ranks_host, int32_t* evict_ranks_host, int32_t* evict_slots_host,
                     int32_t* fill_slots_host);
/* Copy of the cached weight, fp32[cache_rows*dim]. Synchronous. */
int cache_copy_rows(fc_cache* c, float* rows_host);
/* The pinned, frequency-ordered host table (library- or caller-allocated). */
float* cache_host_weight(fc_cache* c);
const char* cache_strerror(int code);

/* ---- static module (Section 4.2): id frequency statistics -> freq_rank, built on the GPU ---- */
typedef struct fc_freq fc_freq; /* opaque accumulator of per-id occurrence counts */

/* Zeroed counters for ids in [0, num_rows) on the current device; work is enqueued on hip_stream. */
int freq_create(int64_t num_rows, void* hip_stream, fc_freq** out);
/* counts[id] += 1 for each of the n ids (int64, device memory): one scan step over the dataset, or over a sample of
 * it when the dataset is too large (Section 4.2).  Asynchronous; ids outside [0, num_rows) are skipped and make
 * freq_build fail with FC_ERR_ID_OUT_OF_RANGE.  The counters are 32 bits wide: once the ids of all calls together would
 * exceed 2^31 - 1 the call returns FC_ERR_COUNT_OVERFLOW and counts nothing (sample the dataset instead). */
int freq_add(fc_freq* f, const int64_t* ids_dev, int64_t n);
/* Order the rows from high to low occurrence count, equal counts by lower id:
 *   freq_rank_host[id] = position of id in that order (the idx_map cache_create takes), int32[num_rows];
 *   inv_rank_host[r]   = id at position r, int32[num_rows];   counts_host[id] = its count.  Each may be NULL.
 * Synchronous; the counters stay valid (more freq_add / freq_build calls may follow). */
int freq_build(fc_freq* f, int32_t* freq_rank_host, int32_t* inv_rank_host, int32_t* counts_host);
int freq_destroy(fc_freq* f);
/* Re-order an embedding table by frequency: dst[r, :] = src[inv_rank[r], :] for r in [0, num_rows), fp32 rows of `dim`.
 * src_pinned and dst_pinned are distinct page-locked, GPU-mapped host buffers (the rows cross the host link twice);
 * inv_rank_host is an ordinary host array.  Synchronous.  Errors: INVALID_ARG, NOT_PERMUTATION, NOT_PINNED, HIP. */
int table_reorder(const float* src_pinned, float* dst_pinned, const int32_t* inv_rank_host, int64_t num_rows,
                  int32_t dim, void* hip_stream);

/* ---- per-kernel timing with HIP events on the handle's own streams (for the benchmark) ---- */
int cache_profile_enable(fc_cache* c, int32_t on);   /* on=1 starts recording, 0 stops; resets totals when turned on */
int cache_profile_count(void);                        /* number of timed kernels / copies                               */
const char* cache_profile_name(int32_t k);
/* total milliseconds and number of launches of timed item k since profiling was enabled; synchronises */
int cache_profile_get(fc_cache* c, int32_t k, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* FREQCACHE_H */
