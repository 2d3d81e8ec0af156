// C-ABI entry points of the freqcache library: set-up, warm-up, flush, introspection, profiling.
// The per-batch work lives in fc_prepare.hip (Algorithm 1) and fc_embedding.hip (EmbeddingBag + SGD).
#include "fc_internal.h"

#include <stdio.h>

#include <new>
#include <stdlib.h>
#include <string.h>
#include <string>
#include <vector>

namespace fc {

// ---- profiling ----
static const char* const kProfNames[P_COUNT] = {
    "remap_mark", "rank_count", "rank_plan", "rank_emit", "evict_gather", "evict_store", "free_count", "free_assign",
    "miss_fill", "slots_out", "bag_fwd", "sort_hist", "sort_scan", "sort_scatter", "bwd_reduce", "bwd_fixup",
    "h2d_block", "d2h_block", "flush_rows", "rows_in"};

ProfScope::ProfScope(fc_cache* c_, int item_, hipStream_t s_) : c(c_), s(s_), item(item_) {
    if (!c || !c->prof_on) return;
    for (hipEvent_t* e : {&a, &b}) {
        if (!c->ev_pool.empty()) { *e = c->ev_pool.back(); c->ev_pool.pop_back(); }
        else if (hipEventCreate(e) != hipSuccess) { *e = nullptr; }
    }
    if (a) (void)hipEventRecord(a, s);
}
ProfScope::~ProfScope() {
    if (!a || !b) return;
    (void)hipEventRecord(b, s);
    c->spans.push_back({item, a, b});
}
void prof_collect(fc_cache* c) {
    (void)hipStreamSynchronize(c->stream);
    (void)hipStreamSynchronize(c->side);
    if (c->aux) (void)hipStreamSynchronize(c->aux);
    if (c->pre) (void)hipStreamSynchronize(c->pre);
    // FC_TIMELINE=<file>: besides the totals, every span's start and end in us since the first span of this collection,
    // one "name start end" line each (which kernels really run side by side, and what waits for what)
    FILE*& timeline = c->timeline;          // per handle: two caches in one process keep separate files
    const char* want = getenv("FC_TIMELINE");
    if (timeline && (!want || c->timeline_path != want)) { fclose(timeline); timeline = nullptr; }
    if (!timeline && want && *want) { timeline = fopen(want, "w"); c->timeline_path = want; }
    if (timeline && !c->spans.empty()) fprintf(timeline, "# %zu spans\n", c->spans.size());
    for (const ProfSpan& sp : c->spans) {
        float ms = 0.f;
        if (timeline) {
            float t0 = 0.f, t1 = 0.f;
            if (hipEventElapsedTime(&t0, c->spans.front().a, sp.a) == hipSuccess && hipEventElapsedTime(&t1, c->spans.front().a, sp.b) == hipSuccess)
                fprintf(timeline, "%s %.1f %.1f\n", kProfNames[sp.item], t0 * 1e3f, t1 * 1e3f);
        }
        if (hipEventElapsedTime(&ms, sp.a, sp.b) == hipSuccess) { c->prof_ms[sp.item] += ms; c->prof_n[sp.item] += 1; }
        c->ev_pool.push_back(sp.a);
        c->ev_pool.push_back(sp.b);
    }
    c->spans.clear();
    if (timeline) fflush(timeline);
}

// ---- state initialisation ----
// first `count` entries: identity, rest -1
__global__ void k_iota_or_neg(int32_t* p, int64_t n, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = i < count ? (int32_t)i : -1;
}
// bitmap with the first `count` bits set
__global__ void k_bits_prefix(uint32_t* p, int64_t words, int64_t count) {
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < words; w += (int64_t)gridDim.x * blockDim.x) {
        const int64_t lo = w * 32;
        uint32_t v = 0;
        if (count >= lo + 32) v = 0xFFFFFFFFu;
        else if (count > lo) v = (1u << (count - lo)) - 1u;
        p[w] = v;
    }
}
__global__ void k_set_ctl(Ctl* ctl, int nfree) {
    ctl->err_flags = 0; ctl->async_flags = 0; ctl->nfree = nfree;
    ctl->status = 0; ctl->n_unique = 0; ctl->n_miss = 0; ctl->need = 0;
}

static int reset_state(fc_cache* c, bool warm) {
    hipStream_t st = c->stream;
    (void)gather_wait(c);
    c->gather_pending = false;
    for (hipStream_t x : {c->pre, c->pf, c->side}) if (x) FC_HIP(hipStreamSynchronize(x));
    c->next_pending = false; c->last_pst = c->stream;
    c->planned.valid = false; c->last_index_stream = nullptr; c->move_stream[0] = c->move_stream[1] = nullptr; c->pf_dep = nullptr;
    c->quiesce_stream = nullptr;
    c->fetch_timed[0] = c->fetch_timed[1] = false; c->last_copy_buf = -1;
    for (bool& b : c->copy_timed) b = false;
    for (PresortRec& r : c->rec) r.valid = false;
    if (c->dma_evict) { pool_wait(c, pool_published(c)); for (int64_t& r : c->blk_rows) r = 0; }
    const int64_t words = c->NB * RT_WORDS;
    k_iota_or_neg<<<1024, 256, 0, st>>>(c->rank_slot, c->N, warm ? c->C : 0);
    k_iota_or_neg<<<256, 256, 0, st>>>(c->slot_rank, c->C, warm ? c->C : 0);
    k_bits_prefix<<<256, 256, 0, st>>>(c->ubits, words, 0);
    k_bits_prefix<<<256, 256, 0, st>>>(c->pbits, words, 0);
    k_bits_prefix<<<256, 256, 0, st>>>(c->rbits, words, warm ? c->C : 0);
    k_set_ctl<<<1, 1, 0, st>>>(c->ctl, warm ? 0 : (int)c->C);
    FC_HIP(hipGetLastError());
    if (c->dirty) FC_HIP(hipMemsetAsync(c->dirty, 0, (size_t)c->C, st));   // loaded rows equal their host copies
    if (warm) FC_HIP(hipMemcpyAsync(c->cache, c->host, (size_t)c->C * c->D * 4, hipMemcpyHostToDevice, st));
    else FC_HIP(hipMemsetAsync(c->cache, 0, (size_t)c->C * c->D * 4, st));   // empty slots read as zeros
    FC_HIP(hipStreamSynchronize(st));
    c->last = fc_stats{};
    c->have_lists = false;
    return FC_OK;
}

static void destroy(fc_cache* c) {
    if (!c) return;
    if (c->tune_early && getenv("FC_TUNE_REPORT"))
        fprintf(stderr, "freqcache: early-fetch workgroups settled at %d (fetch / copy ratio %.3f)\n", c->fill_blocks_early, c->tune_ratio);
    (void)hipSetDevice(c->device);
    if (c->timeline) { fclose(c->timeline); c->timeline = nullptr; }
    (void)gather_wait(c);              // no gather thread is about to enqueue a copy
    if (c->stream || c->side) (void)hipDeviceSynchronize();
    gather_destroy(c);
    pool_destroy(c);
    for (int k = 0; k < 2; ++k) {
        for (void* p : {(void*)c->arrive_pin[k], (void*)c->miss_pin[k], (void*)c->src_pin[k]}) if (p) (void)hipHostFree(p);
        if (c->ev_list[k]) (void)hipEventDestroy(c->ev_list[k]);
    }
    for (int b = 0; b < DMA_BLOCKS; ++b) {
        if (c->blk_pin[b]) (void)hipHostFree(c->blk_pin[b]);
        if (c->vrank_pin[b]) (void)hipHostFree(c->vrank_pin[b]);
        if (c->vrank_buf[b]) (void)hipFree(c->vrank_buf[b]);
        if (c->ev_d2h[b]) (void)hipEventDestroy(c->ev_d2h[b]);
    }
    for (auto& set : c->lists) for (int32_t* p : set) if (p) (void)hipFree(p);
    if (c->dirty) (void)hipFree(c->dirty);
    if (c->dcount) (void)hipFree(c->dcount);
    if (c->dctl) (void)hipHostFree(c->dctl);
    for (int k = 0; k < 2; ++k) {
        if (c->arrive[k]) (void)hipFree(c->arrive[k]);
        for (hipEvent_t e : {c->ev_arrive[k], c->ev_fetch_a[k], c->ev_fetch_b[k]}) if (e) (void)hipEventDestroy(e);
    }
    for (int b = 0; b < DMA_BLOCKS; ++b)
        for (hipEvent_t e : {c->ev_copy_a[b], c->ev_copy_b[b]}) if (e) (void)hipEventDestroy(e);
    for (void* p : {(void*)c->freq_rank, (void*)c->rank_slot, (void*)c->slot_rank, (void*)c->cache, (void*)c->ubits,
                    (void*)c->rbits, (void*)c->tcount, (void*)c->hitpart, (void*)c->bsum, (void*)c->moff, (void*)c->vtake, (void*)c->voff,
                    (void*)c->rbuf,
                    (void*)c->ctl, (void*)c->stage_dev, (void*)c->stage_dev2, (void*)c->part, (void*)c->pmeta, (void*)c->pbits})
        if (p) (void)hipFree(p);
    for (SortBufs& sb : c->sb)
        for (void* p : {(void*)sb.keysA, (void*)sb.valsA, (void*)sb.keysB, (void*)sb.valsB, (void*)sb.ghist, (void*)sb.dtot, (void*)sb.stot[0], (void*)sb.stot[1]})
            if (p) (void)hipFree(p);
    for (PresortRec& r : c->rec) if (r.ev_sorted) (void)hipEventDestroy(r.ev_sorted);
    for (void* p : {(void*)c->hctl, (void*)c->stage_pin, (void*)c->list_pin}) if (p) (void)hipHostFree(p);
    if (c->own_host && c->host) (void)hipHostFree(c->host);
    for (const ProfSpan& sp : c->spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    for (hipEvent_t e : {c->ev_sort_tail, c->ev_assign_done, c->ev_emit_done, c->ev_quiesce, c->ev_evict_done, c->ev_gather_done, c->ev_slots, c->ev_s_now, c->ev_pre_done, c->ev_index_done, c->ev_move_done[0], c->ev_move_done[1]}) if (e) (void)hipEventDestroy(e);
    if (c->side) (void)hipStreamDestroy(c->side);
    if (c->pre) (void)hipStreamDestroy(c->pre);
    if (c->pf) (void)hipStreamDestroy(c->pf);
    delete c;
}

// ---- library streams on hardware queues of their own -------------------------------------------------------------
// A process has few hardware queues (four by default) and the runtime hands them to streams as they are created, so
// two streams may share one, and work on them then runs one after the other whatever the events say.  The pipelined
// schedule needs the caller's stream and the three library streams to run side by side.  Which streams share a queue
// cannot be asked, but it can be seen: a kernel that spins for a fixed time on one stream, a trivial kernel on the
// other; if the trivial one finishes long before the spinning one, the two streams are served side by side.
__global__ void k_spin(long long ticks, int* sink) {
    const long long t0 = wall_clock64();                  // constant 100 MHz counter
    while (wall_clock64() - t0 < ticks) { }
    if (sink && ticks < 0) *sink = 1;
}
__global__ void k_touch(int* sink) { if (sink && threadIdx.x == 12345) *sink = 1; }

// true: work on b runs while work on a is busy.  On any error: true (take the stream, nothing to be gained by being picky).
static bool run_side_by_side(hipStream_t a, hipStream_t b) {
    hipEvent_t e0 = nullptr, e1 = nullptr, e2 = nullptr;
    bool ok = true;
    if (hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess && hipEventCreate(&e2) == hipSuccess) {
        const long long spin_ticks = 30000;               // 300 us
        (void)hipEventRecord(e0, a);
        k_spin<<<1, 64, 0, a>>>(spin_ticks, nullptr);
        (void)hipEventRecord(e1, a);
        k_touch<<<1, 64, 0, b>>>(nullptr);
        (void)hipEventRecord(e2, b);
        float spin_ms = 0.f, other_ms = 0.f;
        if (hipStreamSynchronize(a) == hipSuccess && hipStreamSynchronize(b) == hipSuccess &&
            hipEventElapsedTime(&spin_ms, e0, e1) == hipSuccess && hipEventElapsedTime(&other_ms, e0, e2) == hipSuccess)
            ok = other_ms < 0.5f * spin_ms;
    }
    (void)hipGetLastError();
    for (hipEvent_t e : {e0, e1, e2}) if (e) (void)hipEventDestroy(e);
    return ok;
}

// Three non-blocking streams that run side by side with the caller's stream and with each other, chosen among a few
// candidates; whatever is left over when the candidates run out is taken as it comes.
static int make_library_streams(fc_cache* c) {
    hipStream_t* want[3] = {&c->side, &c->pre, &c->pf};
    std::vector<hipStream_t> rejected;
    int have = 0;
    for (int tries = 0; tries < 12 && have < 3; ++tries) {
        hipStream_t s = nullptr;
        FC_HIP(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        bool good = run_side_by_side(c->stream, s);
        for (int k = 0; k < have && good; ++k) good = run_side_by_side(*want[k], s);
        if (good) *want[have++] = s; else rejected.push_back(s);
    }
    while (have < 3 && !rejected.empty()) { *want[have++] = rejected.back(); rejected.pop_back(); }
    for (hipStream_t s : rejected) (void)hipStreamDestroy(s);
    while (have < 3) FC_HIP(hipStreamCreateWithFlags(want[have++], hipStreamNonBlocking));
    return FC_OK;
}

static int create(int64_t N, int32_t D, int64_t C, const int32_t* freq_rank, float* host_weight, int64_t staging_rows,
                  int32_t flags, void* hip_stream, fc_cache* c) {
    FC_HIP(hipGetDevice(&c->device));
    FC_TRY(noalloc_setup(c->device));
    c->N = N; c->C = C; c->D = D; c->flags = flags;
    c->stream = (hipStream_t)hip_stream;
    c->vec = (D % 4 == 0) ? 4 : (D % 2 == 0) ? 2 : 1;
    const int nv = D / c->vec;
    c->lpr = 1;
    while (c->lpr < nv && c->lpr < 64) c->lpr <<= 1;
    if (staging_rows <= 0) staging_rows = C < 524288 ? C : 524288;
    if (staging_rows > C) staging_rows = C;
    c->staging_rows = staging_rows;
    if (const char* e = getenv("FC_EVICT_BLOCKS")) { const int v = atoi(e); if (v >= 1 && v <= 4096) c->evict_blocks = v; }
    if (flags & FC_EVICT_DMA) c->fill_blocks = 40;
    if (const char* e = getenv("FC_FILL_BLOCKS")) { const int v = atoi(e); if (v >= 1) c->fill_blocks = v; }
    if (const char* e = getenv("FC_FILL_BLOCKS_EARLY")) { const int v = atoi(e); if (v >= 1) { c->fill_blocks_early = v; c->tune_early = false; } }
    if (const char* e = getenv("FC_FILL_BLOCKS_EARLY_START")) { const int v = atoi(e); if (v >= 1) c->fill_blocks_early = v; }   // still tuned
    c->fill_blocks_early_max = c->fill_blocks_early;
    if (const char* e = getenv("FC_FWD_SORTED")) c->fwd_sorted = atoi(e) != 0;
    if (const char* e = getenv("FC_SORT_TAIL")) c->sort_tail_side = atoi(e) != 0;
    if (const char* e = getenv("FC_SORT_BITS")) c->sort_max_bits = atoi(e);
    if (const char* e = getenv("FC_SORT_FUSED")) c->sort_no_fuse = atoi(e) == 0;
    if (const char* e = getenv("FC_AHEAD_MISS_PCT")) { const float v = (float)atof(e); if (v >= 0.f) c->ahead_miss_pct = v; }
    if (const char* e = getenv("FC_FWD_BAGS")) { const int v = atoi(e); if (v == 1 || v == 2 || v == 4) c->fwd_bags = v; }
    if (const char* e = getenv("FC_MARK_IPT")) { const int v = atoi(e); if (v >= 1 && v <= 64) c->mark_ids_per_thread = v; }
    if (const char* e = getenv("FC_EVICT_EARLY")) c->evict_early = atoi(e);
    c->NB = cdiv(cdiv(N, 32), RT_WORDS);
    const size_t words = (size_t)c->NB * RT_WORDS;

    // host table
    if (host_weight) {
        hipPointerAttribute_t attr;
        hipError_t e = hipPointerGetAttributes(&attr, host_weight);
        if (e != hipSuccess || attr.type != hipMemoryTypeHost) { (void)hipGetLastError(); return FC_ERR_NOT_PINNED; }
        c->host = host_weight;
        c->own_host = false;
    } else {
        if (hipHostMalloc((void**)&c->host, (size_t)N * D * 4, hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError(); c->host = nullptr; return FC_ERR_OOM_PINNED;
        }
        c->own_host = true;
    }
    if (hipHostGetDevicePointer((void**)&c->host_dev, c->host, 0) != hipSuccess) { (void)hipGetLastError(); return FC_ERR_NOT_PINNED; }

    FC_HIP(hipMalloc((void**)&c->freq_rank, (size_t)N * 4));
    FC_HIP(hipMalloc((void**)&c->rank_slot, (size_t)N * 4));
    FC_HIP(hipMalloc((void**)&c->slot_rank, (size_t)C * 4));
    FC_HIP(hipMalloc((void**)&c->cache, (size_t)C * D * 4));
    FC_HIP(hipMalloc((void**)&c->ubits, words * 4));
    FC_HIP(hipMalloc((void**)&c->rbits, words * 4));
    FC_HIP(hipMalloc((void**)&c->pbits, words * 4));
    FC_HIP(hipMalloc((void**)&c->tcount, (size_t)cdiv(C, 1024) * 4));
    FC_HIP(hipMalloc((void**)&c->hitpart, 256 * 4));
    FC_HIP(hipMalloc((void**)&c->bsum, (size_t)c->NB * 3 * 4));
    FC_HIP(hipMalloc((void**)&c->moff, (size_t)c->NB * 4));
    FC_HIP(hipMalloc((void**)&c->vtake, (size_t)c->NB * 4));
    FC_HIP(hipMalloc((void**)&c->voff, (size_t)c->NB * 4));
    c->dma_evict = (flags & FC_EVICT_DMA) != 0;
    c->dirty_track = (flags & FC_DIRTY_TRACK) != 0;
    for (auto& set : c->lists)
        for (int k = 0; k < 7; ++k) {
            const bool wanted = k < 3 || (k == 3 && c->dma_evict) || (k == 4 && (!c->dma_evict || c->dirty_track)) ||
                                (k >= 5 && c->dirty_track);
            if (wanted) FC_HIP(hipMalloc((void**)&set[k], (size_t)C * 4));
        }
    if (c->dirty_track) {
        FC_HIP(hipMalloc((void**)&c->dirty, (size_t)C));
        FC_HIP(hipMalloc((void**)&c->dcount, (size_t)cdiv(C, 1024) * 4));
        if (hipHostMalloc((void**)&c->dctl, 2 * sizeof(int32_t), hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); return FC_ERR_OOM_PINNED; }
        c->dctl[0] = c->dctl[1] = 0;
    }
    if (c->dma_evict) {
        for (int b = 0; b < DMA_BLOCKS; ++b) {
            FC_HIP(hipMalloc((void**)&c->vrank_buf[b], (size_t)C * 4));
            if (hipHostMalloc((void**)&c->blk_pin[b], (size_t)staging_rows * D * 4, hipHostMallocDefault) != hipSuccess ||
                hipHostMalloc((void**)&c->vrank_pin[b], (size_t)staging_rows * 4, hipHostMallocDefault) != hipSuccess) {
                (void)hipGetLastError(); return FC_ERR_OOM_PINNED;
            }
            FC_HIP(hipEventCreateWithFlags(&c->ev_d2h[b], hipEventDisableTiming | hipEventBlockingSync));
        }
    }
    use_list_set(c, 0);
    FC_HIP(hipMalloc((void**)&c->ctl, sizeof(Ctl)));
    FC_HIP(hipMalloc((void**)&c->stage_dev, (size_t)staging_rows * D * 4 * (c->dma_evict ? DMA_BLOCKS : 1)));
    if (hipHostMalloc((void**)&c->hctl, sizeof(HostCtl), hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); return FC_ERR_OOM_PINNED; }
    memset(c->hctl, 0, sizeof(HostCtl));
    if (flags & FC_TRANSMIT_STAGED) {
        FC_HIP(hipMalloc((void**)&c->stage_dev2, (size_t)staging_rows * D * 4));
        if (hipHostMalloc((void**)&c->stage_pin, (size_t)staging_rows * D * 4, hipHostMallocDefault) != hipSuccess ||
            hipHostMalloc((void**)&c->list_pin, (size_t)C * 2 * 4, hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError(); return FC_ERR_OOM_PINNED;
        }
    }
    FC_TRY(make_library_streams(c));
    // FC_FETCH_CU_MASK=<k> (experiment): the stream of the early row fetch may only use k compute units, spread evenly
    if (const char* e = getenv("FC_FETCH_CU_MASK")) {
        const int k = atoi(e);
        hipDeviceProp_t prop;
        if (k >= 1 && hipGetDeviceProperties(&prop, c->device) == hipSuccess && k < prop.multiProcessorCount) {
            const int cus = prop.multiProcessorCount;
            std::vector<uint32_t> mask((size_t)(cus + 31) / 32, 0u);
            for (int i = 0; i < k; ++i) { const int b = (int)((int64_t)i * cus / k); mask[b >> 5] |= 1u << (b & 31); }
            hipStream_t ms = nullptr;
            if (hipExtStreamCreateWithCUMask(&ms, (uint32_t)mask.size(), mask.data()) == hipSuccess) {
                (void)hipStreamDestroy(c->pf);
                c->pf = ms;
            } else (void)hipGetLastError();
        }
    }
    c->aux = c->pf;
    c->pst = c->last_pst = c->stream;
    c->presort = (flags & FC_NO_PRESORT) == 0;
    for (hipEvent_t* e : {&c->ev_sort_tail, &c->ev_assign_done, &c->ev_emit_done, &c->ev_quiesce, &c->ev_evict_done, &c->ev_gather_done, &c->ev_slots, &c->ev_s_now, &c->ev_pre_done, &c->ev_index_done, &c->ev_move_done[0], &c->ev_move_done[1], &c->ev_arrive[0], &c->ev_arrive[1],
                          &c->rec[0].ev_sorted, &c->rec[1].ev_sorted})
        FC_HIP(hipEventCreateWithFlags(e, hipEventDisableTiming));
    if (c->dma_evict) {
        for (int k = 0; k < 2; ++k) { FC_HIP(hipEventCreate(&c->ev_fetch_a[k])); FC_HIP(hipEventCreate(&c->ev_fetch_b[k])); }
        for (int b = 0; b < DMA_BLOCKS; ++b) { FC_HIP(hipEventCreate(&c->ev_copy_a[b])); FC_HIP(hipEventCreate(&c->ev_copy_b[b])); }
    } else {
        c->tune_early = false;
    }
    FC_HIP(hipMemcpy(c->freq_rank, freq_rank, (size_t)N * 4, hipMemcpyHostToDevice));
    if (c->dma_evict) {
        int threads = 8;
        if (const char* e = getenv("FC_SCATTER_THREADS")) { const int v = atoi(e); if (v >= 1 && v <= 64) threads = v; }
        FC_TRY(pool_create(c, threads));
    }
    c->miss_dma = (flags & FC_MISS_DMA) != 0 && !c->dirty_track;
    if (c->miss_dma) {
        for (int k = 0; k < 2; ++k) {
            if (hipHostMalloc((void**)&c->arrive_pin[k], (size_t)staging_rows * D * 4, hipHostMallocDefault) != hipSuccess ||
                hipHostMalloc((void**)&c->miss_pin[k], (size_t)staging_rows * 4, hipHostMallocDefault) != hipSuccess ||
                hipHostMalloc((void**)&c->src_pin[k], (size_t)staging_rows * 4, hipHostMallocDefault) != hipSuccess) {
                (void)hipGetLastError(); return FC_ERR_OOM_PINNED;
            }
            FC_HIP(hipEventCreateWithFlags(&c->ev_list[k], hipEventDisableTiming));
        }
        int threads = 6;
        if (const char* e = getenv("FC_GATHER_THREADS")) { const int v = atoi(e); if (v >= 1 && v <= 64) threads = v; }
        FC_TRY(gather_create(c, threads));
    }
    return reset_state(c, (flags & FC_WARM) != 0);
}

}  // namespace fc

using namespace fc;

// Duration in us between two timing events if both have completed, else a negative number.
static float elapsed_us(hipEvent_t a, hipEvent_t b) {
    if (hipEventQuery(b) != hipSuccess) { (void)hipGetLastError(); return -1.f; }
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, a, b) != hipSuccess) { (void)hipGetLastError(); return -1.f; }
    return ms * 1e3f;
}

// One step of the controller described at fc_cache::tune_early: the fetch that last used list set k against the newest
// finished block copy (no copy at all: the fetch has the link to itself and may take what it can use).
static void tune_fetch_grid(fc_cache* c, int k) {
    if (!c->fetch_timed[k]) return;
    const float f_us = elapsed_us(c->ev_fetch_a[k], c->ev_fetch_b[k]);
    if (f_us <= 0.f) return;
    float d_us = -1.f;
    if (c->last_copy_buf >= 0)
        for (int i = 0; i < DMA_BLOCKS && d_us <= 0.f; ++i) {
            const int b = (c->last_copy_buf - i + DMA_BLOCKS) % DMA_BLOCKS;
            if (c->copy_timed[b]) d_us = elapsed_us(c->ev_copy_a[b], c->ev_copy_b[b]);
        }
    const float r = d_us > 0.f ? f_us / d_us : 2.f;
    c->tune_ratio = c->tune_ratio <= 0.f ? r : 0.75f * c->tune_ratio + 0.25f * r;
    if (++c->tune_count < 6) return;
    c->tune_count = 0;
    if (c->tune_ratio < 0.98f && c->fill_blocks_early > 8) --c->fill_blocks_early;
    else if (c->tune_ratio > 1.06f && c->fill_blocks_early < c->fill_blocks_early_max) ++c->fill_blocks_early;
}

// the arrival block of list set k (cache_plan_next fetches missing rows into it ahead of time)
static bool ensure_arrival_block(fc_cache* c, int k) {
    if (c->arrive[k]) return true;
    if (hipMalloc((void**)&c->arrive[k], (size_t)c->staging_rows * c->D * 4) != hipSuccess) {
        (void)hipGetLastError(); c->arrive[k] = nullptr;
        return false;
    }
    return true;
}

// cache_plan_next: the planned batch's missing rows into the arrival block of its list set, on the stream pf
static int fetch_early(fc_cache* c, int64_t M) {
    const int k = c->lset;
    if (!ensure_arrival_block(c, k)) return FC_OK;   // no room for the block: the rows are fetched at cache_advance instead
    if (c->miss_dma) {
        // host threads gather the rows, the DMA engine carries them; ev_arrive[k] is recorded by the thread that hands over
        // the last chunk, and cache_advance waits (on the host) for that record before it makes its stream wait for it
        FC_TRY(gather_start(c, M));
        c->gather_pending = true;
        c->planned.arrived = true;
        return FC_OK;
    }
    if (c->tune_early) tune_fetch_grid(c, k);
    FC_HIP(hipStreamWaitEvent(c->pf, c->ev_emit_done, 0));       // which rows are missing and where their newest copies are
    if (c->pf_dep) FC_HIP(hipStreamWaitEvent(c->pf, c->pf_dep, 0));
    if (c->dma_evict) {
        FC_HIP(hipEventRecord(c->ev_fetch_a[k], c->pf));
        FC_TRY(launch_fill_rows(c, c->pf, M, c->arrive[k], c->staging_rows, c->fill_blocks_early));
        FC_HIP(hipEventRecord(c->ev_fetch_b[k], c->pf));
        c->fetch_timed[k] = true;
    } else {
        FC_TRY(launch_copy_rows(c, c->pf, P_MISS_FILL, c->arrive[k], nullptr, c->staging_rows, c->host_dev, c->miss_ranks, c->N, M, c->fill_blocks));
    }
    FC_HIP(hipEventRecord(c->ev_arrive[k], c->pf));
    c->planned.arrived = true;
    return FC_OK;
}

// the caller's stream takes over from the look-ahead stream: everything cache_prepare_next enqueued comes first
static int adopt_next(fc_cache* c) {
    if (c->planned.valid) {            // a batch planned ahead whose rows have not moved yet: move them now
        const MovePlan mv = c->planned;
        c->planned.valid = false;
        FC_TRY(prepare_move(c, c->stream, mv));
    }
    if (c->next_pending || c->last_pst != c->stream) {
        FC_HIP(hipStreamWaitEvent(c->stream, c->ev_pre_done, 0));
        c->next_pending = false;
        c->last_pst = c->stream;
    }
    c->cur_ticket = c->pending_ticket;     // the batch prepared ahead of time (if any) is the current one now
    return FC_OK;
}

extern "C" {

int cache_create(int64_t num_rows, int32_t dim, int64_t cache_rows, const int32_t* freq_rank_host, float* host_weight,
                 int64_t staging_rows, int32_t flags, void* hip_stream, fc_cache** out) {
    const int64_t LIM = ((int64_t)1 << 31) - 65536;
    if (!out) return FC_ERR_INVALID_ARG;
    *out = nullptr;
    if (!freq_rank_host || num_rows <= 0 || num_rows >= LIM || dim <= 0 || dim > 1024 || cache_rows <= 0 || cache_rows > num_rows ||
        staging_rows < 0 || (flags & ~(FC_WARM | FC_TRANSMIT_STAGED | FC_EVICT_DMA | FC_NO_PRESORT | FC_DIRTY_TRACK | FC_INPUTS_READY | FC_MISS_DMA)) ||
        ((flags & FC_TRANSMIT_STAGED) && (flags & (FC_EVICT_DMA | FC_MISS_DMA))))
        return FC_ERR_INVALID_ARG;
    if ((flags & FC_WARM) && !host_weight) return FC_ERR_INVALID_ARG;   // nothing to warm up from yet
    {   // idx_map must be a permutation: the host table is the original table re-ordered (Section 4.2)
        std::vector<uint8_t> seen;
        try { seen.assign((size_t)num_rows, 0); } catch (const std::bad_alloc&) { return FC_ERR_INVALID_ARG; }
        for (int64_t i = 0; i < num_rows; ++i) {
            const int32_t r = freq_rank_host[i];
            if (r < 0 || r >= num_rows || seen[r]) return FC_ERR_NOT_PERMUTATION;
            seen[r] = 1;
        }
    }
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) { (void)hipGetLastError(); return FC_ERR_HIP; }
    fc_cache* c = new (std::nothrow) fc_cache();
    if (!c) return FC_ERR_OOM_PINNED;                    // host memory
    const int rc = create(num_rows, dim, cache_rows, freq_rank_host, host_weight, staging_rows, flags, hip_stream, c);
    if (rc != FC_OK) { destroy(c); return rc; }
    *out = c;
    return FC_OK;
}

int cache_reserve(fc_cache* c, int64_t max_ids, int32_t pipelined) {
    const int64_t LIM = ((int64_t)1 << 31) - 65536;
    if (!c || max_ids < 0 || max_ids >= LIM) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    FC_TRY(ensure_rbuf(c, max_ids));
    FC_TRY(reserve_bwd(c, max_ids));
    if (pipelined && !(c->flags & FC_TRANSMIT_STAGED))
        for (int k = 0; k < 2; ++k) if (!ensure_arrival_block(c, k)) return FC_ERR_OOM_DEVICE;
    return FC_OK;
}

int cache_warm(fc_cache* c) {
    if (!c) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    FC_TRY(adopt_next(c));
    FC_HIP(hipStreamSynchronize(c->stream));
    FC_HIP(hipStreamSynchronize(c->side));
    c->evict_pending = false;
    return reset_state(c, true);
}

int cache_prepare(fc_cache* c, const int64_t* ids_dev, int64_t n, const int64_t* offsets_dev, int64_t num_bags,
                  int32_t* slots_dev) {
    if (!c) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    FC_HIP(hipEventRecord(c->ev_s_now, c->stream));
    FC_TRY(adopt_next(c));
    const int rc = prepare_impl(c, c->stream, false, ids_dev, n, offsets_dev, num_bags, slots_dev);
    if (rc == FC_OK) c->cur_ticket = c->pending_ticket = c->ticket;
    return rc;
}

int cache_prepare_next(fc_cache* c, const int64_t* ids_dev, int64_t n, const int64_t* offsets_dev, int64_t num_bags,
                       int32_t* slots_dev) {
    if (!c) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    // everything the caller has enqueued so far (the backward pass of the batch before the current one, and the
    // input buffers of this call) is complete before this call's row movement, or before all of it when the last
    // prepare ran on the caller's stream
    FC_HIP(hipEventRecord(c->ev_s_now, c->stream));
    if (c->last_pst != c->pre) FC_HIP(hipStreamWaitEvent(c->pre, c->ev_s_now, 0));
    const int rc = prepare_impl(c, c->pre, true, ids_dev, n, offsets_dev, num_bags, slots_dev);
    c->pst = c->stream;
    // also after a refusal (nothing changed then): the streams stay ordered all the same
    FC_HIP(hipEventRecord(c->ev_pre_done, c->pre));
    c->last_pst = c->pre;
    c->next_pending = true;
    if (rc == FC_OK) c->pending_ticket = c->ticket;
    return rc;
}

int cache_plan_next(fc_cache* c, const int64_t* ids_dev, int64_t n, const int64_t* offsets_dev, int64_t num_bags,
                    int32_t* slots_dev) {
    if (!c || (c->flags & FC_TRANSMIT_STAGED)) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    if (c->planned.valid) FC_TRY(cache_advance(c));
    // The index half touches no rows, so it need not wait for the row movement, forward or backward work the caller
    // enqueued since the last cache_prepare / cache_advance: it is ordered behind the caller's stream as of the entry
    // of that call (which covers the backward pass whose sorted pairs this call's sort will overwrite).
    // With FC_INPUTS_READY the decisions themselves wait for nothing on the caller's stream (they read the ids and the
    // library's own index state, which only index halves change); the slot write-out, the first kernel to touch a buffer
    // of the caller's, still waits.  With FC_DIRTY_TRACK the row movement of the current batch marks rows as in transit,
    // which the planned batch's decisions read: no head start then.
    // Running ahead pays where HBM binds the step and costs where the host link does (the early fetch and the evicted-block
    // copy then overlap all the time and slow each other down).  Which of the two it is follows from the bytes: a missing row
    // crosses the link once each way, a lookup and a bag move one row each through HBM, and the two rates differ by a factor
    // of about 100, so the link binds once the previous batch missed more than about 2 rows per 100 lookups-and-bags/2
    // (config 4: 1.7 before its hot set rotates, 2.9 and 3.5 after; config 2: 9.6).  FC_AHEAD_MISS_PCT moves the threshold.
    const bool may_run_ahead = (c->flags & FC_INPUTS_READY) && !c->dirty_track;
    const bool early = may_run_ahead && (double)c->last.n_miss * 100.0 <= (double)c->ahead_miss_pct * 0.5 * (double)(n + num_bags);
    c->ahead_now = early;
    if (!early) FC_HIP(hipStreamWaitEvent(c->pre, c->ev_s_now, 0));
    // FC_DIRTY_TRACK: which victims of the current batch are in transit is only marked by its row movement
    if (c->dirty_track && c->move_stream[c->lset]) FC_HIP(hipStreamWaitEvent(c->pre, c->ev_move_done[c->lset], 0));
    MovePlan mv;
    // the slot write-out is folded into the first kernel of the sort (one launch and one pass over the ranks fewer)
    const bool fold = c->presort && n > 0 && num_bags > 0;
    const int rc = prepare_index(c, c->pre, false, ids_dev, n, offsets_dev, num_bags, slots_dev, &mv, early ? c->ev_s_now : nullptr, fold);
    c->pst = c->stream;
    c->last_pst = c->pre;
    c->next_pending = true;
    if (rc != FC_OK) {
        FC_HIP(hipEventRecord(c->ev_pre_done, c->pre));
        return rc;
    }
    c->planned = mv;
    c->pending_ticket = c->ticket;
    int rc2 = FC_OK;
    // Missing rows ahead of time: they are not resident, so nothing the caller's stream still does to the current
    // batch changes them; their newest copy is in the host table or in an evicted-row block (transit marks), and the
    // latest row movement, which produced both, is the only thing to wait for.  Victims leave, and these rows enter
    // their slots, at cache_advance.
    if (mv.M > 0 && mv.M <= c->staging_rows) rc2 = fetch_early(c, mv.M);
    if (fold) {
        c->pst = c->pre;
        const int rs = presort_impl(c, slots_dev, n, offsets_dev, num_bags, slots_dev);
        c->pst = c->stream;
        if (rs != FC_OK) FC_TRY(launch_slots_out(c, c->pre, slots_dev, n));     // no sort: the plain write-out
        FC_HIP(hipEventRecord(c->ev_index_done, c->pre));
    } else if (n > 0) { c->pst = c->pre; (void)presort_impl(c, slots_dev, n, offsets_dev, num_bags); c->pst = c->stream; }
    FC_HIP(hipEventRecord(c->ev_pre_done, c->pre));
    return rc2;
}

int cache_advance(fc_cache* c) {
    if (!c) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    FC_HIP(hipEventRecord(c->ev_s_now, c->stream));
    if (c->planned.valid) return adopt_next(c);
    if (c->next_pending) {
        FC_HIP(hipStreamWaitEvent(c->stream, c->ev_pre_done, 0));
        c->next_pending = false;
    }
    c->cur_ticket = c->pending_ticket;
    return FC_OK;
}

int embedding_bag_fwd(fc_cache* c, const int32_t* slots_dev, int64_t n, const int64_t* offsets_dev, int64_t num_bags,
                      float* out_dev) {
    return fwd_impl(c, slots_dev, n, offsets_dev, num_bags, out_dev);
}

int embedding_bag_bwd_sgd(fc_cache* c, const int32_t* slots_dev, int64_t n, const int64_t* offsets_dev,
                          int64_t num_bags, const float* grad_out_dev, float lr) {
    return bwd_impl(c, slots_dev, n, offsets_dev, num_bags, grad_out_dev, lr);
}

int embedding_bag_bwd_sgd_noalloc(fc_cache* c, const int32_t* slots_dev, int64_t n, const int64_t* offsets_dev,
                                  int64_t num_bags, const float* grad_out_dev, float lr) {
    return bwd_noalloc_impl(c, slots_dev, n, offsets_dev, num_bags, grad_out_dev, lr);
}

int cache_flush(fc_cache* c) {
    if (!c) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    FC_TRY(adopt_next(c));
    FC_HIP(hipStreamSynchronize(c->side));      // pending evicted rows first: flush must not be overtaken
    c->evict_pending = false;
    FC_TRY(dma_quiesce(c, c->stream));
    if (c->flags & FC_TRANSMIT_STAGED) {
        // the cached weight is contiguous: bulk-copy slot ranges, scatter the resident ones on the host
        std::vector<int32_t> sr((size_t)c->C);
        FC_HIP(hipMemcpyAsync(sr.data(), c->slot_rank, (size_t)c->C * 4, hipMemcpyDeviceToHost, c->stream));
        FC_HIP(hipStreamSynchronize(c->stream));
        if (c->dirty) {                // dirty rows only: a clean slot counts as empty for the scatter below
            std::vector<uint8_t> dr((size_t)c->C);
            FC_HIP(hipMemcpy(dr.data(), c->dirty, (size_t)c->C, hipMemcpyDeviceToHost));
            for (int64_t s = 0; s < c->C; ++s) if (!dr[s]) sr[s] = -1;
        }
        const size_t rowb = (size_t)c->D * 4;
        for (int64_t s0 = 0; s0 < c->C; s0 += c->staging_rows) {
            const int64_t rows = c->C - s0 < c->staging_rows ? c->C - s0 : c->staging_rows;
            {
                ProfScope ps(c, P_D2H_BLOCK, c->stream);
                FC_HIP(hipMemcpyAsync(c->stage_pin, c->cache + (size_t)s0 * c->D, rows * rowb, hipMemcpyDeviceToHost, c->stream));
            }
            FC_HIP(hipStreamSynchronize(c->stream));
#pragma omp parallel for schedule(static)
            for (int64_t j = 0; j < rows; ++j)
                if (sr[s0 + j] >= 0) memcpy(c->host + (size_t)sr[s0 + j] * c->D, c->stage_pin + (size_t)j * c->D, rowb);
        }
    } else {
        FC_TRY(launch_flush_rows(c, c->stream));
    }
    if (c->dirty) FC_HIP(hipMemsetAsync(c->dirty, 0, (size_t)c->C, c->stream));   // the host table is current for every resident row
    FC_HIP(hipStreamSynchronize(c->stream));
    return FC_OK;
}

int cache_check(fc_cache* c) {
    if (!c) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    FC_TRY(adopt_next(c));
    FC_HIP(hipStreamSynchronize(c->aux));
    FC_HIP(hipStreamSynchronize(c->stream));
    FC_HIP(hipStreamSynchronize(c->side));
    FC_TRY(dma_quiesce(c, c->stream));
    FC_HIP(hipStreamSynchronize(c->stream));
    Ctl h;
    FC_HIP(hipMemcpy(&h, c->ctl, sizeof(Ctl), hipMemcpyDeviceToHost));
    if (h.async_flags) {
        FC_HIP(hipMemset(&c->ctl->async_flags, 0, 4));
        return FC_ERR_BAD_SLOT;
    }
    return FC_OK;
}

int cache_destroy(fc_cache* c) {
    if (!c) return FC_ERR_INVALID_ARG;
    destroy(c);
    return FC_OK;
}

int cache_last_stats(const fc_cache* c, fc_stats* out) {
    if (!c || !out) return FC_ERR_INVALID_ARG;
    *out = c->last;
    return FC_OK;
}

int cache_copy_state(fc_cache* c, int32_t* slot_rank_host, int32_t* rank_slot_host) {
    if (!c) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    FC_HIP(hipStreamSynchronize(c->pre));
    FC_HIP(hipStreamSynchronize(c->stream));
    if (slot_rank_host) FC_HIP(hipMemcpy(slot_rank_host, c->slot_rank, (size_t)c->C * 4, hipMemcpyDeviceToHost));
    if (rank_slot_host) {
        FC_HIP(hipMemcpy(rank_slot_host, c->rank_slot, (size_t)c->N * 4, hipMemcpyDeviceToHost));
        if (c->dma_evict)      // "in transit" is an internal shade of "not resident"
            for (int64_t r = 0; r < c->N; ++r) if (rank_slot_host[r] < -1) rank_slot_host[r] = -1;
    }
    return FC_OK;
}

int cache_last_lists(fc_cache* c, int32_t* miss_ranks_host, int32_t* evict_ranks_host, int32_t* evict_slots_host,
                     int32_t* fill_slots_host) {
    if (!c) return FC_ERR_INVALID_ARG;
    if (!c->have_lists) return FC_OK;
    FC_HIP(hipSetDevice(c->device));
    FC_HIP(hipStreamSynchronize(c->pre));
    FC_HIP(hipStreamSynchronize(c->stream));
    const size_t m = (size_t)c->last.n_miss * 4, v = (size_t)c->last.n_evict * 4;
    if (miss_ranks_host && m) FC_HIP(hipMemcpy(miss_ranks_host, c->miss_ranks, m, hipMemcpyDeviceToHost));
    if (fill_slots_host && m) FC_HIP(hipMemcpy(fill_slots_host, c->fill_slots, m, hipMemcpyDeviceToHost));
    if (evict_ranks_host && v) FC_HIP(hipMemcpy(evict_ranks_host, c->vrank, v, hipMemcpyDeviceToHost));
    if (evict_slots_host && v) FC_HIP(hipMemcpy(evict_slots_host, c->vslot, v, hipMemcpyDeviceToHost));
    return FC_OK;
}

int cache_copy_rows(fc_cache* c, float* rows_host) {
    if (!c || !rows_host) return FC_ERR_INVALID_ARG;
    FC_HIP(hipSetDevice(c->device));
    FC_HIP(hipStreamSynchronize(c->pre));
    FC_HIP(hipStreamSynchronize(c->stream));
    FC_HIP(hipMemcpy(rows_host, c->cache, (size_t)c->C * c->D * 4, hipMemcpyDeviceToHost));
    return FC_OK;
}

float* cache_host_weight(fc_cache* c) { return c ? c->host : nullptr; }

const char* cache_strerror(int code) {
    switch (code) {
        case FC_OK: return "ok";
        case FC_ERR_INVALID_ARG: return "invalid argument";
        case FC_ERR_ID_OUT_OF_RANGE: return "id outside [0, num_rows)";
        case FC_ERR_BAD_OFFSETS: return "bag offsets do not tile [0, n)";
        case FC_ERR_BATCH_EXCEEDS_CACHE: return "batch touches more distinct rows than the cache holds";
        case FC_ERR_NOT_PERMUTATION: return "freq_rank is not a permutation";
        case FC_ERR_OOM_DEVICE: return "out of device memory";
        case FC_ERR_OOM_PINNED: return "out of pinned host memory";
        case FC_ERR_HIP: return "HIP runtime error or no usable GPU";
        case FC_ERR_NOT_PINNED: return "host_weight is not pinned, GPU-mapped memory";
        case FC_ERR_BAD_SLOT: return "slot index outside [0, cache_rows)";
        case FC_ERR_COUNT_OVERFLOW: return "freq_add: more ids than the 32-bit counters can hold";
        case FC_ERR_SCRATCH_EXCEEDED: return "batch too large for the fixed scratch of embedding_bag_bwd_sgd_noalloc";
        default: return "unknown error";
    }
}

int cache_profile_enable(fc_cache* c, int32_t on) {
    if (!c) return FC_ERR_INVALID_ARG;
    prof_collect(c);
    if (on) { for (int k = 0; k < P_COUNT; ++k) { c->prof_ms[k] = 0; c->prof_n[k] = 0; } }
    c->prof_on = on != 0;
    return FC_OK;
}

int cache_profile_count(void) { return P_COUNT; }

const char* cache_profile_name(int32_t k) { return (k >= 0 && k < P_COUNT) ? kProfNames[k] : ""; }

int cache_profile_get(fc_cache* c, int32_t k, double* total_ms, int64_t* launches) {
    if (!c || k < 0 || k >= P_COUNT) return FC_ERR_INVALID_ARG;
    prof_collect(c);
    if (total_ms) *total_ms = c->prof_ms[k];
    if (launches) *launches = c->prof_n[k];
    return FC_OK;
}

}  // extern "C"
