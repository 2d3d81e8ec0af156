// DMA miss path (FC_MISS_DMA): the paper's block transmitter for the host -> device direction (Section 4.3), pipelined.
// cache_plan_next copies the list of missing rows to the host; a small pool of host threads gathers those rows out of
// the frequency-ordered host table into a pinned block, chunk by chunk, and as each chunk is complete hands it to the
// DMA engine (hipMemcpyAsync on the fetch stream) into the arrival block in HBM.  No compute unit reads host memory;
// cache_advance then copies the arrived rows into their slots as it does after the zero-copy fetch.  Rows whose newest
// copy is still in an evicted-row block (in transit) are left out here: cache_advance takes them from that block.
#include "fc_internal.h"

#include <string.h>

#include <atomic>
#include <condition_variable>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

namespace fc {

constexpr int GATHER_MAX_CHUNKS = 64;

struct GatherPool {
    fc_cache* c = nullptr;
    std::vector<std::thread> threads;
    std::mutex m;
    std::condition_variable cv_job, cv_done;
    uint64_t published = 0, completed = 0;     // jobs are numbered 1, 2, ...; at most one is outstanding
    struct Job { int k = 0; int64_t M = 0, chunk = 0; int nchunks = 0; } job;
    std::atomic<int> chunk_left[GATHER_MAX_CHUNKS];   // threads still working on chunk i
    std::atomic<int> chunks_sent{0};
    std::atomic<int> failed{0};
    bool stop = false;
};

static void gather_worker(GatherPool* p, int t, int T) {
    fc_cache* c = p->c;
    (void)hipSetDevice(c->device);
    const size_t rowb = (size_t)c->D * 4;
    for (uint64_t next = 1;; ++next) {
        GatherPool::Job j;
        {
            std::unique_lock<std::mutex> lk(p->m);
            p->cv_job.wait(lk, [&] { return p->stop || p->published >= next; });
            if (p->published < next) return;
            j = p->job;
        }
        (void)hipEventSynchronize(c->ev_list[j.k]);            // the lists of missing rows are in pinned memory
        const int32_t* ranks = c->miss_pin[j.k];
        const int32_t* src = c->dma_evict ? c->src_pin[j.k] : nullptr;
        float* blk = c->arrive_pin[j.k];
        const float* host = c->host;
        for (int ch = 0; ch < j.nchunks; ++ch) {
            const int64_t r0 = ch * j.chunk, r1 = r0 + j.chunk < j.M ? r0 + j.chunk : j.M;
            const int64_t a = r0 + (r1 - r0) * t / T, b = r0 + (r1 - r0) * (t + 1) / T;
            for (int64_t r = a; r < b; ++r)
                if (!src || src[r] == -1) memcpy(blk + (size_t)r * c->D, host + (size_t)ranks[r] * c->D, rowb);
            if (p->chunk_left[ch].fetch_sub(1) == 1) {
                // the chunk is complete: over the link by DMA (copies on one stream run in the order they were enqueued;
                // which thread enqueues which chunk does not matter)
                if (hipMemcpyAsync(c->arrive[j.k] + (size_t)r0 * c->D, blk + (size_t)r0 * c->D, (size_t)(r1 - r0) * rowb,
                                   hipMemcpyHostToDevice, c->pf) != hipSuccess) { (void)hipGetLastError(); p->failed = 1; }
                if (p->chunks_sent.fetch_add(1) == j.nchunks - 1) {
                    if (hipEventRecord(c->ev_arrive[j.k], c->pf) != hipSuccess) { (void)hipGetLastError(); p->failed = 1; }
                    std::lock_guard<std::mutex> lk(p->m);
                    p->completed = next;
                    p->cv_done.notify_all();
                }
            }
        }
        {   // the next job reuses the chunk counters: not before every thread is through with this one
            std::unique_lock<std::mutex> lk(p->m);
            p->cv_done.wait(lk, [&] { return p->completed >= next || p->stop; });
        }
    }
}

int gather_create(fc_cache* c, int threads) {
    GatherPool* p = new (std::nothrow) GatherPool();
    if (!p) return FC_ERR_INVALID_ARG;
    p->c = c;
    for (auto& x : p->chunk_left) x = 0;
    c->gpool = p;
    try {
        for (int t = 0; t < threads; ++t) p->threads.emplace_back(gather_worker, p, t, threads);
    } catch (...) {
        gather_destroy(c);
        return FC_ERR_INVALID_ARG;
    }
    return FC_OK;
}

void gather_destroy(fc_cache* c) {
    GatherPool* p = c->gpool;
    if (!p) return;
    {
        std::lock_guard<std::mutex> lk(p->m);
        p->stop = true;
    }
    p->cv_job.notify_all();
    p->cv_done.notify_all();
    for (std::thread& t : p->threads) if (t.joinable()) t.join();
    delete p;
    c->gpool = nullptr;
}

// Blocks until the latest job's rows are all handed to the DMA engine and ev_arrive of its list set is recorded.
int gather_wait(fc_cache* c) {
    GatherPool* p = c->gpool;
    if (!p) return FC_OK;
    std::unique_lock<std::mutex> lk(p->m);
    p->cv_done.wait(lk, [&] { return p->completed >= p->published; });
    return p->failed.exchange(0) ? FC_ERR_HIP : FC_OK;
}

// cache_plan_next: the planned batch's M missing rows (list set k = c->lset) by the DMA path.  Enqueues the list copies
// on the fetch stream and wakes the pool; returns at once.
int gather_start(fc_cache* c, int64_t M) {
    GatherPool* p = c->gpool;
    const int k = c->lset;
    FC_TRY(gather_wait(c));                                    // one job at a time (cache_advance has waited already)
    FC_HIP(hipStreamWaitEvent(c->pf, c->ev_emit_done, 0));
    // without the DMA evict transmitter there are no transit marks: rows evicted by the current batch are stored into the
    // host table by a kernel, which has to be through before any of them may be gathered (the lists land after it)
    if (!c->dma_evict && c->pf_dep) FC_HIP(hipStreamWaitEvent(c->pf, c->pf_dep, 0));
    FC_HIP(hipMemcpyAsync(c->miss_pin[k], c->miss_ranks, (size_t)M * 4, hipMemcpyDeviceToHost, c->pf));
    if (c->dma_evict) FC_HIP(hipMemcpyAsync(c->src_pin[k], c->fill_src, (size_t)M * 4, hipMemcpyDeviceToHost, c->pf));
    FC_HIP(hipEventRecord(c->ev_list[k], c->pf));
    int64_t chunk = 4096;
    if (cdiv(M, chunk) > GATHER_MAX_CHUNKS) chunk = cdiv(M, GATHER_MAX_CHUNKS);
    {
        std::lock_guard<std::mutex> lk(p->m);
        p->job.k = k; p->job.M = M; p->job.chunk = chunk; p->job.nchunks = (int)cdiv(M, chunk);
        for (int i = 0; i < p->job.nchunks; ++i) p->chunk_left[i] = (int)p->threads.size();
        p->chunks_sent = 0;
        p->published += 1;
    }
    p->cv_job.notify_all();
    return FC_OK;
}

}  // namespace fc
