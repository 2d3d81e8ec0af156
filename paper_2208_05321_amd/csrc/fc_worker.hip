// Host side of the DMA evict transmitter: a small pool of threads that scatters evicted-row blocks, once their
// device -> host copy has landed in pinned memory, into the frequency-ordered host table
// (paper Section 4.3, data transmitter: rows travel as one block and are put in their places on the receiving side).
// Blocks are numbered 1, 2, ... in hand-over order and scattered one after the other, so a
// row evicted twice ends with its newer value.
#include "fc_internal.h"

#include <atomic>
#include <condition_variable>
#include <mutex>
#include <string.h>
#include <thread>
#include <vector>

namespace fc {

struct ScatterPool {
    std::vector<std::thread> threads;
    std::mutex m;
    std::condition_variable cv_job, cv_done;
    uint64_t published = 0, completed = 0;
    struct Job { int buf; int64_t rows; } jobs[DMA_BLOCKS] = {};
    std::atomic<int> remaining[DMA_BLOCKS];
    bool stop = false;
};

static void worker(fc_cache* c, ScatterPool* p, int k, int K) {
    (void)hipSetDevice(c->device);
    const size_t rowb = (size_t)c->D * 4;
    for (uint64_t next = 1;; ++next) {
        ScatterPool::Job j;
        {
            std::unique_lock<std::mutex> lk(p->m);
            p->cv_job.wait(lk, [&] { return p->stop || p->published >= next; });
            if (p->published < next) return;       // stop requested and nothing left to do
            j = p->jobs[next % DMA_BLOCKS];
            // blocks land strictly one after the other: a row evicted again two batches later must not be
            // overtaken by its older copy in the hands of a slower thread
            p->cv_done.wait(lk, [&] { return p->completed + 1 >= next; });
        }
        (void)hipEventSynchronize(c->ev_d2h[j.buf]);   // the block and its rank list are in pinned memory
        const int64_t a = j.rows * k / K, b = j.rows * (k + 1) / K;
        const float* blk = c->blk_pin[j.buf];
        const int32_t* vr = c->vrank_pin[j.buf];
        float* host = c->host;
        for (int64_t r = a; r < b; ++r) memcpy(host + (size_t)vr[r] * c->D, blk + (size_t)r * c->D, rowb);
        if (p->remaining[next % DMA_BLOCKS].fetch_sub(1) == 1) {
            std::lock_guard<std::mutex> lk(p->m);
            p->completed = next;
            p->cv_done.notify_all();
        }
    }
}

int pool_create(fc_cache* c, int threads) {
    ScatterPool* p = new (std::nothrow) ScatterPool();
    if (!p) return FC_ERR_INVALID_ARG;
    for (auto& r : p->remaining) r = 0;
    c->pool = p;
    try {
        for (int k = 0; k < threads; ++k) p->threads.emplace_back(worker, c, p, k, threads);
    } catch (...) {
        pool_destroy(c);
        return FC_ERR_INVALID_ARG;
    }
    return FC_OK;
}

void pool_destroy(fc_cache* c) {
    ScatterPool* p = c->pool;
    if (!p) return;
    {
        std::lock_guard<std::mutex> lk(p->m);
        p->stop = true;
    }
    p->cv_job.notify_all();
    for (std::thread& t : p->threads) if (t.joinable()) t.join();
    delete p;
    c->pool = nullptr;
}

void pool_publish(fc_cache* c, int buf, int64_t rows) {
    ScatterPool* p = c->pool;
    std::lock_guard<std::mutex> lk(p->m);
    const uint64_t seq = p->published + 1;
    p->jobs[seq % DMA_BLOCKS] = {buf, rows};
    p->remaining[seq % DMA_BLOCKS] = (int)p->threads.size();
    p->published = seq;
    p->cv_job.notify_all();
}

void pool_wait(fc_cache* c, uint64_t seq) {
    ScatterPool* p = c->pool;
    if (!p) return;
    std::unique_lock<std::mutex> lk(p->m);
    p->cv_done.wait(lk, [&] { return p->completed >= seq; });
}

uint64_t pool_published(fc_cache* c) {
    ScatterPool* p = c->pool;
    if (!p) return 0;
    std::lock_guard<std::mutex> lk(p->m);
    return p->published;
}

}  // namespace fc
