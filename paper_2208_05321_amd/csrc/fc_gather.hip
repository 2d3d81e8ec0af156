// DMA miss path (FC_MISS_DMA): the paper's block transmitter for the host -> device direction (Section 4.3), pipelined.
// cache_plan_next copies the list of missing rows to the host; a small pool of host threads (gather_pool.h) gathers those
// rows out of the frequency-ordered host table into a pinned block, chunk by chunk, and as each chunk is complete hands it
// to the DMA engine (hipMemcpyAsync on the fetch stream) into the arrival block in HBM.  No compute unit reads host memory;
// cache_advance then copies the arrived rows into their slots as it does after the zero-copy fetch.  Rows whose newest
// copy is still in an evicted-row block (in transit) are left out here: cache_advance takes them from that block.
#include "fc_internal.h"
#include "gather_pool.h"

#include <string.h>

#include <new>

namespace fc {

constexpr int GATHER_MAX_CHUNKS = 64;

struct GatherHooks {
    fc_cache* c;
    void thread_start() const { (void)hipSetDevice(c->device); }
    void wait_lists(int k) const { (void)hipEventSynchronize(c->ev_list[k]); }      // the lists of missing rows are in pinned memory
    void gather(int k, int64_t a, int64_t b) const {
        const size_t rowb = (size_t)c->D * 4;
        const int32_t* ranks = c->miss_pin[k];
        const int32_t* src = c->dma_evict ? c->src_pin[k] : nullptr;
        float* blk = c->arrive_pin[k];
        for (int64_t r = a; r < b; ++r)
            if (!src || src[r] == -1) memcpy(blk + (size_t)r * c->D, c->host + (size_t)ranks[r] * c->D, rowb);
    }
    bool send(int k, int64_t r0, int64_t r1) const {
        if (hipMemcpyAsync(c->arrive[k] + (size_t)r0 * c->D, c->arrive_pin[k] + (size_t)r0 * c->D, (size_t)(r1 - r0) * c->D * 4,
                           hipMemcpyHostToDevice, c->pf) == hipSuccess) return true;
        (void)hipGetLastError();
        return false;
    }
    bool finish(int k) const {
        if (hipEventRecord(c->ev_arrive[k], c->pf) == hipSuccess) return true;
        (void)hipGetLastError();
        return false;
    }
};

struct GatherPool {
    ChunkGatherPool<GATHER_MAX_CHUNKS, GatherHooks> pool;
    GatherPool(fc_cache* c, int threads) : pool(GatherHooks{c}, threads) {}
};

int gather_create(fc_cache* c, int threads) {
    try {
        c->gpool = new GatherPool(c, threads);
    } catch (...) {
        c->gpool = nullptr;
        return FC_ERR_INVALID_ARG;
    }
    return FC_OK;
}

void gather_destroy(fc_cache* c) {
    delete c->gpool;            // stops and joins the threads
    c->gpool = nullptr;
}

// Blocks until the latest job's rows are all handed to the DMA engine and ev_arrive of its list set is recorded.
int gather_wait(fc_cache* c) {
    if (!c->gpool) return FC_OK;
    return c->gpool->pool.wait() ? FC_OK : FC_ERR_HIP;
}

// cache_plan_next: the planned batch's M missing rows (list set k = c->lset) by the DMA path.  Enqueues the list copies
// on the fetch stream and wakes the pool; returns at once.
int gather_start(fc_cache* c, int64_t M) {
    const int k = c->lset;
    FC_TRY(gather_wait(c));                                    // one job at a time (cache_advance has waited already)
    FC_HIP(hipStreamWaitEvent(c->pf, c->ev_emit_done, 0));
    // without the DMA evict transmitter there are no transit marks: rows evicted by the current batch are stored into the
    // host table by a kernel, which has to be through before any of them may be gathered (the lists land after it)
    if (!c->dma_evict && c->pf_dep) FC_HIP(hipStreamWaitEvent(c->pf, c->pf_dep, 0));
    FC_HIP(hipMemcpyAsync(c->miss_pin[k], c->miss_ranks, (size_t)M * 4, hipMemcpyDeviceToHost, c->pf));
    if (c->dma_evict) FC_HIP(hipMemcpyAsync(c->src_pin[k], c->fill_src, (size_t)M * 4, hipMemcpyDeviceToHost, c->pf));
    FC_HIP(hipEventRecord(c->ev_list[k], c->pf));
    c->gpool->pool.start(k, M, 4096);
    return FC_OK;
}

}  // namespace fc
