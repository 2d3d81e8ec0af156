// Host side of the DMA evict transmitter, GPU-facing half: the scatter pool of scatter_pool.h with hooks that wait for
// a block's device -> host copy (an event on the side stream) and copy its rows into the frequency-ordered host table
// (paper Section 4.3, data transmitter).
#include "fc_internal.h"
#include "scatter_pool.h"

#include <string.h>

#include <new>

namespace fc {

struct EvictHooks {
    fc_cache* c;
    void thread_start() const { (void)hipSetDevice(c->device); }
    void wait_landed(int buf) const { (void)hipEventSynchronize(c->ev_d2h[buf]); }   // block and rank list are in pinned memory
    void scatter(int buf, int64_t a, int64_t b) const {
        const size_t rowb = (size_t)c->D * 4;
        const float* blk = c->blk_pin[buf];
        const int32_t* vr = c->vrank_pin[buf];
        float* host = c->host;
        for (int64_t r = a; r < b; ++r) memcpy(host + (size_t)vr[r] * c->D, blk + (size_t)r * c->D, rowb);
    }
};

struct ScatterPool : BlockScatterPool<DMA_BLOCKS, EvictHooks> {
    using BlockScatterPool<DMA_BLOCKS, EvictHooks>::BlockScatterPool;
};

int pool_create(fc_cache* c, int threads) {
    try {
        c->pool = new ScatterPool(EvictHooks{c}, threads);
    } catch (...) {
        c->pool = nullptr;
        return FC_ERR_INVALID_ARG;
    }
    return FC_OK;
}

void pool_destroy(fc_cache* c) {
    delete c->pool;
    c->pool = nullptr;
}

void pool_publish(fc_cache* c, int buf, int64_t rows) { (void)c->pool->publish(buf, rows); }

void pool_wait(fc_cache* c, uint64_t seq) {
    if (c->pool) c->pool->wait(seq);
}

uint64_t pool_published(fc_cache* c) { return c->pool ? c->pool->published() : 0; }

}  // namespace fc
