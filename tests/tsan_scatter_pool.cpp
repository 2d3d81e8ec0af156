// Thread-sanitizer harness for the scatter pool of the DMA evict transmitter (csrc/scatter_pool.h), with the GPU left
// out: a mock "DMA engine" thread marks blocks as landed after a random delay, the pool's worker threads scatter them
// into a small table in which the same rows are written by block after block.  Checks: blocks complete strictly in
// hand-over order, a buffer is never reused before its previous block is complete, and the table ends as a sequential
// replay of the blocks would leave it (a row evicted twice keeps its newer value).  Built and run by
// tests/test_sanitizers.py with -fsanitize=thread; exit code 0 = all checks passed.
#include "scatter_pool.h"

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <random>

namespace {

constexpr int RING = 4;
constexpr int TABLE_ROWS = 96;      // few rows: consecutive blocks keep hitting the same ones
constexpr int MAX_ROWS = 64;

struct Block { int32_t rank[MAX_ROWS]; int64_t value[MAX_ROWS]; };

struct Shared {
    Block buf[RING];
    std::mutex m;
    std::condition_variable cv;
    bool landed[RING] = {};
    int64_t table[TABLE_ROWS] = {};
    std::atomic<int> busy[RING];     // 1 while a block in this buffer is between publish and completion
};

struct MockHooks {
    Shared* s;
    void thread_start() const {}
    void wait_landed(int b) const {
        std::unique_lock<std::mutex> lk(s->m);
        s->cv.wait(lk, [&] { return s->landed[b]; });
    }
    void scatter(int b, int64_t a, int64_t e) const {
        for (int64_t r = a; r < e; ++r) s->table[s->buf[b].rank[r]] = s->buf[b].value[r];
    }
};

}  // namespace

int main(int argc, char** argv) {
    const int blocks = argc > 1 ? atoi(argv[1]) : 300;
    const int threads = argc > 2 ? atoi(argv[2]) : 6;
    Shared sh;
    for (auto& b : sh.busy) b = 0;
    int64_t expect[TABLE_ROWS] = {};
    std::mt19937 rng(12345);
    int failures = 0;
    {
        fc::BlockScatterPool<RING, MockHooks> pool(MockHooks{&sh}, threads);
        std::vector<std::thread> dma;
        for (uint64_t seq = 1; seq <= (uint64_t)blocks; ++seq) {
            const int b = (int)(seq % RING);
            if (seq > RING) pool.wait(seq - RING);                       // the library's rule for reusing a buffer
            if (pool.completed() + RING < seq) { fprintf(stderr, "buffer %d reused before block %llu was complete\n", b, (unsigned long long)(seq - RING)); ++failures; }
            {
                std::lock_guard<std::mutex> lk(sh.m);
                sh.landed[b] = false;
            }
            const int rows = 1 + (int)(rng() % MAX_ROWS);
            // distinct ranks within a block (a batch evicts a row at most once), shared between blocks
            int perm[TABLE_ROWS];
            for (int i = 0; i < TABLE_ROWS; ++i) perm[i] = i;
            for (int i = 0; i < rows; ++i) { const int j = i + (int)(rng() % (TABLE_ROWS - i)); std::swap(perm[i], perm[j]); }
            for (int i = 0; i < rows; ++i) {
                sh.buf[b].rank[i] = perm[i];
                sh.buf[b].value[i] = (int64_t)seq * 1000 + i;
                expect[perm[i]] = (int64_t)seq * 1000 + i;
            }
            const uint64_t got = pool.publish(b, rows);
            if (got != seq) { fprintf(stderr, "publish returned %llu for block %llu\n", (unsigned long long)got, (unsigned long long)seq); ++failures; }
            const int delay_us = (int)(rng() % 300);
            dma.emplace_back([&sh, b, delay_us] {                         // the copy lands some time after the hand-over
                std::this_thread::sleep_for(std::chrono::microseconds(delay_us));
                std::lock_guard<std::mutex> lk(sh.m);
                sh.landed[b] = true;
                sh.cv.notify_all();
            });
            if (dma.size() > 64) { for (auto& t : dma) t.join(); dma.clear(); }
        }
        pool.wait((uint64_t)blocks);
        if (pool.completed() != (uint64_t)blocks || pool.published() != (uint64_t)blocks) { fprintf(stderr, "counts differ at the end\n"); ++failures; }
        for (auto& t : dma) t.join();
    }   // the destructor stops and joins the workers
    for (int r = 0; r < TABLE_ROWS; ++r)
        if (sh.table[r] != expect[r]) { fprintf(stderr, "row %d holds %lld, a sequential replay gives %lld\n", r, (long long)sh.table[r], (long long)expect[r]); ++failures; }
    if (failures) { fprintf(stderr, "%d checks failed\n", failures); return 1; }
    printf("ok: %d blocks, %d threads\n", blocks, threads);
    return 0;
}
