// Thread-sanitizer harness for the gather pool of the DMA miss path (csrc/gather_pool.h), with the GPU left out: the "host
// table" is an array of row values, the list of missing rows "lands" after a random delay (a mock copy thread), send()
// copies a chunk of the pinned block into a mock device block, finish() marks the arrival.  Checks: every row of a job
// is gathered exactly once and sent exactly once, a chunk is sent only when all of its rows have been gathered, finish()
// runs once per job and after every send, wait() returns only then, the device block holds the right rows, jobs of very
// different sizes (1 row .. more than MAX_CHUNKS * min_chunk) follow each other, a failed send is reported by the next
// wait() and by that one only.  Built and run by tests/test_sanitizers.py with -fsanitize=thread; exit code 0 = all passed.
#include "gather_pool.h"

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <random>

namespace {

constexpr int MAX_CHUNKS = 8;
constexpr int64_t MAX_ROWS = 6000;
constexpr int64_t TABLE_ROWS = 50000;

struct Shared {
    int64_t table[TABLE_ROWS];
    int32_t ranks[2][MAX_ROWS];
    int64_t pinned[2][MAX_ROWS], device[2][MAX_ROWS];
    std::atomic<int> gathered[MAX_ROWS], sent[MAX_ROWS];
    std::atomic<int> finished{0}, sends{0}, bad{0};
    std::atomic<int> fail_next_send{0};
    std::mutex m;
    std::condition_variable cv;
    bool landed[2] = {false, false};
};

struct MockHooks {
    Shared* s;
    void thread_start() const {}
    void wait_lists(int k) const {
        std::unique_lock<std::mutex> lk(s->m);
        s->cv.wait(lk, [&] { return s->landed[k]; });
    }
    void gather(int k, int64_t a, int64_t b) const {
        for (int64_t r = a; r < b; ++r) {
            s->pinned[k][r] = s->table[s->ranks[k][r]];
            s->gathered[r].fetch_add(1);
        }
    }
    bool send(int k, int64_t r0, int64_t r1) const {
        if (s->finished.load() != 0) s->bad.fetch_add(1);                  // a send after the job was declared complete
        for (int64_t r = r0; r < r1; ++r) {
            if (s->gathered[r].load() != 1) s->bad.fetch_add(1);           // sent before (or without) being gathered
            s->device[k][r] = s->pinned[k][r];
            s->sent[r].fetch_add(1);
        }
        s->sends.fetch_add(1);
        return s->fail_next_send.exchange(0) == 0;
    }
    bool finish(int) const {
        s->finished.fetch_add(1);
        return true;
    }
};

}  // namespace

int main(int argc, char** argv) {
    const int jobs = argc > 1 ? atoi(argv[1]) : 200;
    const int threads = argc > 2 ? atoi(argv[2]) : 6;
    static Shared sh;
    for (int64_t i = 0; i < TABLE_ROWS; ++i) sh.table[i] = i * 7 + 1;
    std::mt19937 rng(4321);
    int failures = 0;
    {
        fc::ChunkGatherPool<MAX_CHUNKS, MockHooks> pool(MockHooks{&sh}, threads);
        std::vector<std::thread> copies;
        for (int job = 0; job < jobs; ++job) {
            const int k = job & 1;
            const int kind = (int)(rng() % 4);
            const int64_t M = kind == 0 ? 1 + (int64_t)(rng() % 5) : kind == 1 ? MAX_ROWS - (int64_t)(rng() % 3) : 1 + (int64_t)(rng() % MAX_ROWS);
            // the previous job is complete (wait() below), so its lists and counters may be rewritten
            for (int64_t r = 0; r < M; ++r) { sh.ranks[k][r] = (int32_t)(rng() % TABLE_ROWS); sh.gathered[r] = 0; sh.sent[r] = 0; }
            sh.finished = 0; sh.sends = 0;
            {
                std::lock_guard<std::mutex> lk(sh.m);
                sh.landed[k] = false;
            }
            const bool inject = job % 17 == 5;
            if (inject) sh.fail_next_send = 1;
            pool.start(k, M, 256);
            const int delay_us = (int)(rng() % 200);
            copies.emplace_back([k, delay_us] {                       // the list copy lands some time after the job was posted
                std::this_thread::sleep_for(std::chrono::microseconds(delay_us));
                std::lock_guard<std::mutex> lk(sh.m);
                sh.landed[k] = true;
                sh.cv.notify_all();
            });
            const bool ok = pool.wait();
            if (ok == inject) { fprintf(stderr, "job %d: wait() returned %d, a failure was %sinjected\n", job, (int)ok, inject ? "" : "not "); ++failures; }
            if (sh.finished.load() != 1) { fprintf(stderr, "job %d: finish ran %d times\n", job, sh.finished.load()); ++failures; }
            const int64_t chunk = (M + 255) / 256 > MAX_CHUNKS ? (M + MAX_CHUNKS - 1) / MAX_CHUNKS : 256;
            if (sh.sends.load() != (int)((M + chunk - 1) / chunk)) { fprintf(stderr, "job %d: %d sends for %lld rows\n", job, sh.sends.load(), (long long)M); ++failures; }
            for (int64_t r = 0; r < M; ++r) {
                if (sh.gathered[r].load() != 1 || sh.sent[r].load() != 1) { fprintf(stderr, "job %d row %lld: gathered %d sent %d\n", job, (long long)r, sh.gathered[r].load(), sh.sent[r].load()); ++failures; break; }
                if (sh.device[k][r] != sh.table[sh.ranks[k][r]]) { fprintf(stderr, "job %d row %lld: wrong value\n", job, (long long)r); ++failures; break; }
            }
            if (copies.size() > 64) { for (auto& t : copies) t.join(); copies.clear(); }
        }
        if (!pool.wait()) { fprintf(stderr, "a failure reported twice\n"); ++failures; }
        pool.start(0, 0, 256);                                          // no rows: no job
        if (!pool.wait()) ++failures;
        for (auto& t : copies) t.join();
    }   // the destructor stops and joins the workers
    if (sh.bad.load()) { fprintf(stderr, "%d ordering violations\n", sh.bad.load()); ++failures; }
    if (failures) { fprintf(stderr, "%d checks failed\n", failures); return 1; }
    printf("ok: %d jobs, %d threads\n", jobs, threads);
    return 0;
}
