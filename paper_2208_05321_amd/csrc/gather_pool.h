// Host side of the DMA miss path, free of any GPU runtime call so that it can be built and exercised on its own (the
// thread sanitizer run in tests/ uses it with mocked copies): a small pool of threads that gathers the rows of one job
// (a planned batch's missing rows) out of the host table into a pinned block, chunk by chunk, and hands every chunk to
// the copy engine as soon as all threads are through with it (paper Section 4.3, data transmitter: rows are collected
// into one block on the sending side and travel as a block).
//
// One job is outstanding at a time: start() waits for the previous one.  Every thread takes a share of every chunk; the
// thread that finishes a chunk last sends it, and the one that sends the last chunk of the job signals the job's end.
#pragma once

#include <stdint.h>

#include <atomic>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

namespace fc {

// Hooks:  void thread_start();                             once per worker thread
//         void wait_lists(int k);                          returns once the row lists of list set k are in host memory
//         void gather(int k, int64_t a, int64_t b);        rows [a, b) of the job into the pinned block of set k
//         bool send(int k, int64_t r0, int64_t r1);        rows [r0, r1) of that block to the device; false = failed
//         bool finish(int k);                              every chunk has been sent: mark the job's arrival; false = failed
template <int MAX_CHUNKS, class Hooks>
class ChunkGatherPool {
 public:
    ChunkGatherPool(const Hooks& hooks, int threads) : hooks_(hooks) {
        for (auto& x : chunk_left_) x = 0;
        try {
            for (int t = 0; t < threads; ++t) threads_.emplace_back([this, t, threads] { work(t, threads); });
        } catch (...) {
            shutdown();
            throw;
        }
    }
    ~ChunkGatherPool() { shutdown(); }
    ChunkGatherPool(const ChunkGatherPool&) = delete;
    ChunkGatherPool& operator=(const ChunkGatherPool&) = delete;

    // M rows of list set k, in chunks of at least min_chunk rows (at most MAX_CHUNKS chunks); returns at once
    // (a failure noted by an earlier job stays noted until the caller's next wait())
    void start(int k, int64_t M, int64_t min_chunk) {
        if (M <= 0) return;                 // nothing to gather: no job (a job with no chunk would never be signalled)
        {
            std::unique_lock<std::mutex> lk(m_);
            cv_done_.wait(lk, [&] { return completed_ >= published_; });
        }
        int64_t chunk = min_chunk;
        if ((M + chunk - 1) / chunk > MAX_CHUNKS) chunk = (M + MAX_CHUNKS - 1) / MAX_CHUNKS;
        std::lock_guard<std::mutex> lk(m_);
        job_.k = k; job_.M = M; job_.chunk = chunk; job_.nchunks = (int)((M + chunk - 1) / chunk);
        for (int i = 0; i < job_.nchunks; ++i) chunk_left_[i] = (int)threads_.size();
        chunks_sent_ = 0;
        published_ += 1;
        cv_job_.notify_all();
    }
    // until the latest job's chunks have all been sent and finish() has run; false if any send / finish failed since the last wait
    bool wait() {
        std::unique_lock<std::mutex> lk(m_);
        cv_done_.wait(lk, [&] { return completed_ >= published_; });
        return failed_.exchange(0) == 0;
    }
    int threads() const { return (int)threads_.size(); }

 private:
    struct Job { int k = 0; int64_t M = 0, chunk = 0; int nchunks = 0; };

    void shutdown() {
        {
            std::lock_guard<std::mutex> lk(m_);
            stop_ = true;
        }
        cv_job_.notify_all();
        cv_done_.notify_all();
        for (std::thread& t : threads_) if (t.joinable()) t.join();
        threads_.clear();
    }

    void work(int t, int T) {
        hooks_.thread_start();
        for (uint64_t next = 1;; ++next) {
            Job j;
            {
                std::unique_lock<std::mutex> lk(m_);
                cv_job_.wait(lk, [&] { return stop_ || published_ >= next; });
                if (published_ < next) return;
                j = job_;
            }
            hooks_.wait_lists(j.k);
            for (int ch = 0; ch < j.nchunks; ++ch) {
                const int64_t r0 = ch * j.chunk, r1 = r0 + j.chunk < j.M ? r0 + j.chunk : j.M;
                hooks_.gather(j.k, r0 + (r1 - r0) * t / T, r0 + (r1 - r0) * (t + 1) / T);
                if (chunk_left_[ch].fetch_sub(1) == 1) {
                    // the chunk is complete (the counter orders the other threads' rows before this point): send it;
                    // which thread sends which chunk does not matter, copies on one stream run in the order they are enqueued
                    if (!hooks_.send(j.k, r0, r1)) failed_ = 1;
                    if (chunks_sent_.fetch_add(1) == j.nchunks - 1) {
                        if (!hooks_.finish(j.k)) failed_ = 1;
                        std::lock_guard<std::mutex> lk(m_);
                        completed_ = next;
                        cv_done_.notify_all();
                    }
                }
            }
            {   // the next job reuses the chunk counters: not before every thread is through with this one
                std::unique_lock<std::mutex> lk(m_);
                cv_done_.wait(lk, [&] { return completed_ >= next || stop_; });
            }
        }
    }

    Hooks hooks_;
    std::vector<std::thread> threads_;
    std::mutex m_;
    std::condition_variable cv_job_, cv_done_;
    uint64_t published_ = 0, completed_ = 0;     // jobs are numbered 1, 2, ...
    Job job_;
    std::atomic<int> chunk_left_[MAX_CHUNKS];    // threads still working on chunk i
    std::atomic<int> chunks_sent_{0};
    std::atomic<int> failed_{0};
    bool stop_ = false;
};

}  // namespace fc
