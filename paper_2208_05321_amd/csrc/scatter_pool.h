// Host side of the DMA evict transmitter, free of any GPU runtime call so that it can be built and exercised on its own
// (the thread sanitizer run in tests/ uses it with a mocked "block has landed" signal): a small pool of threads that
// takes evicted-row blocks in hand-over order and puts their rows in their places in the host table
// (paper Section 4.3, data transmitter: rows travel as one block and are scattered on the receiving side).
//
// Blocks are numbered 1, 2, ... as they are published.  Every thread takes a share of every block; block k+1 is not
// touched before block k is complete, so a row evicted twice ends with its newer value.  A block lives in one of RING
// buffers: the publisher may reuse buffer b only after the block that last used it is complete (wait()).
#pragma once

#include <stdint.h>

#include <atomic>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

namespace fc {

// Hooks:  void thread_start();                           once per worker thread
//         void wait_landed(int buf);                     returns once block buffer `buf` is complete in host memory
//         void scatter(int buf, int64_t a, int64_t b);   rows [a, b) of that block go to their places
template <int RING, class Hooks>
class BlockScatterPool {
 public:
    BlockScatterPool(const Hooks& hooks, int threads) : hooks_(hooks) {
        for (auto& r : remaining_) r = 0;
        try {
            for (int k = 0; k < threads; ++k) threads_.emplace_back([this, k, threads] { work(k, threads); });
        } catch (...) {
            shutdown();
            throw;
        }
    }
    ~BlockScatterPool() { shutdown(); }
    BlockScatterPool(const BlockScatterPool&) = delete;
    BlockScatterPool& operator=(const BlockScatterPool&) = delete;

    // block in buffer `buf` with `rows` rows; its number is returned
    uint64_t publish(int buf, int64_t rows) {
        std::lock_guard<std::mutex> lk(m_);
        const uint64_t seq = published_ + 1;
        jobs_[seq % RING] = {buf, rows};
        remaining_[seq % RING] = (int)threads_.size();
        published_ = seq;
        cv_job_.notify_all();
        return seq;
    }
    // until block number `seq` is in the host table
    void wait(uint64_t seq) {
        std::unique_lock<std::mutex> lk(m_);
        cv_done_.wait(lk, [&] { return completed_ >= seq; });
    }
    uint64_t published() {
        std::lock_guard<std::mutex> lk(m_);
        return published_;
    }
    uint64_t completed() {
        std::lock_guard<std::mutex> lk(m_);
        return completed_;
    }

 private:
    struct Job { int buf; int64_t rows; };

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

    void work(int k, int K) {
        hooks_.thread_start();
        for (uint64_t next = 1;; ++next) {
            Job j;
            {
                std::unique_lock<std::mutex> lk(m_);
                cv_job_.wait(lk, [&] { return stop_ || published_ >= next; });
                if (published_ < next) return;       // stop requested and nothing left to do
                j = jobs_[next % RING];
                // strictly one block after the other: a row evicted again later must not be overtaken by its older
                // copy in the hands of a slower thread
                cv_done_.wait(lk, [&] { return completed_ + 1 >= next; });
            }
            hooks_.wait_landed(j.buf);
            const int64_t a = j.rows * k / K, b = j.rows * (k + 1) / K;
            hooks_.scatter(j.buf, a, b);
            if (remaining_[next % RING].fetch_sub(1) == 1) {
                std::lock_guard<std::mutex> lk(m_);
                completed_ = next;
                cv_done_.notify_all();
            }
        }
    }

    Hooks hooks_;
    std::vector<std::thread> threads_;
    std::mutex m_;
    std::condition_variable cv_job_, cv_done_;
    uint64_t published_ = 0, completed_ = 0;
    Job jobs_[RING] = {};
    std::atomic<int> remaining_[RING];
    bool stop_ = false;
};

}  // namespace fc
