// Host threads of the page-cache path's memcpy hop (Sec. IV-B "Data Flow": pinned memory <-> page cache is a
// CPU memcpy): a pool that copies pieces handed to it and counts each piece down on the command's own counter.
// No GPU calls in here: the pool is exercised on its own, under ThreadSanitizer, by tests/test_workers_cpu.py.
#pragma once

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <mutex>
#include <thread>
#include <vector>

namespace kvb {

struct CopyTask {
    void *dst;
    const void *src;
    size_t bytes;
    std::atomic<int> *pending;
};

class Workers {
public:
    void start(int n)
    {
        if ((int)threads_.size() == n) return;
        stop();
        quit_ = false;
        for (int i = 0; i < n; ++i) threads_.emplace_back([this] { loop(); });
    }
    void stop()
    {
        {
            std::lock_guard<std::mutex> g(mu_);
            quit_ = true;
        }
        cv_.notify_all();
        for (auto &t : threads_) t.join();
        threads_.clear();
    }
    // All pieces of one command under one lock; sleeping threads are woken only if there are any, and no
    // more of them than there are pieces (the issuing thread pays for every wake-up call).
    void push(const CopyTask *t, int n)
    {
        int wake = 0;
        {
            std::lock_guard<std::mutex> g(mu_);
            for (int i = 0; i < n; ++i) q_.push_back(t[i]);
            queued_.store((int)q_.size(), std::memory_order_release);
            wake = std::min(n, sleeping_);
        }
        if (wake >= (int)threads_.size()) cv_.notify_all();
        else for (int i = 0; i < wake; ++i) cv_.notify_one();
    }
    int size() const { return (int)threads_.size(); }
    ~Workers() { stop(); }

private:
    void loop()
    {
        for (;;) {
            CopyTask t;
            // pieces arrive every few tens of microseconds while a call runs, and a sleeping thread takes about
            // that long to wake: poll the queue length for a short while before going to sleep
            for (int spin = 0; spin < kSpinsBeforeSleep && queued_.load(std::memory_order_acquire) == 0; ++spin) __builtin_ia32_pause();
            {
                std::unique_lock<std::mutex> g(mu_);
                if (q_.empty() && !quit_) {
                    ++sleeping_;
                    cv_.wait(g, [this] { return quit_ || !q_.empty(); });
                    --sleeping_;
                }
                if (q_.empty()) {
                    if (quit_) return;
                    continue;
                }
                t = q_.front();
                q_.pop_front();
                queued_.store((int)q_.size(), std::memory_order_release);
            }
            std::memcpy(t.dst, t.src, t.bytes);
            t.pending->fetch_sub(1, std::memory_order_release);
        }
    }
    std::vector<std::thread> threads_;
    std::deque<CopyTask> q_;
    std::mutex mu_;
    std::condition_variable cv_;
    bool quit_ = false;
    int sleeping_ = 0;  // threads inside cv_.wait (under mu_)
    std::atomic<int> queued_{0};  // queue length, readable without the lock
    static constexpr int kSpinsBeforeSleep = 4000;  // roughly 50-100 us
};

}  // namespace kvb
