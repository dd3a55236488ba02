// A few host threads kept by a context for the main node's bookkeeping of many rounds
// (layer choice and decode-vector solves of ngc_coded_rounds).  Threads are created on first
// need and sleep on a condition variable between jobs: waking them costs a few microseconds
// each, creating them afresh per call some ten times that.  One job at a time; the caller
// starts it, does its own share, and waits.
#pragma once

#include <condition_variable>
#include <cstdint>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

class ngc_host_pool {
public:
    ngc_host_pool() = default;
    ngc_host_pool(const ngc_host_pool&) = delete;
    ngc_host_pool& operator=(const ngc_host_pool&) = delete;

    ~ngc_host_pool() {
        {
            std::lock_guard<std::mutex> lk(mu_);
            stop_ = true;
        }
        cv_work_.notify_all();
        for (auto& t : threads_)
            if (t.joinable()) t.join();
    }

    // Runs fn(1), ..., fn(count) on pool threads and returns at once; wait() returns when all
    // of them have.  fn must not throw.  No second start before wait().
    void start(int count, std::function<void(int)> fn) {
        if (count <= 0) return;
        std::unique_lock<std::mutex> lk(mu_);
        while ((int)threads_.size() < count) {
            // a thread created here takes part in the job being started: it starts out having
            // seen the generation before it
            const int idx = (int)threads_.size();
            const uint64_t seen = generation_;
            threads_.emplace_back([this, idx, seen] { loop(idx, seen); });
        }
        job_ = std::move(fn);
        want_ = count;
        active_ = count;
        ++generation_;
        lk.unlock();
        cv_work_.notify_all();
    }

    void wait() {
        std::unique_lock<std::mutex> lk(mu_);
        cv_done_.wait(lk, [this] { return active_ == 0; });
    }

private:
    void loop(int idx, uint64_t seen) {
        for (;;) {
            std::function<void(int)> job;
            {
                std::unique_lock<std::mutex> lk(mu_);
                cv_work_.wait(lk, [&] { return stop_ || generation_ != seen; });
                if (stop_) return;
                seen = generation_;
                if (idx >= want_) continue;
                job = job_;
            }
            job(idx + 1);
            {
                std::lock_guard<std::mutex> lk(mu_);
                --active_;
            }
            cv_done_.notify_all();
        }
    }

    std::vector<std::thread> threads_;
    std::mutex mu_;
    std::condition_variable cv_work_, cv_done_;
    std::function<void(int)> job_;
    uint64_t generation_ = 0;
    int want_ = 0, active_ = 0;
    bool stop_ = false;
};
