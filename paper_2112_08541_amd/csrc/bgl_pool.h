// Host thread pool of the host tier: plain C++ (no HIP), so that it can also be
// built and stress-tested on its own with a thread sanitizer.
#pragma once

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <cstdint>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

namespace bgl {

// A few host threads that run one job at a time: tasks 0..tasks-1, claimed in
// increasing order.  run() also works on the calling thread and returns when
// all tasks are done; start() returns at once, done_prefix() tells how many
// leading tasks are complete (the caller launches work on them meanwhile),
// help_one() lets the caller take a task itself when it has nothing else to do,
// and wait() ends the job.
class Pool {
public:
    using Fn = std::function<void(int64_t)>;

    explicit Pool(int threads)
    {
        for (int i = 0; i < std::max(threads, 1); ++i) workers_.emplace_back([this] { loop(); });
    }
    ~Pool()
    {
        {
            std::lock_guard<std::mutex> lk(m_);
            stop_ = true;
        }
        cv_.notify_all();
        for (auto &t : workers_) t.join();
    }
    int threads() const { return (int)workers_.size(); }

    void start(int64_t tasks, const Fn &fn)
    {
        if ((int64_t)done_.size() < tasks) done_ = std::vector<std::atomic<uint8_t>>((size_t)tasks);
        for (int64_t k = 0; k < tasks; ++k) done_[(size_t)k].store(0, std::memory_order_relaxed);
        prefix_ = 0;
        {
            std::lock_guard<std::mutex> lk(m_);
            fn_ = &fn;
            tasks_ = tasks;
            next_.store(0);
            busy_ = (int)workers_.size();
            ++gen_;
        }
        cv_.notify_all();
    }
    // number of leading tasks that are complete (their writes are visible to the caller)
    int64_t done_prefix()
    {
        while (prefix_ < tasks_ && done_[(size_t)prefix_].load(std::memory_order_acquire)) ++prefix_;
        return prefix_;
    }
    // Between start() and wait(): the calling thread runs one task that nobody has claimed yet.
    // False when none is left.
    bool help_one()
    {
        if (next_.load(std::memory_order_relaxed) >= tasks_) return false;
        const int64_t k = next_.fetch_add(1);
        if (k >= tasks_) return false;
        (*fn_)(k);
        done_[(size_t)k].store(1, std::memory_order_release);
        return true;
    }
    void wait()
    {
        std::unique_lock<std::mutex> lk(m_);
        idle_.wait(lk, [this] { return busy_ == 0; });
        fn_ = nullptr;
    }
    void run(int64_t tasks, const Fn &fn)
    {
        if (tasks <= 0) return;
        start(tasks, fn);
        work();
        wait();
    }

private:
    void work()
    {
        for (;;) {
            const int64_t k = next_.fetch_add(1);
            if (k >= tasks_) return;
            (*fn_)(k);
            done_[(size_t)k].store(1, std::memory_order_release);
        }
    }
    void loop()
    {
        uint64_t seen = 0;
        for (;;) {
            {
                std::unique_lock<std::mutex> lk(m_);
                cv_.wait(lk, [&] { return stop_ || gen_ != seen; });
                if (stop_) return;
                seen = gen_;
            }
            work();
            {
                std::lock_guard<std::mutex> lk(m_);
                if (--busy_ == 0) idle_.notify_one();
            }
        }
    }

    std::vector<std::thread> workers_;
    std::mutex m_;
    std::condition_variable cv_, idle_;
    const Fn *fn_ = nullptr;
    int64_t tasks_ = 0;
    std::atomic<int64_t> next_{0};
    std::vector<std::atomic<uint8_t>> done_;
    int64_t prefix_ = 0;
    int busy_ = 0;
    uint64_t gen_ = 0;
    bool stop_ = false;
};

}  // namespace bgl
