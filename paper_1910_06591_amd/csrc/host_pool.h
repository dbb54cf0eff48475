// A few persistent host threads for the library's large host-side copies (frames into pinned staging rows, the
// flat weight vector into its pinned staging buffer): a copy of several MB is memory-bound on one core at
// ~10 GB/s, and starting threads per call costs as much as the copy saves.  run(n, fn) calls fn(0) .. fn(n-1)
// once each, fn(0) on the calling thread, and returns when all are done.  One caller at a time per pool.
#pragma once
#include <condition_variable>
#include <cstring>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

namespace seedinf {

class HostPool {
public:
    explicit HostPool(int workers)
    {
        for (int i = 0; i < workers; ++i) th_.emplace_back([this, i] { loop(i + 1); });
    }
    ~HostPool()
    {
        {
            std::lock_guard<std::mutex> l(m_);
            stop_ = true;
            ++gen_;
        }
        cv_.notify_all();
        for (auto& t : th_) t.join();
    }
    HostPool(const HostPool&) = delete;
    HostPool& operator=(const HostPool&) = delete;
    int size() const { return (int)th_.size() + 1; }

    void run(int n, const std::function<void(int)>& fn)
    {
        if (n <= 1 || th_.empty()) {
            for (int i = 0; i < n; ++i) fn(i);
            return;
        }
        {
            std::lock_guard<std::mutex> l(m_);
            fn_ = &fn;
            n_ = n;
            pending_ = (int)th_.size();
            ++gen_;
        }
        cv_.notify_all();
        const int stride = size();
        for (int i = 0; i < n; i += stride) fn(i);           // the caller takes every stride-th item, starting with 0
        std::unique_lock<std::mutex> l(m_);
        done_.wait(l, [this] { return pending_ == 0; });
        fn_ = nullptr;
    }

private:
    void loop(int me)
    {
        unsigned long seen = 0;
        for (;;) {
            const std::function<void(int)>* fn;
            int n;
            {
                std::unique_lock<std::mutex> l(m_);
                cv_.wait(l, [&] { return gen_ != seen; });
                seen = gen_;
                if (stop_) return;
                fn = fn_;
                n = n_;
            }
            const int stride = size();
            for (int i = me; i < n; i += stride) (*fn)(i);
            {
                std::lock_guard<std::mutex> l(m_);
                if (--pending_ == 0) done_.notify_one();
            }
        }
    }
    std::vector<std::thread> th_;
    std::mutex m_;
    std::condition_variable cv_, done_;
    const std::function<void(int)>* fn_ = nullptr;
    int n_ = 0, pending_ = 0;
    unsigned long gen_ = 0;
    bool stop_ = false;
};

// memcpy of a large block, cut into pieces over the pool (pool == nullptr: a plain memcpy)
inline void pool_memcpy(HostPool* pool, void* dst, const void* src, size_t bytes)
{
    constexpr size_t PIECE = (size_t)1 << 20;
    const int n = (int)((bytes + PIECE - 1) / PIECE);
    if (n <= 1 || !pool) {
        memcpy(dst, src, bytes);
        return;
    }
    pool->run(n, [&](int i) {
        const size_t o = (size_t)i * PIECE;
        memcpy((char*)dst + o, (const char*)src + o, bytes - o < PIECE ? bytes - o : PIECE);
    });
}

}  // namespace seedinf
