// Memory-backed slow tier paced on the host (see paced_pool.h).
#include "paced_pool.h"

#include <sys/prctl.h>

#include <algorithm>

namespace tio {

void PacedPool::guard(const char *what, hipError_t e) {
    if (e != hipSuccess) throw EngineError{std::string(what) + ": " + hipGetErrorString(e)};
}

PacedPool::PacedPool(hipStream_t d2h, hipStream_t h2d, uint64_t bytes_per_s) : bw_(bytes_per_s) {
    stream_[0] = d2h;
    stream_[1] = h2d;
    shared_ = d2h == h2d;
    const int n = shared_ ? 1 : 2;
    for (int i = 0; i < n; ++i) guard("hipEventCreate", hipEventCreateWithFlags(&chan_[i].copied, hipEventDisableTiming));
    int dev = 0;
    (void)hipGetDevice(&dev);
    for (int i = 0; i < n; ++i) {
        chan_[i].thread = std::thread([this, dev, i] {
            try {
                guard("hipSetDevice", hipSetDevice(dev));
                (void)::prctl(PR_SET_TIMERSLACK, 1000UL);       // sleeps that end within microseconds of their deadline
                run(i);
            } catch (const EngineError &e) {
                std::lock_guard<std::mutex> lk(mu_);
                if (error_.empty()) error_ = e.msg;
                cv_.notify_all();
            } catch (const std::exception &e) {
                std::lock_guard<std::mutex> lk(mu_);
                if (error_.empty()) error_ = e.what();
                cv_.notify_all();
            }
        });
    }
}

PacedPool::~PacedPool() {
    {
        std::lock_guard<std::mutex> lk(mu_);
        stop_ = true;
    }
    cv_.notify_all();
    for (auto &c : chan_) if (c.thread.joinable()) c.thread.join();
    for (auto &c : chan_) if (c.copied) (void)hipEventDestroy(c.copied);
}

void PacedPool::set_pairs(int n) {
    std::lock_guard<std::mutex> lk(mu_);
    off_done_.assign((size_t)std::max(n, 0), 0);
    pre_done_.assign((size_t)std::max(n, 0), 0);
}

void PacedPool::check() {
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw EngineError{error_};
}

uint64_t PacedPool::submit_offload(int pair, hipEvent_t after, const void *dev, uint64_t where, uint64_t bytes,
                                   hipEvent_t done, hipEvent_t t0, hipEvent_t t1) {
    auto r = std::make_shared<Request>();
    r->pair = pair; r->after = after; r->done = done; r->t0 = t0; r->t1 = t1;
    r->dev = (uint8_t *)dev; r->slot = (uint8_t *)(uintptr_t)where; r->bytes = bytes;
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw EngineError{error_};
    if (pair < 0 || (size_t)pair >= off_done_.size() || !bytes || !where) throw EngineError{"bad offload request"};
    r->seq = ++submitted_[0];
    chan_[0].queue.push_back(r);
    cv_.notify_all();
    return r->seq;
}

uint64_t PacedPool::submit_prefetch(int pair, hipEvent_t after, void *dev, uint64_t where, uint64_t bytes, Dep written,
                                    std::vector<Dep> landed, std::vector<hipEvent_t> after_more, hipEvent_t done,
                                    hipEvent_t t0, hipEvent_t t1) {
    auto r = std::make_shared<Request>();
    r->prefetch = true;
    r->pair = pair; r->after = after; r->done = done; r->t0 = t0; r->t1 = t1;
    r->dev = (uint8_t *)dev; r->slot = (uint8_t *)(uintptr_t)where; r->bytes = bytes;
    r->written = written; r->landed = std::move(landed); r->after_more = std::move(after_more);
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw EngineError{error_};
    if (pair < 0 || (size_t)pair >= pre_done_.size() || !bytes || !where) throw EngineError{"bad prefetch request"};
    r->seq = ++submitted_[1];
    chan_[shared_ ? 0 : 1].queue.push_back(r);
    cv_.notify_all();
    return r->seq;
}

void PacedPool::wait_table(const std::vector<uint64_t> &tab, int pair, uint64_t seq) {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return stop_ || !error_.empty() || tab[pair] >= seq; });
    if (!error_.empty()) throw EngineError{error_};
    if (tab[pair] < seq) throw EngineError{"the engine was stopped"};
}
// the emulated transfer is one event: recorded, out of the arena and complete on the slow tier at once
void PacedPool::wait_offload_recorded(int pair, uint64_t seq) { wait_table(off_done_, pair, seq); }
void PacedPool::wait_offload_landed(int pair, uint64_t seq) { wait_table(off_done_, pair, seq); }
void PacedPool::wait_offload_written(int pair, uint64_t seq) { wait_table(off_done_, pair, seq); }
void PacedPool::wait_prefetch_recorded(int pair, uint64_t seq) { wait_table(pre_done_, pair, seq); }

void PacedPool::wait_consumed(int dir, uint64_t seq) {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return !error_.empty() || consumed_[dir] >= seq; });
    if (!error_.empty()) throw EngineError{error_};
}

void PacedPool::drain() {
    {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [&] { return !error_.empty() || (completed_[0] == submitted_[0] && completed_[1] == submitted_[1]); });
        if (!error_.empty()) throw EngineError{error_};
    }
    guard("hipStreamSynchronize", hipStreamSynchronize(stream_[0]));
    guard("hipStreamSynchronize", hipStreamSynchronize(stream_[1]));
}

void PacedPool::wait_dep(const Dep &d, bool written) {
    if (!d.seq) return;
    MigrationEngine *e = d.eng ? d.eng : this;
    if (written) e->wait_offload_written(d.pair, d.seq); else e->wait_offload_landed(d.pair, d.seq);
}

void PacedPool::run(int ch) {
    Channel &c = chan_[ch];
    for (;;) {
        std::shared_ptr<Request> r;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_.wait(lk, [&] { return stop_ || !error_.empty() || !c.queue.empty(); });
            if (stop_ || !error_.empty()) return;
            r = c.queue.front();
            c.queue.pop_front();
        }
        const int dir = r->prefetch ? 1 : 0;
        hipStream_t s = stream_[dir];
        // dependencies: the transfer cannot begin before all of them
        if (r->prefetch) {
            wait_dep(r->written, true);
            for (const Dep &d : r->landed) wait_dep(d, false);
        }
        guard("hipEventSynchronize", hipEventSynchronize(r->after));
        for (hipEvent_t e : r->after_more) guard("hipEventSynchronize", hipEventSynchronize(e));
        {
            std::lock_guard<std::mutex> lk(mu_);
            if (stop_) return;
            consumed_[dir] = r->seq;
            cv_.notify_all();
        }
        const Clock::time_point begin = std::max(Clock::now(), c.free_at);
        if (r->t0) guard("hipEventRecord", hipEventRecord(r->t0, s));
        // the slot is pinned host memory or device memory: the runtime picks the engine from the addresses
        guard("hipMemcpyAsync", r->prefetch ? hipMemcpyAsync(r->dev, r->slot, r->bytes, hipMemcpyDefault, s)
                                            : hipMemcpyAsync(r->slot, r->dev, r->bytes, hipMemcpyDefault, s));
        guard("hipEventRecord", hipEventRecord(c.copied, s));
        guard("hipEventSynchronize", hipEventSynchronize(c.copied));
        // the copy itself ran at the speed of the link; completion is signalled when the emulated channel is done
        const uint64_t bw = bw_.load();
        Clock::time_point end = Clock::now();
        if (bw) {
            const auto emulated = begin + std::chrono::nanoseconds((int64_t)((double)r->bytes / (double)bw * 1e9));
            if (emulated > end) {
                const auto spin = std::chrono::microseconds(30);
                if (emulated - end > spin) std::this_thread::sleep_until(emulated - spin);
                while (Clock::now() < emulated) {}
                end = emulated;
            }
        }
        c.free_at = end;
        if (poison_ && !r->prefetch) poison_(s, r->dev, r->bytes);
        if (r->t1) guard("hipEventRecord", hipEventRecord(r->t1, s));
        guard("hipEventRecord", hipEventRecord(r->done, s));
        std::lock_guard<std::mutex> lk(mu_);
        (r->prefetch ? pre_done_ : off_done_)[r->pair] = r->seq;
        ++completed_[dir];
        cv_.notify_all();
    }
}

}  // namespace tio
