// Memory-backed slow tier paced on the host (see paced_pool.h).
#include "paced_pool.h"

#include <sys/prctl.h>

#include <algorithm>

namespace tio {

void PacedPool::guard(const char *what, hipError_t e) {
    if (e != hipSuccess) throw EngineError{std::string(what) + ": " + hipGetErrorString(e)};
}

PacedPool::PacedPool(hipStream_t d2h, hipStream_t h2d, uint64_t bytes_per_s, bool device_pool) : bw_(bytes_per_s) {
    kind_ = device_pool ? hipMemcpyDeviceToDeviceNoCU : hipMemcpyDefault;
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

void PacedPool::set_policy(uint64_t chunk_bytes, bool urgent_first, bool ready_queue) {
    std::lock_guard<std::mutex> lk(mu_);
    chunk_ = chunk_bytes;
    urgent_first_ = urgent_first;
    ready_queue_ = ready_queue;
}

uint64_t PacedPool::submit_offload(int pair, hipEvent_t after, const void *dev, uint64_t where, uint64_t bytes,
                                   hipEvent_t done, hipEvent_t t0, hipEvent_t t1, bool urgent) {
    auto r = std::make_shared<Request>();
    r->pair = pair; r->after = after; r->done = done; r->t0 = t0; r->t1 = t1; r->urgent = urgent;
    r->dev = (uint8_t *)dev; r->slot = (uint8_t *)(uintptr_t)where; r->bytes = bytes;
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw EngineError{error_};
    if (pair < 0 || (size_t)pair >= off_done_.size() || !bytes || !where) throw EngineError{"bad offload request"};
    r->seq = ++submitted_[0];
    unconsumed_[0].insert(r->seq);
    chan_[0].queue.push_back(r);
    cv_.notify_all();
    return r->seq;
}

uint64_t PacedPool::submit_prefetch(int pair, hipEvent_t after, void *dev, uint64_t where, uint64_t bytes, Dep written,
                                    std::vector<Dep> landed, std::vector<hipEvent_t> after_more, hipEvent_t done,
                                    hipEvent_t t0, hipEvent_t t1, bool urgent) {
    auto r = std::make_shared<Request>();
    r->prefetch = true;
    r->pair = pair; r->after = after; r->done = done; r->t0 = t0; r->t1 = t1; r->urgent = urgent;
    r->dev = (uint8_t *)dev; r->slot = (uint8_t *)(uintptr_t)where; r->bytes = bytes;
    r->written = written; r->landed = std::move(landed); r->after_more = std::move(after_more);
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw EngineError{error_};
    if (pair < 0 || (size_t)pair >= pre_done_.size() || !bytes || !where) throw EngineError{"bad prefetch request"};
    r->seq = ++submitted_[1];
    unconsumed_[1].insert(r->seq);
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
bool PacedPool::offload_landed_now(int pair, uint64_t seq) {
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw EngineError{error_};
    return off_done_[pair] >= seq;
}
bool PacedPool::offload_written_now(int pair, uint64_t seq) { return offload_landed_now(pair, seq); }

void PacedPool::wait_consumed(int dir, uint64_t seq) {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return !error_.empty() || !unconsumed_[dir].count(seq); });
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

int PacedPool::choose(const std::vector<uint8_t> &ready, const std::vector<uint8_t> &urgent, bool urgent_first, bool ready_queue) {
    if (ready.empty()) return -1;
    if (!ready_queue) return ready[0] ? 0 : -1;           // strictly the order submitted
    int first = -1;
    for (size_t i = 0; i < ready.size(); ++i) {
        if (!ready[i]) continue;
        if (!urgent_first) return (int)i;
        if (urgent[i]) return (int)i;
        if (first < 0) first = (int)i;
    }
    return first;
}

// Have the request's dependencies been met?  Never blocks.  Progress is remembered, so every event and table is asked
// only until it has answered yes once.  The compute-progress event comes first: the moment it is seen complete the
// caller may record it again for the next iteration (wait_consumed).
bool PacedPool::ready(Request &r) {
    auto seen = [&](hipEvent_t e) {
        const hipError_t q = hipEventQuery(e);
        if (q == hipSuccess) return true;
        if (q != hipErrorNotReady) guard("hipEventQuery", q);
        (void)hipGetLastError();
        return false;
    };
    if (!r.after_seen) {
        if (!seen(r.after)) return false;
        r.after_seen = true;
        std::lock_guard<std::mutex> lk(mu_);
        unconsumed_[r.prefetch ? 1 : 0].erase(r.seq);
        cv_.notify_all();
    }
    while (r.more_seen < r.after_more.size()) {
        if (!seen(r.after_more[r.more_seen])) return false;
        ++r.more_seen;
    }
    if (r.prefetch) {
        if (!r.written_seen) {
            if (r.written.seq) {
                MigrationEngine *e = r.written.eng ? r.written.eng : this;
                if (!e->offload_written_now(r.written.pair, r.written.seq)) return false;
            }
            r.written_seen = true;
        }
        while (r.landed_seen < r.landed.size()) {
            const Dep &d = r.landed[r.landed_seen];
            if (d.seq) {
                MigrationEngine *e = d.eng ? d.eng : this;
                if (!e->offload_landed_now(d.pair, d.seq)) return false;
            }
            ++r.landed_seen;
        }
    }
    return true;
}

void PacedPool::run(int ch) {
    Channel &c = chan_[ch];
    std::vector<std::shared_ptr<Request>> snap;
    std::vector<uint8_t> is_ready, is_urgent;
    for (;;) {
        uint64_t chunk;
        bool urgent_first, ready_queue;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_.wait(lk, [&] { return stop_ || !error_.empty() || !c.queue.empty(); });
            if (stop_ || !error_.empty()) return;
            snap.assign(c.queue.begin(), c.queue.end());
            chunk = chunk_; urgent_first = urgent_first_; ready_queue = ready_queue_;
        }
        // which of the queued requests could go now?  (every one is asked, so that compute-progress events are taken
        // over as early as possible, whichever request is served)
        is_ready.assign(snap.size(), 0);
        is_urgent.assign(snap.size(), 0);
        for (size_t i = 0; i < snap.size(); ++i) {
            is_ready[i] = ready(*snap[i]) ? 1 : 0;
            is_urgent[i] = snap[i]->urgent ? 1 : 0;
        }
        const int pick = choose(is_ready, is_urgent, urgent_first, ready_queue);
        if (pick < 0) {                                       // readiness depends on GPU events: look again shortly
            std::unique_lock<std::mutex> lk(mu_);
            if (stop_ || !error_.empty()) return;
            cv_.wait_for(lk, std::chrono::microseconds(20));
            continue;
        }
        Request &r = *snap[pick];
        const int dir = r.prefetch ? 1 : 0;
        hipStream_t s = stream_[dir];
        const uint64_t left = r.bytes - r.moved, n = chunk ? std::min(chunk, left) : left;
        const Clock::time_point begin = std::max(Clock::now(), c.free_at);
        if (r.moved == 0 && r.t0) guard("hipEventRecord", hipEventRecord(r.t0, s));
        // the slot is pinned host memory or device memory
        guard("hipMemcpyAsync", r.prefetch ? hipMemcpyAsync(r.dev + r.moved, r.slot + r.moved, n, kind_, s)
                                           : hipMemcpyAsync(r.slot + r.moved, r.dev + r.moved, n, kind_, s));
        guard("hipEventRecord", hipEventRecord(c.copied, s));
        guard("hipEventSynchronize", hipEventSynchronize(c.copied));
        // the copy itself ran at the speed of the link; the chunk counts as delivered when the emulated channel is done
        const uint64_t bw = bw_.load();
        Clock::time_point end = Clock::now();
        if (bw) {
            const auto emulated = begin + std::chrono::nanoseconds((int64_t)((double)n / (double)bw * 1e9));
            if (emulated > end) {
                const auto spin = std::chrono::microseconds(30);
                if (emulated - end > spin) std::this_thread::sleep_until(emulated - spin);
                while (Clock::now() < emulated) {}
                end = emulated;
            }
        }
        c.free_at = end;
        r.moved += n;
        if (r.moved < r.bytes) continue;
        if (poison_ && !r.prefetch) poison_(s, r.dev, r.bytes);
        if (r.t1) guard("hipEventRecord", hipEventRecord(r.t1, s));
        guard("hipEventRecord", hipEventRecord(r.done, s));
        // the tables below release prefetches into the vacated range on the other stream: the fill that poisons it must
        // have run by then (without poisoning nothing is pending here: the last chunk's copy has been waited for)
        if (poison_ && !r.prefetch) guard("hipEventSynchronize", hipEventSynchronize(r.done));
        std::lock_guard<std::mutex> lk(mu_);
        (r.prefetch ? pre_done_ : off_done_)[r.pair] = r.seq;
        ++completed_[dir];
        c.queue.erase(std::find(c.queue.begin(), c.queue.end(), snap[pick]));
        cv_.notify_all();
    }
}

}  // namespace tio
