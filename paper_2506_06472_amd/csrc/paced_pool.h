// Memory-backed slow tier with an emulated bandwidth (the stand-in for the paper's storage tier, and the
// host-memory tier of Section 3.2): the pool is pinned host memory or a device buffer outside the arena.
// Each direction is a thread that takes requests in order: it waits for the request's dependencies, starts
// the DMA copy, and signals completion when the emulated channel (bytes / bandwidth after the later of
// "dependencies met" and "channel free") would have delivered the tensor.  Timing is done on the host, so
// no helper kernels run beside the compute kernels (thousands of one-wavefront pacing kernels per
// iteration were measured to slow concurrent GEMMs by a third).
#pragma once
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <memory>
#include <mutex>
#include <thread>
#include <vector>

#include "migration_engine.h"

namespace tio {

class PacedPool : public MigrationEngine {
   public:
    // d2h == h2d: offloads and prefetches share one channel and one FIFO
    PacedPool(hipStream_t d2h, hipStream_t h2d, uint64_t bytes_per_s);
    ~PacedPool() override;
    PacedPool(const PacedPool &) = delete;
    PacedPool &operator=(const PacedPool &) = delete;

    void set_bandwidth(uint64_t bytes_per_s) { bw_.store(bytes_per_s); }   // applies to requests not yet started
    void set_pairs(int n_pairs) override;
    // `where` is the address of the tensor's slot in the pool
    uint64_t submit_offload(int pair, hipEvent_t after, const void *dev, uint64_t where, uint64_t bytes, hipEvent_t done,
                            hipEvent_t t0, hipEvent_t t1) override;
    uint64_t submit_prefetch(int pair, hipEvent_t after, void *dev, uint64_t where, uint64_t bytes, Dep written,
                             std::vector<Dep> landed, std::vector<hipEvent_t> after_more, hipEvent_t done, hipEvent_t t0,
                             hipEvent_t t1) override;
    void wait_offload_recorded(int pair, uint64_t seq) override;
    void wait_prefetch_recorded(int pair, uint64_t seq) override;
    void wait_offload_landed(int pair, uint64_t seq) override;
    void wait_offload_written(int pair, uint64_t seq) override;
    void wait_consumed(int dir, uint64_t seq) override;
    void drain() override;
    void check() override;

   private:
    using Clock = std::chrono::steady_clock;
    struct Request {
        bool prefetch = false;
        int pair = -1;
        uint64_t seq = 0;
        hipEvent_t after = nullptr, done = nullptr, t0 = nullptr, t1 = nullptr;
        uint8_t *dev = nullptr, *slot = nullptr;
        uint64_t bytes = 0;
        Dep written{nullptr, -1, 0};
        std::vector<Dep> landed;
        std::vector<hipEvent_t> after_more;
    };
    struct Channel {                         // one per thread
        std::deque<std::shared_ptr<Request>> queue;
        Clock::time_point free_at{};
        hipEvent_t copied = nullptr;
        std::thread thread;
    };
    void run(int ch);
    void wait_table(const std::vector<uint64_t> &tab, int pair, uint64_t seq);
    void wait_dep(const Dep &d, bool written);
    void guard(const char *what, hipError_t e);

    hipStream_t stream_[2];
    bool shared_ = false;
    std::atomic<uint64_t> bw_;
    std::mutex mu_;
    std::condition_variable cv_;
    bool stop_ = false;
    std::string error_;
    Channel chan_[2];                        // shared: only chan_[0] is used
    uint64_t submitted_[2] = {0, 0}, consumed_[2] = {0, 0}, completed_[2] = {0, 0};   // per direction
    std::vector<uint64_t> off_done_, pre_done_;                                       // per pair: latest sequence number
};

}  // namespace tio
