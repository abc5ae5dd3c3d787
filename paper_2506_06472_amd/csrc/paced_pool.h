// Memory-backed slow tier with an emulated bandwidth (the stand-in for the paper's storage tier, and the
// host-memory tier of Section 3.2): the pool is pinned host memory or a device buffer outside the arena.
// Each direction is a thread with a ready queue (Section 3.2, "Minimize kernel stalls"; Section 3.3): whenever its
// channel is free it looks through the submitted requests in order for those whose dependencies are met (compute
// progress, the tensor's own offload, the offloads that vacate the destination), takes the first urgent one,
// else the first one, and moves one chunk of it: an urgent request overtakes pending ones at a chunk boundary, and
// a request that is still blocked never holds up one that could go.  A chunk counts as delivered when the emulated
// channel (bytes / bandwidth after the later of "chunk started" and "channel free") would have delivered it.
// Timing is done on the host, so no helper kernels run beside the compute kernels (thousands of one-wavefront
// pacing kernels per iteration were measured to slow concurrent GEMMs by a third).
#pragma once
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <memory>
#include <mutex>
#include <set>
#include <thread>
#include <vector>

#include "migration_engine.h"

namespace tio {

class PacedPool : public MigrationEngine {
   public:
    static constexpr uint64_t kDefaultChunk = (uint64_t)16 << 20;
    // d2h == h2d: offloads and prefetches share one channel and one queue.  device_pool: the pool is device memory; its
    // copies are then asked to run on the DMA engines (device-to-device copies default to a copy kernel, which takes
    // compute units and memory bandwidth away from the training kernels in bursts of a whole tensor)
    PacedPool(hipStream_t d2h, hipStream_t h2d, uint64_t bytes_per_s, bool device_pool = false);
    ~PacedPool() override;
    PacedPool(const PacedPool &) = delete;
    PacedPool &operator=(const PacedPool &) = delete;

    void set_bandwidth(uint64_t bytes_per_s) { bw_.store(bytes_per_s); }   // applies to chunks not yet started
    // chunk_bytes 0: whole tensors; urgent_first false: ready requests in the order submitted; ready_queue false: strictly
    // the order submitted (the channel waits for the dependencies of the oldest request).  The engine must be idle.
    void set_policy(uint64_t chunk_bytes, bool urgent_first, bool ready_queue);
    void set_pairs(int n_pairs) override;
    // `where` is the address of the tensor's slot in the pool
    uint64_t submit_offload(int pair, hipEvent_t after, const void *dev, uint64_t where, uint64_t bytes, hipEvent_t done,
                            hipEvent_t t0, hipEvent_t t1, bool urgent) override;
    uint64_t submit_prefetch(int pair, hipEvent_t after, void *dev, uint64_t where, uint64_t bytes, Dep written,
                             std::vector<Dep> landed, std::vector<hipEvent_t> after_more, hipEvent_t done, hipEvent_t t0,
                             hipEvent_t t1, bool urgent) override;
    void wait_offload_recorded(int pair, uint64_t seq) override;
    void wait_prefetch_recorded(int pair, uint64_t seq) override;
    void wait_offload_landed(int pair, uint64_t seq) override;
    void wait_offload_written(int pair, uint64_t seq) override;
    bool offload_landed_now(int pair, uint64_t seq) override;
    bool offload_written_now(int pair, uint64_t seq) override;
    void wait_consumed(int dir, uint64_t seq) override;
    void drain() override;
    void check() override;

    // The choice a free channel makes, as a pure function for tests: `ready` and `urgent` describe the queued requests
    // in the order submitted; returns the index of the one to serve next, or -1 if none may go.
    static int choose(const std::vector<uint8_t> &ready, const std::vector<uint8_t> &urgent, bool urgent_first,
                      bool ready_queue);

   private:
    using Clock = std::chrono::steady_clock;
    struct Request {
        bool prefetch = false, urgent = false;
        int pair = -1;
        uint64_t seq = 0;
        hipEvent_t after = nullptr, done = nullptr, t0 = nullptr, t1 = nullptr;
        uint8_t *dev = nullptr, *slot = nullptr;
        uint64_t bytes = 0, moved = 0;          // moved: bytes of the chunks already delivered
        Dep written{nullptr, -1, 0};
        std::vector<Dep> landed;
        std::vector<hipEvent_t> after_more;
        // progress of the readiness check (only the channel's thread touches these)
        bool after_seen = false;
        size_t more_seen = 0, landed_seen = 0;
        bool written_seen = false;
    };
    struct Channel {                         // one per thread
        std::deque<std::shared_ptr<Request>> queue;
        Clock::time_point free_at{};
        hipEvent_t copied = nullptr;
        std::thread thread;
    };
    void run(int ch);
    bool ready(Request &r);                  // non-blocking; called without the lock by the channel's thread
    void wait_table(const std::vector<uint64_t> &tab, int pair, uint64_t seq);
    void guard(const char *what, hipError_t e);

    hipStream_t stream_[2];
    bool shared_ = false;
    hipMemcpyKind kind_ = hipMemcpyDefault;
    std::atomic<uint64_t> bw_;
    uint64_t chunk_ = kDefaultChunk;
    bool urgent_first_ = true, ready_queue_ = true;
    std::mutex mu_;
    std::condition_variable cv_;
    bool stop_ = false;
    std::string error_;
    Channel chan_[2];                        // shared: only chan_[0] is used
    uint64_t submitted_[2] = {0, 0}, completed_[2] = {0, 0};                          // per direction
    std::set<uint64_t> unconsumed_[2];       // per direction: requests whose `after` event the engine has not yet seen complete
    std::vector<uint64_t> off_done_, pre_done_;                                       // per pair: latest sequence number
};

}  // namespace tio
