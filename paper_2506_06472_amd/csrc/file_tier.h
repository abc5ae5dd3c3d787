// File-backed slow tier of the migration engine (Section 3.3 of the paper: tensors move between GPU
// memory and storage).  The platform has no direct storage-to-GPU path, so every transfer goes through
// a ring of pinned staging chunks: offloads are DMA copies into a chunk followed by a positional write of
// that chunk, prefetches are positional reads into a chunk followed by a DMA copy.  The file is opened
// for direct I/O (no page cache) where the file system allows it; direct I/O then runs on ordinary
// page-aligned buffers, because the kernel cannot pin HIP's pinned host memory a second time.  Each direction is a FIFO, like the
// copy streams of the memory-backed tiers, so the planner's channel model carries over.
//
// Threads: per direction one thread that walks the request queue and a few I/O workers; the prefetch
// direction has a second thread that issues the DMA copies as the reads land.  Every cross-thread
// dependency is a host-side sequence number under one mutex; HIP events are only waited on by the thread
// or stream that the recording thread handed them to.
#pragma once
#include <hip/hip_runtime_api.h>

#include "migration_engine.h"

#include <condition_variable>
#include <cstdint>
#include <deque>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

namespace tio {

using FileTierError = EngineError;

class FileTier : public MigrationEngine {
   public:
    static constexpr uint64_t kAlign = 4096;     // direct I/O: file offsets, lengths and buffers

    // staging: pinned host memory, 4096-byte aligned, split evenly between the two directions
    FileTier(const char *path, void *staging, uint64_t staging_bytes, uint64_t chunk_bytes, hipStream_t d2h,
             hipStream_t h2d, bool buffered);
    ~FileTier() override;
    FileTier(const FileTier &) = delete;
    FileTier &operator=(const FileTier &) = delete;

    bool direct() const { return direct_; }
    uint64_t file_bytes() const { return file_bytes_; }
    void resize(uint64_t bytes);                  // grows the file to at least `bytes`
    void set_pairs(int n_pairs) override;

    // ---- synchronous set-up path (the engine must be idle: call drain() first) ----
    void write_host(uint64_t file_off, const void *src, uint64_t bytes);
    void read_host(uint64_t file_off, void *dst, uint64_t bytes);
    void zero(uint64_t file_off, uint64_t bytes);
    void from_device(uint64_t file_off, const void *dev, uint64_t bytes);
    void to_device(uint64_t file_off, void *dev, uint64_t bytes);

    // ---- asynchronous migration path (MigrationEngine); `where` is a 4096-byte aligned file offset ----
    // (requests are served in the order submitted: `urgent` is accepted and not used by this tier)
    uint64_t submit_offload(int pair, hipEvent_t after, const void *dev, uint64_t where, uint64_t bytes, hipEvent_t done,
                            hipEvent_t t0, hipEvent_t t1, bool urgent) override;
    uint64_t submit_prefetch(int pair, hipEvent_t after, void *dev, uint64_t where, uint64_t bytes, Dep written,
                             std::vector<Dep> landed, std::vector<hipEvent_t> after_more, hipEvent_t done, hipEvent_t t0,
                             hipEvent_t t1, bool urgent) override;
    bool offload_landed_now(int pair, uint64_t seq) override;
    bool offload_written_now(int pair, uint64_t seq) override;
    void wait_offload_recorded(int pair, uint64_t seq) override;
    void wait_prefetch_recorded(int pair, uint64_t seq) override;
    void wait_offload_landed(int pair, uint64_t seq) override;
    void wait_offload_written(int pair, uint64_t seq) override;
    void wait_consumed(int dir, uint64_t seq) override;
    void drain() override;                        // every submitted request has completed, file I/O included
    void check() override;
    uint64_t bytes_written() const { return bytes_written_; }
    uint64_t bytes_read() const { return bytes_read_; }

   private:
    struct Slot {
        uint8_t *buf = nullptr;
        hipEvent_t ev = nullptr;
        bool busy = false;          // offload: until the chunk is in the file; prefetch: until its DMA copy was issued and has finished
        bool read_done = false;     // prefetch: the read into buf has completed
        bool dma_issued = false;    // prefetch: ev has been recorded behind the chunk's DMA copy
    };
    struct Request {
        int pair = -1;
        uint64_t seq = 0;
        hipEvent_t after = nullptr, done = nullptr, t0 = nullptr, t1 = nullptr;
        uint8_t *dev = nullptr;
        uint64_t file_off = 0, bytes = 0;
        Dep written{nullptr, -1, 0};
        std::vector<Dep> landed;
        std::vector<hipEvent_t> after_more;
        uint64_t chunks_left = 0;   // offload: chunks not yet in the file
    };
    struct Job {                    // one chunk
        std::shared_ptr<Request> req;
        int slot = 0;
        uint64_t off = 0, n = 0;    // offset inside the request, payload bytes
        bool first = false, last = false;
    };
    struct Dir {
        hipStream_t stream = nullptr;
        std::vector<Slot> ring;
        uint64_t next_slot = 0;
        std::deque<std::shared_ptr<Request>> queue;     // submitted, not yet taken by the direction's thread
        std::deque<Job> io;                              // chunks for the I/O workers
        std::deque<Job> dma;                             // prefetch: chunks whose read was submitted, in order
        uint64_t submitted = 0, consumed = 0, completed = 0;
        std::vector<std::thread> threads;
    };

    void offload_thread(int);
    void offload_worker(int w);
    void prefetch_reader(int);
    void prefetch_issuer(int);
    void prefetch_worker(int w);
    void chunk_io(bool write, uint8_t *staging, uint64_t n, uint64_t file_off, uint8_t *bounce);
    int acquire(Dir &d, std::unique_lock<std::mutex> &lk, bool prefetch);
    void fail_locked(const std::string &msg);
    void wait_dep(const Dep &d, bool written, std::unique_lock<std::mutex> &lk);
    void io_all(bool write, uint8_t *buf, uint64_t n, uint64_t file_off);
    void guard(const char *what, hipError_t e);

    int fd_ = -1;
    bool direct_ = false;
    uint64_t chunk_ = 0, file_bytes_ = 0;
    uint8_t *sync_buf_ = nullptr;                        // first offload chunk, used by the set-up path
    std::vector<uint8_t *> bounce_;                      // direct I/O: page-aligned ordinary buffers (workers, then set-up path)
    std::mutex mu_;
    std::condition_variable cv_;
    bool stop_ = false;
    std::string error_;
    Dir dir_[2];                                         // 0 offload, 1 prefetch
    std::vector<uint64_t> off_recorded_, off_landed_, off_written_, pre_recorded_;   // per pair: latest sequence number
    uint64_t bytes_written_ = 0, bytes_read_ = 0;
};

}  // namespace tio
