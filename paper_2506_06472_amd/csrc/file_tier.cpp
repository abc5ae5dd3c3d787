// File-backed slow tier: staging ring, I/O threads and the two FIFO directions (see file_tier.h).
#include "file_tier.h"

#include <fcntl.h>
#include <sys/stat.h>
#include <sys/types.h>
#include <unistd.h>

#include <algorithm>
#include <cerrno>
#include <cstdlib>
#include <cstring>

namespace tio {

namespace {
constexpr int kWorkers = 4;                      // I/O workers per direction
constexpr uint64_t kMaxSlots = 64;
inline uint64_t align_up(uint64_t x) { return (x + FileTier::kAlign - 1) / FileTier::kAlign * FileTier::kAlign; }
}  // namespace

void FileTier::guard(const char *what, hipError_t e) {
    if (e != hipSuccess) throw FileTierError{std::string(what) + ": " + hipGetErrorString(e)};
}

FileTier::FileTier(const char *path, void *staging, uint64_t staging_bytes, uint64_t chunk_bytes, hipStream_t d2h,
                   hipStream_t h2d, bool buffered) {
    if (!path || !*path) throw FileTierError{"empty file name"};
    chunk_ = chunk_bytes ? chunk_bytes : ((uint64_t)8 << 20);
    if (chunk_ % kAlign || chunk_ < kAlign) throw FileTierError{"chunk size must be a multiple of 4096 bytes"};
    if (!staging || ((uintptr_t)staging % kAlign)) throw FileTierError{"staging buffer must be 4096-byte aligned pinned host memory"};
    const uint64_t per_dir = std::min(kMaxSlots, staging_bytes / 2 / chunk_);
    if (per_dir < 2) throw FileTierError{"staging buffer must hold at least two chunks per direction (" + std::to_string(4 * chunk_) + " bytes)"};
    if (!buffered) fd_ = ::open(path, O_RDWR | O_CREAT | O_DIRECT | O_CLOEXEC, 0600);
    direct_ = fd_ >= 0;
    if (buffered || (fd_ < 0 && errno == EINVAL)) fd_ = ::open(path, O_RDWR | O_CREAT | O_CLOEXEC, 0600);   // or: file system without direct I/O
    if (fd_ < 0) throw FileTierError{std::string("cannot open ") + path + ": " + std::strerror(errno)};
    struct stat sb;
    if (::fstat(fd_, &sb) == 0) file_bytes_ = (uint64_t)sb.st_size;
    dir_[0].stream = d2h;
    dir_[1].stream = h2d;
    try {
        for (int d = 0; d < 2; ++d) {
            dir_[d].ring.resize(per_dir);
            for (uint64_t i = 0; i < per_dir; ++i) {
                dir_[d].ring[i].buf = (uint8_t *)staging + ((uint64_t)d * per_dir + i) * chunk_;
                guard("hipEventCreate", hipEventCreateWithFlags(&dir_[d].ring[i].ev, hipEventDisableTiming));
            }
        }
    } catch (...) {
        for (auto &d : dir_) for (auto &s : d.ring) if (s.ev) (void)hipEventDestroy(s.ev);
        ::close(fd_);
        throw;
    }
    sync_buf_ = dir_[0].ring[0].buf;
    if (direct_) {
        // direct I/O cannot pin the pages of HIP's pinned host memory (the kernel answers EFAULT), so the
        // file is read and written through ordinary page-aligned buffers, one per I/O worker and one for
        // the set-up path, with a host copy between them and the staging chunks
        bounce_.assign(2 * kWorkers + 1, nullptr);
        for (auto &b : bounce_) {
            void *q = nullptr;
            if (::posix_memalign(&q, kAlign, chunk_) != 0) {
                for (auto *x : bounce_) std::free(x);
                for (auto &d : dir_) for (auto &sl : d.ring) if (sl.ev) (void)hipEventDestroy(sl.ev);
                ::close(fd_);
                throw FileTierError{"out of host memory for the direct-I/O buffers"};
            }
            b = (uint8_t *)q;
        }
    }
    set_pairs(0);
    int dev = 0;
    (void)hipGetDevice(&dev);
    auto run = [this, dev](void (FileTier::*body)(int), int w) {
        return std::thread([this, dev, body, w] {
            try {
                guard("hipSetDevice", hipSetDevice(dev));
                (this->*body)(w);
            } catch (const FileTierError &e) {
                std::lock_guard<std::mutex> lk(mu_);
                fail_locked(e.msg);
            } catch (const std::exception &e) {
                std::lock_guard<std::mutex> lk(mu_);
                fail_locked(e.what());
            }
        });
    };
    dir_[0].threads.push_back(run(&FileTier::offload_thread, 0));
    for (int i = 0; i < kWorkers; ++i) dir_[0].threads.push_back(run(&FileTier::offload_worker, i));
    dir_[1].threads.push_back(run(&FileTier::prefetch_reader, 0));
    dir_[1].threads.push_back(run(&FileTier::prefetch_issuer, 0));
    for (int i = 0; i < kWorkers; ++i) dir_[1].threads.push_back(run(&FileTier::prefetch_worker, kWorkers + i));
}

FileTier::~FileTier() {
    {
        std::lock_guard<std::mutex> lk(mu_);
        stop_ = true;
    }
    cv_.notify_all();
    for (auto &d : dir_) for (auto &t : d.threads) if (t.joinable()) t.join();
    for (auto &d : dir_) for (auto &s : d.ring) if (s.ev) (void)hipEventDestroy(s.ev);
    for (auto *b : bounce_) std::free(b);
    if (fd_ >= 0) ::close(fd_);
}

// one chunk between a staging buffer and the file; `bounce` is the calling thread's direct-I/O buffer
void FileTier::chunk_io(bool write, uint8_t *staging, uint64_t n, uint64_t file_off, uint8_t *bounce) {
    const uint64_t na = align_up(n);
    if (!bounce) { io_all(write, staging, na, file_off); return; }
    if (write) {
        std::memcpy(bounce, staging, n);
        if (na > n) std::memset(bounce + n, 0, na - n);
        io_all(true, bounce, na, file_off);
    } else {
        io_all(false, bounce, na, file_off);
        std::memcpy(staging, bounce, n);
    }
}

void FileTier::fail_locked(const std::string &msg) {
    if (error_.empty()) error_ = msg;
    cv_.notify_all();
}

void FileTier::check() {
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw FileTierError{error_};
}

void FileTier::resize(uint64_t bytes) {
    bytes = align_up(bytes);
    if (bytes <= file_bytes_) return;
    if (::ftruncate(fd_, (off_t)bytes) != 0) throw FileTierError{std::string("cannot grow the slow-tier file: ") + std::strerror(errno)};
    // reserve the blocks now: a full disk is reported here and not in the middle of a step
    const int e = ::posix_fallocate(fd_, 0, (off_t)bytes);
    if (e != 0 && e != EOPNOTSUPP && e != EINVAL) throw FileTierError{std::string("cannot reserve the slow-tier file: ") + std::strerror(e)};
    file_bytes_ = bytes;
}

void FileTier::set_pairs(int n) {
    std::lock_guard<std::mutex> lk(mu_);
    const size_t m = (size_t)std::max(n, 0);
    off_recorded_.assign(m, 0); off_landed_.assign(m, 0); off_written_.assign(m, 0); pre_recorded_.assign(m, 0);
}

void FileTier::io_all(bool write, uint8_t *buf, uint64_t n, uint64_t file_off) {
    if (file_off % kAlign || n % kAlign) throw FileTierError{"unaligned file access"};
    if (file_off + n > file_bytes_) throw FileTierError{"access beyond the end of the slow-tier file"};
    uint64_t done = 0;
    while (done < n) {
        const ssize_t r = write ? ::pwrite(fd_, buf + done, n - done, (off_t)(file_off + done))
                                : ::pread(fd_, buf + done, n - done, (off_t)(file_off + done));
        if (r < 0 && errno == EINTR) continue;
        if (r <= 0) throw FileTierError{std::string(write ? "write to" : "read from") + " the slow-tier file failed: " +
                                        (r == 0 ? "unexpected end of file" : std::strerror(errno))};
        done += (uint64_t)r;
    }
}

// ---------------------------------------------------------------- synchronous set-up path
void FileTier::write_host(uint64_t off, const void *src, uint64_t bytes) {
    for (uint64_t o = 0; o < bytes; o += chunk_) {
        const uint64_t n = std::min(chunk_, bytes - o), na = align_up(n);
        uint8_t *b = direct_ ? bounce_.back() : sync_buf_;
        std::memcpy(b, (const uint8_t *)src + o, n);
        if (na > n) std::memset(b + n, 0, na - n);
        io_all(true, b, na, off + o);
    }
}
void FileTier::read_host(uint64_t off, void *dst, uint64_t bytes) {
    for (uint64_t o = 0; o < bytes; o += chunk_) {
        const uint64_t n = std::min(chunk_, bytes - o);
        uint8_t *b = direct_ ? bounce_.back() : sync_buf_;
        io_all(false, b, align_up(n), off + o);
        std::memcpy((uint8_t *)dst + o, b, n);
    }
}
void FileTier::zero(uint64_t off, uint64_t bytes) {
    uint8_t *b = direct_ ? bounce_.back() : sync_buf_;
    std::memset(b, 0, std::min(chunk_, align_up(bytes)));
    for (uint64_t o = 0; o < bytes; o += chunk_) io_all(true, b, align_up(std::min(chunk_, bytes - o)), off + o);
}
void FileTier::from_device(uint64_t off, const void *dev, uint64_t bytes) {
    for (uint64_t o = 0; o < bytes; o += chunk_) {
        const uint64_t n = std::min(chunk_, bytes - o);
        guard("hipMemcpy", hipMemcpy(sync_buf_, (const uint8_t *)dev + o, n, hipMemcpyDeviceToHost));
        chunk_io(true, sync_buf_, n, off + o, direct_ ? bounce_.back() : nullptr);
    }
}
void FileTier::to_device(uint64_t off, void *dev, uint64_t bytes) {
    for (uint64_t o = 0; o < bytes; o += chunk_) {
        const uint64_t n = std::min(chunk_, bytes - o);
        chunk_io(false, sync_buf_, n, off + o, direct_ ? bounce_.back() : nullptr);
        guard("hipMemcpy", hipMemcpy((uint8_t *)dev + o, sync_buf_, n, hipMemcpyHostToDevice));
    }
}

// ---------------------------------------------------------------- asynchronous path: caller side
uint64_t FileTier::submit_offload(int pair, hipEvent_t after, const void *dev, uint64_t file_off, uint64_t bytes,
                                  hipEvent_t done, hipEvent_t t0, hipEvent_t t1, bool) {
    if (bytes == 0 || file_off % kAlign || file_off + align_up(bytes) > file_bytes_) throw FileTierError{"bad offload request"};
    auto r = std::make_shared<Request>();
    r->pair = pair; r->after = after; r->done = done; r->t0 = t0; r->t1 = t1;
    r->dev = (uint8_t *)dev; r->file_off = file_off; r->bytes = bytes;
    r->chunks_left = (bytes + chunk_ - 1) / chunk_;
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw FileTierError{error_};
    if (pair < 0 || (size_t)pair >= off_recorded_.size()) throw FileTierError{"pair index outside the installed plan"};
    r->seq = ++dir_[0].submitted;
    dir_[0].queue.push_back(r);
    cv_.notify_all();
    return r->seq;
}

uint64_t FileTier::submit_prefetch(int pair, hipEvent_t after, void *dev, uint64_t file_off, uint64_t bytes, Dep written,
                                   std::vector<Dep> landed, std::vector<hipEvent_t> after_more, hipEvent_t done,
                                   hipEvent_t t0, hipEvent_t t1, bool) {
    if (bytes == 0 || file_off % kAlign || file_off + align_up(bytes) > file_bytes_) throw FileTierError{"bad prefetch request"};
    auto r = std::make_shared<Request>();
    r->pair = pair; r->after = after; r->done = done; r->t0 = t0; r->t1 = t1;
    r->dev = (uint8_t *)dev; r->file_off = file_off; r->bytes = bytes;
    r->written = written; r->landed = std::move(landed); r->after_more = std::move(after_more);
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw FileTierError{error_};
    if (pair < 0 || (size_t)pair >= pre_recorded_.size()) throw FileTierError{"pair index outside the installed plan"};
    r->seq = ++dir_[1].submitted;
    dir_[1].queue.push_back(r);
    cv_.notify_all();
    return r->seq;
}

void FileTier::wait_offload_recorded(int pair, uint64_t seq) {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return !error_.empty() || off_recorded_[pair] >= seq; });
    if (!error_.empty()) throw FileTierError{error_};
}
void FileTier::wait_prefetch_recorded(int pair, uint64_t seq) {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return !error_.empty() || pre_recorded_[pair] >= seq; });
    if (!error_.empty()) throw FileTierError{error_};
}
void FileTier::wait_offload_landed(int pair, uint64_t seq) {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return !error_.empty() || off_landed_[pair] >= seq; });
    if (!error_.empty()) throw FileTierError{error_};
}
void FileTier::wait_offload_written(int pair, uint64_t seq) {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return !error_.empty() || off_written_[pair] >= seq; });
    if (!error_.empty()) throw FileTierError{error_};
}
bool FileTier::offload_landed_now(int pair, uint64_t seq) {
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw FileTierError{error_};
    return off_landed_[pair] >= seq;
}
bool FileTier::offload_written_now(int pair, uint64_t seq) {
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_.empty()) throw FileTierError{error_};
    return off_written_[pair] >= seq;
}
// a dependency of a prefetch, on this engine (waited for under the lock) or on another one
void FileTier::wait_dep(const Dep &d, bool written, std::unique_lock<std::mutex> &lk) {
    if (!d.seq) return;
    if (d.eng == this || d.eng == nullptr) {
        const std::vector<uint64_t> &tab = written ? off_written_ : off_landed_;
        cv_.wait(lk, [&] { return stop_ || !error_.empty() || tab[d.pair] >= d.seq; });
        return;
    }
    lk.unlock();
    try {
        if (written) d.eng->wait_offload_written(d.pair, d.seq); else d.eng->wait_offload_landed(d.pair, d.seq);
    } catch (...) { lk.lock(); throw; }
    lk.lock();
}
void FileTier::wait_consumed(int dir, uint64_t seq) {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return !error_.empty() || dir_[dir].consumed >= seq; });
    if (!error_.empty()) throw FileTierError{error_};
}
void FileTier::drain() {
    {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [&] {
            return !error_.empty() || (dir_[0].completed == dir_[0].submitted && dir_[1].completed == dir_[1].submitted);
        });
        if (!error_.empty()) throw FileTierError{error_};
    }
    guard("hipStreamSynchronize", hipStreamSynchronize(dir_[0].stream));
    guard("hipStreamSynchronize", hipStreamSynchronize(dir_[1].stream));
}

// ---------------------------------------------------------------- engine threads
// next staging chunk of the ring, in order; returns -1 when the engine stops
int FileTier::acquire(Dir &d, std::unique_lock<std::mutex> &lk, bool prefetch) {
    const int s = (int)(d.next_slot % d.ring.size());
    Slot &sl = d.ring[s];
    cv_.wait(lk, [&] { return stop_ || !error_.empty() || !sl.busy || (prefetch && sl.dma_issued); });
    if (stop_ || !error_.empty()) return -1;
    if (sl.busy) {                               // prefetch: the chunk's DMA copy was issued; wait for it outside the lock
        lk.unlock();
        guard("hipEventSynchronize", hipEventSynchronize(sl.ev));
        lk.lock();
        if (stop_ || !error_.empty()) return -1;
    }
    sl.busy = true; sl.read_done = false; sl.dma_issued = false;
    ++d.next_slot;
    return s;
}

void FileTier::offload_thread(int) {
    Dir &d = dir_[0];
    for (;;) {
        std::shared_ptr<Request> r;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_.wait(lk, [&] { return stop_ || !error_.empty() || !d.queue.empty(); });
            if (stop_ || !error_.empty()) return;
            r = d.queue.front();
            d.queue.pop_front();
        }
        guard("hipStreamWaitEvent", hipStreamWaitEvent(d.stream, r->after, 0));
        {
            std::lock_guard<std::mutex> lk(mu_);
            d.consumed = r->seq;
            cv_.notify_all();
        }
        if (r->t0) guard("hipEventRecord", hipEventRecord(r->t0, d.stream));
        for (uint64_t off = 0; off < r->bytes; off += chunk_) {
            const uint64_t n = std::min(chunk_, r->bytes - off);
            const bool last = off + n == r->bytes;
            int s;
            {
                std::unique_lock<std::mutex> lk(mu_);
                s = acquire(d, lk, false);
                if (s < 0) return;
            }
            guard("hipMemcpyAsync", hipMemcpyAsync(d.ring[s].buf, r->dev + off, n, hipMemcpyDeviceToHost, d.stream));
            guard("hipEventRecord", hipEventRecord(d.ring[s].ev, d.stream));
            if (last) {
                if (poison_) poison_(d.stream, r->dev, r->bytes);
                if (r->t1) guard("hipEventRecord", hipEventRecord(r->t1, d.stream));
                guard("hipEventRecord", hipEventRecord(r->done, d.stream));
            }
            std::lock_guard<std::mutex> lk(mu_);
            d.io.push_back(Job{r, s, off, n, off == 0, last});
            if (last) off_recorded_[r->pair] = r->seq;
            cv_.notify_all();
        }
    }
}

void FileTier::offload_worker(int w) {
    Dir &d = dir_[0];
    for (;;) {
        Job j;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_.wait(lk, [&] { return stop_ || !error_.empty() || !d.io.empty(); });
            if (stop_ || !error_.empty()) return;
            j = d.io.front();
            d.io.pop_front();
        }
        guard("hipEventSynchronize", hipEventSynchronize(d.ring[j.slot].ev));
        if (j.last) {                            // stream order: every chunk of the request has left the arena
            std::lock_guard<std::mutex> lk(mu_);
            off_landed_[j.req->pair] = j.req->seq;
            cv_.notify_all();
        }
        chunk_io(true, d.ring[j.slot].buf, j.n, j.req->file_off + j.off, direct_ ? bounce_[w] : nullptr);
        std::lock_guard<std::mutex> lk(mu_);
        d.ring[j.slot].busy = false;
        bytes_written_ += j.n;
        if (--j.req->chunks_left == 0) {
            off_written_[j.req->pair] = j.req->seq;
            ++d.completed;
        }
        cv_.notify_all();
    }
}

void FileTier::prefetch_reader(int) {
    Dir &d = dir_[1];
    for (;;) {
        std::shared_ptr<Request> r;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_.wait(lk, [&] { return stop_ || !error_.empty() || !d.queue.empty(); });
            if (stop_ || !error_.empty()) return;
            r = d.queue.front();
            d.queue.pop_front();
            wait_dep(r->written, true, lk);      // the tensor's own offload must be in the file before it is read back
            if (stop_ || !error_.empty()) return;
        }
        for (uint64_t off = 0; off < r->bytes; off += chunk_) {
            const uint64_t n = std::min(chunk_, r->bytes - off);
            std::unique_lock<std::mutex> lk(mu_);
            const int s = acquire(d, lk, true);
            if (s < 0) return;
            const Job j{r, s, off, n, off == 0, off + n == r->bytes};
            d.io.push_back(j);
            d.dma.push_back(j);
            cv_.notify_all();
        }
    }
}

void FileTier::prefetch_worker(int w) {
    Dir &d = dir_[1];
    for (;;) {
        Job j;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_.wait(lk, [&] { return stop_ || !error_.empty() || !d.io.empty(); });
            if (stop_ || !error_.empty()) return;
            j = d.io.front();
            d.io.pop_front();
        }
        chunk_io(false, d.ring[j.slot].buf, j.n, j.req->file_off + j.off, direct_ ? bounce_[w] : nullptr);
        std::lock_guard<std::mutex> lk(mu_);
        d.ring[j.slot].read_done = true;
        bytes_read_ += j.n;
        cv_.notify_all();
    }
}

void FileTier::prefetch_issuer(int) {
    Dir &d = dir_[1];
    for (;;) {
        Job j;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_.wait(lk, [&] { return stop_ || !error_.empty() || !d.dma.empty(); });
            if (stop_ || !error_.empty()) return;
            j = d.dma.front();
            d.dma.pop_front();
            if (j.first) {                       // the destination ranges must have been vacated
                for (const Dep &w : j.req->landed) {
                    wait_dep(w, false, lk);
                    if (stop_ || !error_.empty()) return;
                }
            }
            cv_.wait(lk, [&] { return stop_ || !error_.empty() || d.ring[j.slot].read_done; });
            if (stop_ || !error_.empty()) return;
        }
        Request &r = *j.req;
        if (j.first) {
            guard("hipStreamWaitEvent", hipStreamWaitEvent(d.stream, r.after, 0));
            for (hipEvent_t e : r.after_more) guard("hipStreamWaitEvent", hipStreamWaitEvent(d.stream, e, 0));
            {
                std::lock_guard<std::mutex> lk(mu_);
                d.consumed = r.seq;
                cv_.notify_all();
            }
            if (r.t0) guard("hipEventRecord", hipEventRecord(r.t0, d.stream));
        }
        guard("hipMemcpyAsync", hipMemcpyAsync(r.dev + j.off, d.ring[j.slot].buf, j.n, hipMemcpyHostToDevice, d.stream));
        guard("hipEventRecord", hipEventRecord(d.ring[j.slot].ev, d.stream));
        if (j.last) {
            if (r.t1) guard("hipEventRecord", hipEventRecord(r.t1, d.stream));
            guard("hipEventRecord", hipEventRecord(r.done, d.stream));
        }
        std::lock_guard<std::mutex> lk(mu_);
        d.ring[j.slot].dma_issued = true;
        if (j.last) {
            pre_recorded_[r.pair] = r.seq;
            ++d.completed;
        }
        cv_.notify_all();
    }
}

}  // namespace tio
