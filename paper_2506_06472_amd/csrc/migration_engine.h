// Interface of a slow-tier engine that runs the two migration directions on threads of its own
// (Section 3.3 of the paper).  The host thread that walks the kernel schedule submits requests in plan
// order and blocks, before a kernel, until the completion events that kernel depends on have been
// recorded by the engine; only then can it make the compute stream wait for them.  Every cross-thread
// dependency is a per-pair sequence number; a request may also depend on an offload of another engine.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <string>
#include <vector>

namespace tio {

struct EngineError { std::string msg; };

class MigrationEngine {
   public:
    struct Dep { MigrationEngine *eng; int pair; uint64_t seq; };    // seq 0 = none

    virtual ~MigrationEngine() {}
    virtual void set_pairs(int n_pairs) = 0;      // sequence tables for a newly installed plan (engine idle)
    // debugging aid: called on the offload stream after a tensor's last copy out of the arena has been
    // enqueued and before `done` is recorded, to overwrite the vacated range (nullptr = off)
    using PoisonFn = void (*)(hipStream_t stream, void *dev, uint64_t bytes);
    void set_poison(PoisonFn fn) { poison_ = fn; }
    // urgent: the plan marks the migration as one a stalled kernel waits for (Section 3.2, "Minimize kernel stalls");
    // an engine with a ready queue serves such requests before the other pending ones.
    // `where`: the tensor's place on the slow tier (a file offset, or a host or device address);
    // `after`: event recorded by the caller on the compute stream (the copy may not start before it);
    // `done`: recorded on the direction's stream when the transfer counts as complete; t0/t1: optional
    // timing events recorded at the transfer's begin and end.  Returns the request's sequence number.
    virtual uint64_t submit_offload(int pair, hipEvent_t after, const void *dev, uint64_t where, uint64_t bytes,
                                    hipEvent_t done, hipEvent_t t0, hipEvent_t t1, bool urgent) = 0;
    // written: the offload that must be complete on the slow tier before the tensor is read back;
    // landed: offloads that must have left the arena (their ranges are the destination);
    // after_more: further events, already recorded by the caller, that the copy must wait for
    virtual uint64_t submit_prefetch(int pair, hipEvent_t after, void *dev, uint64_t where, uint64_t bytes, Dep written,
                                     std::vector<Dep> landed, std::vector<hipEvent_t> after_more, hipEvent_t done,
                                     hipEvent_t t0, hipEvent_t t1, bool urgent) = 0;
    // block until `done` of that request has been recorded (a stream can then wait for it)
    virtual void wait_offload_recorded(int pair, uint64_t seq) = 0;
    virtual void wait_prefetch_recorded(int pair, uint64_t seq) = 0;
    // block until that offload has left the arena / is complete on the slow tier
    virtual void wait_offload_landed(int pair, uint64_t seq) = 0;
    virtual void wait_offload_written(int pair, uint64_t seq) = 0;
    // the same two questions without blocking (asked by another engine's thread when it looks for a ready request)
    virtual bool offload_landed_now(int pair, uint64_t seq) = 0;
    virtual bool offload_written_now(int pair, uint64_t seq) = 0;
    // block until the engine has taken over the `after` event of that request (the caller may re-record it);
    // dir 0 offload, 1 prefetch
    virtual void wait_consumed(int dir, uint64_t seq) = 0;
    virtual void drain() = 0;                     // every submitted request has completed
    virtual void check() = 0;                     // throws EngineError if any thread met an error

   protected:
    PoisonFn poison_ = nullptr;
};

}  // namespace tio
