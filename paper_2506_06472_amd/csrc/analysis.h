// Pure-CPU half of the library: trace container, lifetime analysis (Section 3.1), migration
// planner (Section 3.2, Algorithm 1 plus the urgent pass) and the arena address assignment.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/teraio.h"
#include "program.h"

namespace tio {

struct Trace {
    int32_t n_kernels = 0, n_tensors = 0, n_persistent = 0;
    std::vector<int32_t> op, operand_off, operand_tensor, operand_flags;
    std::vector<int64_t> flops, tau;
    std::vector<uint64_t> tensor_bytes;
    std::vector<int32_t> tensor_kind;
    uint64_t structure_hash = 0;       // of everything except tau
    void rehash();
};

struct Period { int32_t tensor; uint64_t bytes; int32_t start, end; };

struct Lifetimes {
    int32_t n_kernels = 0;
    std::vector<uint64_t> M;
    std::vector<Period> periods;                 // sorted by (tensor, start)
    std::vector<std::vector<int32_t>> active;    // per tensor, ascending kernel indices
    uint64_t structure_hash = 0;
    // flat copies for the view
    std::vector<int32_t> v_tensor, v_start, v_end;
    std::vector<uint64_t> v_bytes;
};

// One selected inactive period: the tensor is out of GPU memory at kernels [k_off, k_pre].
struct Pair {
    int32_t tensor; uint64_t bytes;
    int32_t start, end, k_off, k_pre;
    int32_t urgent_off, urgent_pre;
    int32_t tier = 0;                  // 0: slow tier, 1: host-memory tier
    uint64_t host_offset = 0;          // slot in the pool of its tier
    int32_t alloc_before = -1;         // allocation that ends with this pair's offload
    int32_t alloc_after = -1;          // allocation that begins with this pair's prefetch
};

struct Alloc {
    int32_t tensor;
    int32_t first, last;               // unrolled kernel interval of residency (last may be >= N)
    uint64_t address = 0;
    int32_t born_by_pair = -1;         // prefetch pair that fills it, -1: first write by a kernel / always resident
    int32_t ended_by_pair = -1;        // offload pair that empties it, -1: freed after last use / never
    bool whole_cycle = false;          // persistent tensor that never leaves
    std::vector<int32_t> wait_pairs;   // offload events the first writer must wait for (address reuse)
};

struct Plan {
    int32_t n_kernels = 0;
    uint64_t cap = 0, planning_cap = 0, arena_needed = 0, host_needed = 0, bytes_moved = 0, bw = 0;
    int32_t n_greedy = 0, n_forced = 0;
    uint64_t host_peak = 0, host_bw = 0, host_tier_needed = 0;   // host-memory tier: peak bytes held, bandwidth, pool bytes
    std::vector<int32_t> pair_tier;              // exported view of Pair::tier
    uint64_t structure_hash = 0;
    uint64_t serial = 0;               // unique per built plan; the runtime uses it to notice a plan change
    std::vector<uint64_t> Mp;
    std::vector<Pair> pairs;                     // selection order (= pair id)
    std::vector<tio_plan_entry> entries;         // issue order
    std::vector<Alloc> allocs;
    std::vector<tio_alloc> v_allocs;
    std::vector<uint64_t> persistent_home;       // host offset of each persistent tensor's home slot
    // executor tables, indexed by kernel
    std::vector<std::vector<int32_t>> entries_at;        // entry indices with trigger % N == k
    int32_t retime_pass = 0;                             // which re-timing pass produced the selection (0: the first, on the kernel times)
    int64_t predicted_step_ns = 0;                       // with re-timing: the iteration the performance model predicts for this selection
    std::vector<std::vector<int32_t>> kernel_wait_pre;   // pair ids whose prefetch event kernel k waits for
    std::vector<std::vector<int32_t>> kernel_wait_off;   // pair ids whose offload event kernel k waits for
    std::vector<uint8_t> kernel_needs_event;             // record an event after kernel k
    std::vector<std::vector<int32_t>> alloc_of;          // per tensor: indices into allocs
};

Trace trace_from_program(const Program &P);
void model_tau(Trace &t);                        // deterministic stand-in for measured kernel times
Lifetimes analyze(const Trace &t);

struct PlanError { int code; std::string msg; };
// Throws PlanError.
Plan build_plan(const Trace &t, const Lifetimes &life, uint64_t cap, uint64_t bw, const tio_plan_opts &opts);
// Algorithm 1 + urgent pass only (no layout); fills pairs, Mp, n_greedy, n_forced.
void select_periods(const Trace &t, const Lifetimes &life, uint64_t cap, uint64_t bw, bool duplex,
                    uint64_t min_bytes, uint64_t host_bw, uint64_t host_budget, bool clamp_benefit, Plan &out);
// select_periods, then two chains of `passes` more runs of it on the timeline stretched by the stalls the performance
// model predicts for the previous run's plan; returns every run's plan (fields of `proto` copied in), ranked by the
// iteration predicted on the true kernel times, the earlier run first among equals
void select_periods_retimed(const Trace &t, const Lifetimes &life, uint64_t cap, uint64_t bw, bool duplex,
                            uint64_t min_bytes, uint64_t host_bw, uint64_t host_budget, bool clamp_benefit, int passes,
                            const Plan &proto, std::vector<Plan> &out);
// Address assignment and executor tables; returns false when the arena is too small.
bool assign_addresses(const Trace &t, const Lifetimes &life, uint64_t arena_bytes, Plan &plan);
void validate_plan(const Trace &t, const Lifetimes &life, const Plan &plan);   // throws PlanError

// Performance model of the executor (Section 2.2 of the paper asks how fast the slow tier must be; this
// answers it for a given plan): kernels take tau, each direction's channel moves bytes at `bw` (0 =
// instantly) in issue order, a migration is issued when the kernel before its trigger completes, a
// prefetch also waits for its own offload and for every offload whose deadline has passed, and a kernel
// starts when its predecessor, the prefetches due at it and the offloads due at it have completed.
// Returns the duration of the last of `iterations` consecutive iterations (steady state) in ns.
struct SimResult { int64_t step_ns, compute_ns; };
// stretched (optional): per kernel of the last simulated iteration, its own time plus the stall in front of it
SimResult simulate_plan(const Trace &t, const Plan &plan, uint64_t bw, bool duplex, int iterations,
                        std::vector<int64_t> *stretched = nullptr);
// The same question for an engine that keeps a ready queue per channel, moves chunks of at most chunk_bytes and lets
// urgent requests overtake at chunk boundaries (Section 3.2, "Minimize kernel stalls"; Section 3.3).
SimResult simulate_engine(const Trace &t, const Plan &plan, uint64_t bw, bool duplex, int iterations, uint64_t chunk_bytes,
                          bool urgent_first);

// Address of tensor `id` while kernel k (0..N-1) runs, or UINT64_MAX when it is not resident.
uint64_t address_at(const Plan &plan, int32_t tensor, int32_t k);

}  // namespace tio
