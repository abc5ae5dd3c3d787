// C ABI: handles, views and error reporting for the pure-CPU half (trace, lifetimes, plan).
// The runtime entry points (context, training step) live in runtime.hip.
#include <atomic>
#include <cstring>
#include <new>
#include <stdexcept>
#include <string>

#include "analysis.h"
#include "handles.h"

namespace tio {
thread_local std::string g_last_error;
int fail(int code, const std::string &msg) { g_last_error = msg; return code; }
}  // namespace tio

using namespace tio;

#define TIO_GUARD_BEGIN try {
#define TIO_GUARD_END                                                                   \
    } catch (const PlanError &e) { return fail(e.code, e.msg);                          \
    } catch (const std::invalid_argument &e) { return fail(TIO_ERR_INVALID_ARG, e.what()); \
    } catch (const std::bad_alloc &) { return fail(TIO_ERR_OOM_HOST, "out of host memory"); \
    } catch (const std::exception &e) { return fail(TIO_ERR_INVALID_ARG, e.what()); }

extern "C" {

const char *tio_last_error(void) { return g_last_error.c_str(); }
const char *tio_version(void) { return "teraio-mi355x 0.1 (gfx950)"; }

int tio_param_count(const tio_model_cfg *cfg, int32_t *out_n) {
    if (!cfg || !out_n) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_GUARD_BEGIN
    *out_n = (int32_t)list_params(*cfg).size();
    return TIO_OK;
    TIO_GUARD_END
}

int tio_param_info(const tio_model_cfg *cfg, int32_t index, char *name_buf, size_t name_cap, int64_t *out_rows,
                   int64_t *out_cols) {
    if (!cfg) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_GUARD_BEGIN
    auto ps = list_params(*cfg);
    if (index < 0 || index >= (int)ps.size()) return fail(TIO_ERR_INVALID_ARG, "parameter index out of range");
    if (name_buf && name_cap) {
        std::strncpy(name_buf, ps[index].name.c_str(), name_cap - 1);
        name_buf[name_cap - 1] = 0;
    }
    if (out_rows) *out_rows = ps[index].rows;
    if (out_cols) *out_cols = ps[index].cols;
    return TIO_OK;
    TIO_GUARD_END
}

int tio_trace_build(const tio_model_cfg *cfg, tio_trace **out) {
    if (!cfg || !out) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_GUARD_BEGIN
    Program P = build_program(*cfg);
    tio_trace *h = new tio_trace{trace_from_program(P)};
    *out = h;
    return TIO_OK;
    TIO_GUARD_END
}

int tio_trace_import(const tio_trace_view *v, tio_trace **out) {
    if (!v || !out) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_GUARD_BEGIN
    if (v->n_kernels < 1 || v->n_tensors < 1 || v->n_persistent < 0 || v->n_persistent > v->n_tensors)
        return fail(TIO_ERR_INVALID_ARG, "bad trace sizes");
    if (!v->operand_off || !v->operand_tensor || !v->operand_flags || !v->tensor_bytes || !v->tau_ns)
        return fail(TIO_ERR_INVALID_ARG, "null array in trace view");
    Trace t;
    t.n_kernels = v->n_kernels; t.n_tensors = v->n_tensors; t.n_persistent = v->n_persistent;
    t.operand_off.assign(v->operand_off, v->operand_off + v->n_kernels + 1);
    const int nop = t.operand_off.back();
    if (t.operand_off[0] != 0 || nop < 0) return fail(TIO_ERR_INVALID_ARG, "bad operand offsets");
    for (int k = 0; k < v->n_kernels; ++k)
        if (t.operand_off[k + 1] < t.operand_off[k]) return fail(TIO_ERR_INVALID_ARG, "operand offsets must not decrease");
    t.operand_tensor.assign(v->operand_tensor, v->operand_tensor + nop);
    t.operand_flags.assign(v->operand_flags, v->operand_flags + nop);
    for (int k = 0; k < v->n_kernels; ++k)
        for (int i = t.operand_off[k]; i < t.operand_off[k + 1]; ++i) {
            if (t.operand_tensor[i] < 0 || t.operand_tensor[i] >= v->n_tensors) return fail(TIO_ERR_INVALID_ARG, "operand id out of range");
            if (i > t.operand_off[k] && t.operand_tensor[i] <= t.operand_tensor[i - 1])
                return fail(TIO_ERR_INVALID_ARG, "operands of a kernel must be sorted and distinct");
        }
    t.op.assign(v->n_kernels, 0);
    if (v->op) t.op.assign(v->op, v->op + v->n_kernels);
    t.flops.assign(v->n_kernels, 0);
    if (v->flops) t.flops.assign(v->flops, v->flops + v->n_kernels);
    t.tau.assign(v->tau_ns, v->tau_ns + v->n_kernels);
    for (auto x : t.tau) if (x <= 0) return fail(TIO_ERR_INVALID_ARG, "kernel times must be positive");
    t.tensor_bytes.assign(v->tensor_bytes, v->tensor_bytes + v->n_tensors);
    t.tensor_kind.assign(v->n_tensors, KIND_ACT);
    if (v->tensor_kind) t.tensor_kind.assign(v->tensor_kind, v->tensor_kind + v->n_tensors);
    t.rehash();
    *out = new tio_trace{t};
    return TIO_OK;
    TIO_GUARD_END
}

int tio_trace_set_tau(tio_trace *trace, const int64_t *tau, int32_t n) {
    if (!trace || !tau) return fail(TIO_ERR_INVALID_ARG, "null argument");
    if (n != trace->t.n_kernels) return fail(TIO_ERR_INVALID_ARG, "tau length differs from the kernel count");
    for (int i = 0; i < n; ++i) if (tau[i] <= 0) return fail(TIO_ERR_INVALID_ARG, "kernel times must be positive");
    trace->t.tau.assign(tau, tau + n);
    return TIO_OK;
}

int tio_trace_export(const tio_trace *trace, tio_trace_view *out) {
    if (!trace || !out) return fail(TIO_ERR_INVALID_ARG, "null argument");
    const Trace &t = trace->t;
    out->n_kernels = t.n_kernels; out->n_tensors = t.n_tensors; out->n_persistent = t.n_persistent;
    out->n_operands = (int32_t)t.operand_tensor.size();
    out->op = t.op.data(); out->operand_off = t.operand_off.data();
    out->operand_tensor = t.operand_tensor.data(); out->operand_flags = t.operand_flags.data();
    out->flops = t.flops.data(); out->tau_ns = t.tau.data();
    out->tensor_bytes = t.tensor_bytes.data(); out->tensor_kind = t.tensor_kind.data();
    return TIO_OK;
}

void tio_trace_free(tio_trace *trace) { delete trace; }

int tio_analyze_lifetimes(const tio_trace *trace, tio_lifetimes **out) {
    if (!trace || !out) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_GUARD_BEGIN
    *out = new tio_lifetimes{analyze(trace->t)};
    return TIO_OK;
    TIO_GUARD_END
}

int tio_lifetimes_export(const tio_lifetimes *life, tio_lifetimes_view *out) {
    if (!life || !out) return fail(TIO_ERR_INVALID_ARG, "null argument");
    const Lifetimes &L = life->l;
    out->n_kernels = L.n_kernels; out->n_periods = (int32_t)L.periods.size();
    out->M = L.M.data(); out->tensor = L.v_tensor.data(); out->bytes = L.v_bytes.data();
    out->start = L.v_start.data(); out->end = L.v_end.data();
    return TIO_OK;
}

void tio_lifetimes_free(tio_lifetimes *life) { delete life; }

int tio_build_plan(const tio_trace *trace, const tio_lifetimes *life, uint64_t cap, uint64_t bw,
                   const tio_plan_opts *opts, tio_plan **out) {
    if (!trace || !life || !out) return fail(TIO_ERR_INVALID_ARG, "null argument");
    if (cap == 0) return fail(TIO_ERR_INVALID_ARG, "capacity must be positive");
    TIO_GUARD_BEGIN
    tio_plan_opts o{1, 24, 0, 0, 0, 0, 0, 0};
    if (opts) o = *opts;
    static std::atomic<uint64_t> serial{1};
    tio_plan *h = new tio_plan{build_plan(trace->t, life->l, cap, bw, o)};
    h->p.serial = serial.fetch_add(1);
    *out = h;
    return TIO_OK;
    TIO_GUARD_END
}

int tio_plan_export(const tio_plan *plan, tio_plan_view *out) {
    if (!plan || !out) return fail(TIO_ERR_INVALID_ARG, "null argument");
    const Plan &p = plan->p;
    out->n_kernels = p.n_kernels; out->n_entries = (int32_t)p.entries.size();
    out->n_greedy = p.n_greedy; out->n_forced = p.n_forced; out->n_allocs = (int32_t)p.v_allocs.size();
    out->reserved = 0;
    out->entries = p.entries.data(); out->Mp = p.Mp.data(); out->allocs = p.v_allocs.data();
    out->cap_bytes = p.cap; out->planning_cap_bytes = p.planning_cap;
    out->arena_bytes_needed = p.arena_needed; out->host_bytes_needed = p.host_needed;
    out->bytes_per_direction = p.bytes_moved;
    out->n_pairs = (int32_t)p.pair_tier.size(); out->reserved2 = 0;
    out->pair_tier = p.pair_tier.data();
    out->host_tier_bytes_needed = p.host_tier_needed; out->host_tier_peak_bytes = p.host_peak; out->host_tier_bw = p.host_bw;
    out->retime_pass = p.retime_pass; out->reserved3 = 0;
    return TIO_OK;
}

int tio_plan_validate(const tio_trace *trace, const tio_lifetimes *life, const tio_plan *plan) {
    if (!trace || !life || !plan) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_GUARD_BEGIN
    validate_plan(trace->t, life->l, plan->p);
    return TIO_OK;
    TIO_GUARD_END
}

int tio_plan_simulate(const tio_trace *trace, const tio_plan *plan, uint64_t slow_tier_bw, int32_t duplex,
                      int32_t iterations, int64_t *out_step_ns, int64_t *out_compute_ns) {
    if (!trace || !plan || !out_step_ns || !out_compute_ns) return fail(TIO_ERR_INVALID_ARG, "null argument");
    if (iterations < 1) return fail(TIO_ERR_INVALID_ARG, "iterations must be at least 1");
    if (plan->p.n_kernels != trace->t.n_kernels) return fail(TIO_ERR_PLAN_STALE, "plan was built from a different trace");
    TIO_GUARD_BEGIN
    const SimResult r = simulate_plan(trace->t, plan->p, slow_tier_bw, duplex != 0, iterations);
    *out_step_ns = r.step_ns;
    *out_compute_ns = r.compute_ns;
    return TIO_OK;
    TIO_GUARD_END
}

int tio_plan_simulate_engine(const tio_trace *trace, const tio_plan *plan, uint64_t slow_tier_bw, int32_t duplex,
                             int32_t iterations, uint64_t chunk_bytes, int32_t urgent_first, int64_t *out_step_ns,
                             int64_t *out_compute_ns) {
    if (!trace || !plan || !out_step_ns || !out_compute_ns) return fail(TIO_ERR_INVALID_ARG, "null argument");
    if (iterations < 1) return fail(TIO_ERR_INVALID_ARG, "iterations must be at least 1");
    if (plan->p.n_kernels != trace->t.n_kernels) return fail(TIO_ERR_PLAN_STALE, "plan was built from a different trace");
    TIO_GUARD_BEGIN
    const SimResult r = simulate_engine(trace->t, plan->p, slow_tier_bw, duplex != 0, iterations, chunk_bytes, urgent_first != 0);
    *out_step_ns = r.step_ns;
    *out_compute_ns = r.compute_ns;
    return TIO_OK;
    TIO_GUARD_END
}

void tio_plan_free(tio_plan *plan) { delete plan; }

}  // extern "C"
