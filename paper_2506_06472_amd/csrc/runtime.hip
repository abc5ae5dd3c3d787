// Runtime of the training step: context, tensor location table, plan installation and the
// migration engine (Section 3.3 of the paper).  The host walks the kernel schedule once per
// iteration; before kernel k it issues the plan entries triggered at k (offloads on the
// device-to-host stream, prefetches on the host-to-device stream), then makes the compute stream
// wait for exactly the events kernel k depends on (its prefetched operands, and the offloads that
// empty address ranges its outputs reuse), then launches kernel k.  A late migration therefore
// stalls the kernel that needs it and nothing else, which is the paper's "kernel stall".  The slow tier is pinned host
// memory (or a device buffer outside the arena, or a file).  A tier with an emulated bandwidth (paced_pool.h) is run by
// threads of its own with a ready queue per direction: transfers move in chunks, an urgent request whose dependencies are
// met overtakes the pending ones at a chunk boundary, and a blocked request never holds up a ready one (Section 3.2,
// "Minimize kernel stalls").  A tier in a file (file_tier.h) has threads of its own too and serves each direction in the
// order submitted; unthrottled memory tiers are plain hipMemcpyAsync on the tier's two streams, also in the order submitted
// (there urgent entries only come first among the entries of one trigger point).  With engine threads the host blocks, before
// kernel k, until the completion events kernel k depends on have been recorded by those threads.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "analysis.h"
#include "file_tier.h"
#include "handles.h"
#include "kernels.h"
#include "paced_pool.h"

using namespace tio;

namespace {

constexpr uint64_t kReservedTail = 4096;     // end of the arena kept for the runtime

struct HipError { hipError_t e; const char *what; };
#define HIPCHK(x)                                   \
    do {                                            \
        hipError_t _e = (x);                        \
        if (_e != hipSuccess) throw HipError{_e, #x}; \
    } while (0)

inline uint16_t host_f32_to_bf16(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
inline float host_bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

}  // namespace

struct tio_ctx {
    tio_model_cfg cfg;
    tio_runtime_cfg rt;
    Program prog;
    Trace trace;
    Lifetimes life;
    hipStream_t sc = nullptr, sd = nullptr, sh = nullptr;
    hipStream_t sd1 = nullptr, sh1 = nullptr;            // copy streams of the host-memory tier
    uint8_t *arena = nullptr, *host = nullptr, *host1 = nullptr;
    uint64_t bw1 = 0;                                    // bandwidth enforced on the host-memory tier
    uint64_t arena_usable = 0;
    std::vector<uint64_t> home;                          // host offset of every persistent tensor
    uint64_t home_bytes = 0;
    uint64_t bw = 0;
    bool pool_dev = false;                               // the slow-tier pool is device memory (stand-in when the host cannot pin enough)

    Plan plan;                                           // installed plan (copy)
    bool installed = false, params_dirty = true;
    bool failed = false;                                 // a step stopped half-way (HIP or I/O error): tensor state unknown
    std::vector<uint8_t> loaded;                         // per parameter: tio_params_load has been called
    std::vector<uint8_t> reloaded;                       // per parameter: loaded since the step counter was last reset
    size_t n_reloaded = 0;
    std::vector<uint8_t> on_dev;                         // per persistent tensor: latest version is in the arena
    std::vector<uint64_t> dev_addr;
    std::vector<uint8_t> in_host1;                       // per persistent tensor: latest version is in a host-tier slot
    std::vector<uint64_t> host1_off;
    std::vector<std::vector<uint64_t>> ptrs;             // per kernel, per role: arena offset (UINT64_MAX = absent)
    std::vector<hipEvent_t> ev_kernel, ev_off, ev_pre, ev_t0, ev_t1;
    std::vector<uint8_t> rec_kernel, rec_off, rec_pre;
    int step = 0;
    float *loss_pinned = nullptr;                         // 4 KiB of pinned host memory owned by the context
    std::vector<std::vector<float>> grads;
    std::vector<int64_t> last_times;                      // per-kernel ns of the last step run with timing
    std::vector<hipEvent_t> ev_c0, ev_c1;                 // timeline mode: begin / end of every migration
    hipEvent_t ev_step0 = nullptr;
    std::vector<int64_t> tl_k0, tl_k1, tl_c0, tl_c1;      // timeline of the last step run in timeline mode (ns from step start)
    bool timeline = false;
    Plan uncapped;
    bool have_uncapped = false;
    // slow tier in a file: persistent tensors and migrated periods have 4096-byte aligned file ranges
    std::unique_ptr<FileTier> ft;
    std::vector<uint64_t> home_file;                      // per persistent tensor
    uint64_t home_file_bytes = 0;
    std::vector<uint64_t> pair_file;                      // per pair of the installed plan (slow-tier pairs only)
    std::vector<hipEvent_t> ev_req;                       // per plan entry: compute progress at submission
    std::vector<uint64_t> req_seq;                        // per plan entry: sequence number of its last request
    std::vector<uint64_t> off_seq, pre_seq;               // per pair: sequence number of its last offload / prefetch request
    std::vector<MigrationEngine::Dep> ev_off_user;        // per pair: last engine prefetch that waits for ev_off[pair], recorded by this thread
    // memory tiers with an emulated bandwidth: slow tier, host-memory tier
    std::unique_ptr<PacedPool> pp0, pp1;
};

namespace {

void destroy_events(std::vector<hipEvent_t> &v) {
    for (hipEvent_t e : v) if (e) (void)hipEventDestroy(e);
    v.clear();
}
void make_events(std::vector<hipEvent_t> &v, size_t n, bool timing) {
    destroy_events(v);
    v.assign(n, nullptr);
    for (size_t i = 0; i < n; ++i) HIPCHK(hipEventCreateWithFlags(&v[i], timing ? hipEventDefault : hipEventDisableTiming));
}

// debugging aid (tio_runtime_cfg.poison_freed): a vacated arena range is overwritten with NaN patterns, so that a
// kernel that wrongly read it would poison the loss
void poison_range(hipStream_t s, void *dev, uint64_t bytes) { k::fill_u32(s, dev, 0xFFFFFFFFu, (int64_t)(bytes / 4)); }

// the engine that moves the pairs of a tier, or nullptr when they are plain copies on the tier's streams
MigrationEngine *engine_of(tio_ctx *c, int tier) {
    if (tier == 1) return c->pp1 && c->bw1 ? c->pp1.get() : nullptr;
    if (c->ft) return c->ft.get();
    return c->pp0 && c->bw ? c->pp0.get() : nullptr;
}

void sync_all(tio_ctx *c) {
    // an engine's request may depend on another engine's, never on work that is not yet submitted
    if (c->ft) c->ft->drain();
    if (c->pp0) c->pp0->drain();
    if (c->pp1) c->pp1->drain();
    HIPCHK(hipStreamSynchronize(c->sc));
    HIPCHK(hipStreamSynchronize(c->sd));
    HIPCHK(hipStreamSynchronize(c->sh));
    if (c->sd1) HIPCHK(hipStreamSynchronize(c->sd1));
    if (c->sh1) HIPCHK(hipStreamSynchronize(c->sh1));
}

// set-up path: the home slot of persistent tensor t on the slow tier (pinned pool, device pool or file)
void home_from_dev(tio_ctx *c, int t, const void *dev) {
    if (c->ft) c->ft->from_device(c->home_file[t], dev, c->prog.tensors[t].bytes);
    else HIPCHK(hipMemcpy(c->host + c->home[t], dev, c->prog.tensors[t].bytes, hipMemcpyDefault));
}
void home_to_dev(tio_ctx *c, int t, void *dev) {
    if (c->ft) c->ft->to_device(c->home_file[t], dev, c->prog.tensors[t].bytes);
    else HIPCHK(hipMemcpy(dev, c->host + c->home[t], c->prog.tensors[t].bytes, hipMemcpyDefault));
}
void home_from_host(tio_ctx *c, int t, const void *src, uint64_t bytes) {
    if (c->ft) c->ft->write_host(c->home_file[t], src, bytes);
    else if (c->pool_dev) HIPCHK(hipMemcpy(c->host + c->home[t], src, bytes, hipMemcpyHostToDevice));
    else std::memcpy(c->host + c->home[t], src, bytes);
}
void home_to_host(tio_ctx *c, int t, void *dst, uint64_t bytes) {
    if (c->ft) c->ft->read_host(c->home_file[t], dst, bytes);
    else if (c->pool_dev) HIPCHK(hipMemcpy(dst, c->host + c->home[t], bytes, hipMemcpyDeviceToHost));
    else std::memcpy(dst, c->host + c->home[t], bytes);
}

// brings the latest version of every persistent tensor into its home slot on the slow tier
void gather_to_home(tio_ctx *c) {
    sync_all(c);
    if (!c->installed) return;
    for (int t = 0; t < c->prog.n_persistent; ++t) {
        if (c->on_dev[t]) home_from_dev(c, t, c->arena + c->dev_addr[t]);
        else if (c->in_host1[t])      // offloaded to the host-memory tier: that slot holds the latest version
            home_from_host(c, t, c->host1 + c->host1_off[t], c->prog.tensors[t].bytes);
        c->in_host1[t] = 0;
    }
    // a device-to-device hipMemcpy may return before the copy has run, and the context's streams do not
    // wait for the null stream
    if (c->pool_dev) HIPCHK(hipDeviceSynchronize());
}

void install_plan(tio_ctx *c, const Plan &p) {
    const int N = c->trace.n_kernels;
    if (p.structure_hash != c->trace.structure_hash || p.n_kernels != N)
        throw PlanError{TIO_ERR_PLAN_STALE, "plan was built from a different trace"};
    if (p.arena_needed > c->arena_usable)
        throw PlanError{TIO_ERR_ARENA_TOO_SMALL, "plan needs " + std::to_string(p.arena_needed) + " arena bytes, context has " +
                                                     std::to_string(c->arena_usable)};
    std::vector<uint64_t> pair_file(p.pairs.size(), 0);
    uint64_t file_needed = c->home_file_bytes;
    if (c->ft) {
        for (size_t i = 0; i < p.pairs.size(); ++i) {
            const Pair &pr = p.pairs[i];
            if (pr.tier != 0) continue;
            if (pr.tensor < c->prog.n_persistent) pair_file[i] = c->home_file[pr.tensor];
            else { pair_file[i] = file_needed; file_needed += (pr.bytes + FileTier::kAlign - 1) / FileTier::kAlign * FileTier::kAlign; }
        }
    }
    if ((c->ft ? file_needed : p.host_needed) > c->rt.host_bytes)
        throw PlanError{TIO_ERR_OOM_HOST, "plan needs " + std::to_string(c->ft ? file_needed : p.host_needed) +
                                              " slow-tier bytes, pool has " + std::to_string(c->rt.host_bytes)};
    if (p.host_tier_needed > 0 && (!c->host1 || !c->sd1 || !c->sh1 || p.host_tier_needed > c->rt.host_tier_bytes))
        throw PlanError{TIO_ERR_OOM_HOST, "plan needs " + std::to_string(p.host_tier_needed) +
                                              " bytes of a host-memory tier with its two streams, context has " +
                                              std::to_string(c->host1 ? c->rt.host_tier_bytes : 0)};
    const int np = c->prog.n_persistent;
    for (int t = 0; t < np; ++t)
        if (p.persistent_home[t] != c->home[t]) throw PlanError{TIO_ERR_PLAN_INVALID, "home slot mismatch"};
    std::vector<std::vector<uint64_t>> ptrs(N, std::vector<uint64_t>(kMaxRoles, UINT64_MAX));
    for (int k = 0; k < N; ++k)
        for (int r = 0; r < kMaxRoles; ++r) {
            const int t = c->prog.kernels[k].t[r];
            if (t < 0) continue;
            const uint64_t a = address_at(p, t, k);
            if (a == UINT64_MAX) throw PlanError{TIO_ERR_PLAN_INVALID, "operand not resident at kernel " + std::to_string(k)};
            if (a + c->prog.tensors[t].bytes > c->arena_usable) throw PlanError{TIO_ERR_PLAN_INVALID, "address outside the arena"};
            ptrs[k][r] = a;
        }
    // Everything that can reject the plan has been checked.  From here on the context has no plan until the new one
    // is complete: if a step below fails, the latest version of every persistent tensor is in its home slot (that is
    // what gather_to_home leaves) and the next call installs from there.
    gather_to_home(c);
    c->installed = false;
    if (c->ft) {
        c->ft->resize(file_needed);
        c->ft->set_pairs((int)p.pairs.size());
        c->pair_file = pair_file;
    }
    if (c->pp0) c->pp0->set_pairs((int)p.pairs.size());
    if (c->pp1) c->pp1->set_pairs((int)p.pairs.size());
    c->plan = p;
    c->on_dev.assign(np, 0);
    c->dev_addr.assign(np, 0);
    c->in_host1.assign(np, 0);
    c->host1_off.assign(np, 0);
    for (int t = 0; t < np; ++t) {
        const uint64_t a = address_at(p, t, 0);
        if (a == UINT64_MAX) continue;
        // resident at the iteration boundary unless a prefetch issued at trigger 0 brings it in
        bool by_prefetch_at_0 = false;
        for (int ai : p.alloc_of[t]) {
            const Alloc &al = p.allocs[ai];
            if (!al.whole_cycle && al.born_by_pair >= 0 && al.first == 0) by_prefetch_at_0 = true;
        }
        if (by_prefetch_at_0) continue;
        home_to_dev(c, t, c->arena + a);
        c->on_dev[t] = 1;
        c->dev_addr[t] = a;
    }
    if (c->pool_dev) HIPCHK(hipDeviceSynchronize());     // see gather_to_home
    c->ptrs = std::move(ptrs);
    make_events(c->ev_kernel, N, false);
    make_events(c->ev_off, p.pairs.size(), false);
    make_events(c->ev_pre, p.pairs.size(), false);
    c->rec_kernel.assign(N, 0);
    c->rec_off.assign(p.pairs.size(), 0);
    c->rec_pre.assign(p.pairs.size(), 0);
    make_events(c->ev_req, p.entries.size(), false);
    c->req_seq.assign(p.entries.size(), 0);
    c->off_seq.assign(p.pairs.size(), 0);
    c->pre_seq.assign(p.pairs.size(), 0);
    c->ev_off_user.assign(p.pairs.size(), MigrationEngine::Dep{nullptr, -1, 0});
    c->installed = true;
    c->params_dirty = false;
}

void launch(tio_ctx *c, int k) {
    const KernelRec &r = c->prog.kernels[k];
    const tio_model_cfg &m = c->cfg;
    auto P = [&](int role) -> void * { return c->ptrs[k][role] == UINT64_MAX ? nullptr : (void *)(c->arena + c->ptrs[k][role]); };
    const int dt = m.precision;
    const bool rms = m.arch == TIO_ARCH_LLAMA;
    // B: sequences of one micro-batch
    const int64_t B = m.batch / (m.micro_batches > 1 ? m.micro_batches : 1), T = m.seq_len, H = m.n_heads, dh = m.d_model / m.n_heads;
    hipStream_t s = c->sc;
    switch (r.op) {
    case OP_EMBED_FWD: k::embed_fwd(s, dt, (const int32_t *)P(0), P(1), P(2), P(3), r.p[0], r.p[1], r.p[2]); break;
    case OP_NORM_FWD: k::norm_fwd(s, dt, rms, P(0), P(1), P(2), P(3), (float *)P(4), r.p[0], r.p[1], m.norm_eps); break;
    case OP_GEMM:
        k::gemm(s, dt, false, false, r.p[0], r.p[1], r.p[2], P(0), r.p[2], P(1), r.p[2], P(2), P(3), r.p[3], P(4), r.p[3], nullptr, nullptr, 1);
        break;
    case OP_ROPE_FWD: k::rope(s, dt, P(0), B, T, H, dh, m.rope_theta, false); break;
    case OP_ROPE_BWD: k::rope(s, dt, P(0), B, T, H, dh, m.rope_theta, true); break;
    case OP_ATTN_FWD: k::attn_fwd(s, dt, P(0), P(1), (float *)P(2), B, T, H, dh); break;
    case OP_GELU_FWD: k::gelu_fwd(s, dt, P(0), P(1), r.p[0]); break;
    case OP_SWIGLU_FWD: k::swiglu_fwd(s, dt, P(0), P(1), r.p[0], r.p[1]); break;
    case OP_CE_FWD_BWD: k::ce_fwd_bwd(s, dt, P(0), (const int32_t *)P(1), (float *)P(2), r.p[0], r.p[1], r.p[2], r.p[3]); break;
    case OP_LOSS_REDUCE: k::loss_reduce(s, (const float *)P(0), (float *)P(1), r.p[0], r.p[1], r.p[2] != 0); break;
    case OP_GEMM_DX:   // dX[S,n_in] = dY[S,n_out] . W[n_out,n_in]: the weight has the contraction index slow
        k::gemm(s, dt, false, true, r.p[0], r.p[1], r.p[2], P(0), r.p[3], P(1), r.p[1], nullptr, nullptr, 0, P(2), r.p[1], nullptr, nullptr, 1);
        break;
    case OP_GEMM_DW:   // dW[n_out,n_in] = dY^T . X: both operands have the contraction index (tokens) slow;
                       // the row sums of dY^T are the bias gradient
        k::gemm(s, dt, true, true, r.p[0], r.p[1], r.p[2], P(0), r.p[3], P(1), r.p[1], nullptr, nullptr, 0, P(2), r.p[1], P(3), P(4), (int)r.p[4], r.p[5] != 0);
        break;
    case OP_GELU_BWD: k::gelu_bwd(s, dt, P(0), P(1), r.p[0]); break;
    case OP_SWIGLU_BWD: k::swiglu_bwd(s, dt, P(0), P(1), P(2), r.p[0], r.p[1]); break;
    case OP_NORM_BWD:
        k::norm_bwd(s, dt, rms, P(0), P(1), (const float *)P(2), P(3), P(4), P(5), (float *)P(6), r.p[0], r.p[1], r.p[2]);
        break;
    case OP_NORM_BWD_PARAMS: k::norm_bwd_params(s, dt, rms, (const float *)P(0), P(1), P(2), r.p[0], r.p[1], r.p[2] != 0); break;
    case OP_ATTN_BWD_PRE: k::attn_bwd_pre(s, dt, P(0), P(1), (float *)P(2), B, T, H, dh); break;
    case OP_ATTN_BWD: k::attn_bwd(s, dt, P(0), P(1), (const float *)P(2), (const float *)P(3), P(4), B, T, H, dh); break;
    case OP_EMBED_BWD: k::embed_bwd(s, dt, P(0), (const int32_t *)P(1), P(2), r.p[0], r.p[1], r.p[2], r.p[3] != 0); break;
    case OP_POSEMB_BWD: k::posemb_bwd(s, dt, P(0), P(1), r.p[0], r.p[1], r.p[2], r.p[3] != 0); break;
    case OP_ADAMW: {
        const double t = (double)(c->step + 1);
        const float bc1 = (float)(1.0 - std::pow((double)m.beta1, t)), bc2 = (float)(1.0 - std::pow((double)m.beta2, t));
        k::adamw(s, dt, P(0), P(1), (float *)P(2), (float *)P(3), (float *)P(4), r.p[0], m.lr, m.beta1, m.beta2, m.adam_eps,
                 m.weight_decay, bc1, bc2);
        break;
    }
    default: throw PlanError{TIO_ERR_INVALID_ARG, "unknown operator"};
    }
    HIPCHK(hipGetLastError());
}

void capture_grad(tio_ctx *c, int k) {
    const KernelRec &r = c->prog.kernels[k];
    int pi = -1;
    for (int i = 0; i < (int)c->prog.params.size(); ++i) if (c->prog.params[i].grad == r.t[0]) pi = i;
    if (pi < 0) return;
    const int64_t n = r.p[0];
    HIPCHK(hipStreamSynchronize(c->sc));
    std::vector<float> &g = c->grads[pi];
    g.resize(n);
    if (c->cfg.precision == TIO_PREC_BF16) {
        std::vector<uint16_t> tmp(n);
        HIPCHK(hipMemcpy(tmp.data(), c->arena + c->ptrs[k][0], n * 2, hipMemcpyDeviceToHost));
        for (int64_t i = 0; i < n; ++i) g[i] = host_bf16_to_f32(tmp[i]);
    } else {
        HIPCHK(hipMemcpy(g.data(), c->arena + c->ptrs[k][0], n * 4, hipMemcpyDeviceToHost));
    }
}

// one iteration; timing != nullptr: per-kernel elapsed ns measured with events
void check_ids(const tio_ctx *c, const int32_t *tokens, const int32_t *labels) {
    const int64_t S = (int64_t)c->cfg.batch * c->cfg.seq_len;
    for (int64_t i = 0; i < S; ++i) {
        if (tokens[i] < 0 || tokens[i] >= c->cfg.vocab || labels[i] < 0 || labels[i] >= c->cfg.vocab)
            throw PlanError{TIO_ERR_INVALID_ARG, "token or label id outside the vocabulary"};
    }
}

void run_step_body(tio_ctx *c, const int32_t *tokens, const int32_t *labels, bool capture, std::vector<int64_t> *timing,
                   tio_step_stats *st) {
    const int N = c->trace.n_kernels;
    const Plan &p = c->plan;
    const int64_t S = (int64_t)c->cfg.batch * c->cfg.seq_len;
    if (capture) c->grads.assign(c->prog.params.size(), {});
    if (timing) { if ((int)c->ev_t0.size() != N) { make_events(c->ev_t0, N, true); make_events(c->ev_t1, N, true); } }
    const bool tl = c->timeline && timing;
    if (tl) {
        if (c->ev_c0.size() != p.entries.size()) { make_events(c->ev_c0, p.entries.size(), true); make_events(c->ev_c1, p.entries.size(), true); }
        if (!c->ev_step0) HIPCHK(hipEventCreate(&c->ev_step0));
        sync_all(c);
        HIPCHK(hipEventRecord(c->ev_step0, c->sc));
    }
    std::vector<uint8_t> issued(tl ? p.entries.size() : 0, 0);
    const auto w0 = std::chrono::steady_clock::now();
    {   // one token and one label buffer per micro-batch (consecutive groups of sequences)
        const int64_t nmb = (int64_t)c->prog.tokens_ids.size(), Sm = S / nmb;
        for (int64_t j = 0; j < nmb; ++j) {
            HIPCHK(hipMemcpyAsync(c->arena + address_at(p, c->prog.tokens_ids[j], 0), tokens + j * Sm, Sm * 4, hipMemcpyHostToDevice, c->sc));
            HIPCHK(hipMemcpyAsync(c->arena + address_at(p, c->prog.labels_ids[j], 0), labels + j * Sm, Sm * 4, hipMemcpyHostToDevice, c->sc));
        }
    }
    uint64_t d2h = 0, h2d = 0;
    int nmig = 0;
    for (int k = 0; k < N; ++k) {
        const int prev = (k + N - 1) % N;
        for (int ei : p.entries_at[k]) {
            const tio_plan_entry &e = p.entries[ei];
            const Pair &pr = p.pairs[e.pair];
            const bool persistent = e.tensor < c->prog.n_persistent;
            // destination of this pair: the slow tier's pool (or file) and streams, or the host-memory tier's
            const bool t1 = pr.tier == 1;
            hipStream_t so = t1 ? c->sd1 : c->sd, sp = t1 ? c->sh1 : c->sh;
            uint8_t *pool = t1 ? c->host1 : c->host;
            MigrationEngine *eng = engine_of(c, pr.tier);     // nullptr: plain copies on the tier's streams
            auto progress_event = [&]() {                     // compute progress at this trigger point, for an engine
                if (c->req_seq[ei]) eng->wait_consumed(e.kind == TIO_OFFLOAD ? 0 : 1, c->req_seq[ei]);
                HIPCHK(hipEventRecord(c->ev_req[ei], c->sc));
                return c->ev_req[ei];
            };
            auto place = [&]() -> uint64_t {                  // the pair's place on its tier, as its engine addresses it
                return (c->ft && !t1) ? c->pair_file[e.pair] : (uint64_t)(uintptr_t)(pool + pr.host_offset);
            };
            if (e.kind == TIO_OFFLOAD) {
                // first iteration after a plan is installed: an offload that belongs to the end of the
                // previous iteration (trigger wraps to the start of this one) has nothing to copy, the
                // slow-tier home slot already holds the latest version
                if (persistent && !c->on_dev[e.tensor]) continue;
                const Alloc &al = p.allocs[pr.alloc_before];
                if (eng) {
                    const uint64_t seq = eng->submit_offload(e.pair, progress_event(), c->arena + al.address, place(), pr.bytes,
                                                             c->ev_off[e.pair], tl ? c->ev_c0[ei] : nullptr, tl ? c->ev_c1[ei] : nullptr,
                                                             e.urgent != 0);
                    c->req_seq[ei] = c->off_seq[e.pair] = seq;
                    if (tl) issued[ei] = 1;
                } else {
                    // a prefetch run by an engine may still have to take over this pair's previous event
                    if (c->ev_off_user[e.pair].eng) {
                        c->ev_off_user[e.pair].eng->wait_consumed(1, c->ev_off_user[e.pair].seq);
                        c->ev_off_user[e.pair] = {nullptr, -1, 0};
                    }
                    if (c->rec_kernel[prev]) HIPCHK(hipStreamWaitEvent(so, c->ev_kernel[prev], 0));
                    if (tl) { HIPCHK(hipEventRecord(c->ev_c0[ei], so)); issued[ei] = 1; }
                    HIPCHK(hipMemcpyAsync(pool + pr.host_offset, c->arena + al.address, pr.bytes, (c->pool_dev && !t1) ? hipMemcpyDeviceToDeviceNoCU : hipMemcpyDefault, so));
                    if (c->rt.poison_freed) poison_range(so, c->arena + al.address, pr.bytes);
                    if (tl) HIPCHK(hipEventRecord(c->ev_c1[ei], so));
                    HIPCHK(hipEventRecord(c->ev_off[e.pair], so));
                }
                c->rec_off[e.pair] = 1;
                if (persistent) {
                    c->on_dev[e.tensor] = 0;
                    c->in_host1[e.tensor] = t1 ? 1 : 0;
                    c->host1_off[e.tensor] = pr.host_offset;
                }
                d2h += pr.bytes;
            } else {
                const Alloc &al = p.allocs[pr.alloc_after];
                // a persistent tensor whose offload to the host-memory tier belongs to an iteration that never
                // ran (first iteration after the plan was installed) is still in its slow-tier home slot
                const bool from_home = t1 && persistent && !c->in_host1[e.tensor];
                if (from_home && c->ft) {
                    // rare: that home is a range of the file.  Everything issued so far is allowed to finish,
                    // then the tensor is read synchronously.
                    sync_all(c);
                    c->ft->to_device(c->home_file[e.tensor], c->arena + al.address, pr.bytes);
                    HIPCHK(hipEventRecord(c->ev_pre[e.pair], sp));
                    c->pre_seq[e.pair] = 0;
                } else if (eng) {
                    MigrationEngine::Dep written{eng, e.pair, c->rec_off[e.pair] ? c->off_seq[e.pair] : 0};
                    std::vector<MigrationEngine::Dep> landed;
                    std::vector<hipEvent_t> more;
                    for (int q : al.wait_pairs) {
                        if (!c->rec_off[q]) continue;
                        if (MigrationEngine *eq = engine_of(c, p.pairs[q].tier)) landed.push_back({eq, q, c->off_seq[q]});
                        else more.push_back(c->ev_off[q]);   // recorded above by this thread, on the other tier's stream
                    }
                    const uint64_t where = from_home ? (uint64_t)(uintptr_t)(c->host + c->home[e.tensor]) : place();
                    const uint64_t seq = eng->submit_prefetch(e.pair, progress_event(), c->arena + al.address, where, pr.bytes,
                                                              written, landed, more, c->ev_pre[e.pair],
                                                              tl ? c->ev_c0[ei] : nullptr, tl ? c->ev_c1[ei] : nullptr, e.urgent != 0);
                    c->req_seq[ei] = c->pre_seq[e.pair] = seq;
                    for (int q : al.wait_pairs)
                        if (c->rec_off[q] && !engine_of(c, p.pairs[q].tier)) c->ev_off_user[q] = {eng, q, seq};
                    if (tl) issued[ei] = 1;
                } else {
                    const uint8_t *src = from_home ? c->host + c->home[e.tensor] : pool + pr.host_offset;
                    if (c->rec_kernel[prev]) HIPCHK(hipStreamWaitEvent(sp, c->ev_kernel[prev], 0));
                    if (c->rec_off[e.pair]) HIPCHK(hipStreamWaitEvent(sp, c->ev_off[e.pair], 0));
                    for (int q : al.wait_pairs) {
                        if (!c->rec_off[q]) continue;
                        if (MigrationEngine *eq = engine_of(c, p.pairs[q].tier)) eq->wait_offload_recorded(q, c->off_seq[q]);
                        HIPCHK(hipStreamWaitEvent(sp, c->ev_off[q], 0));
                    }
                    if (tl) { HIPCHK(hipEventRecord(c->ev_c0[ei], sp)); issued[ei] = 1; }
                    HIPCHK(hipMemcpyAsync(c->arena + al.address, src, pr.bytes, (c->pool_dev && !(t1 && !from_home)) ? hipMemcpyDeviceToDeviceNoCU : hipMemcpyDefault, sp));
                    if (tl) HIPCHK(hipEventRecord(c->ev_c1[ei], sp));
                    HIPCHK(hipEventRecord(c->ev_pre[e.pair], sp));
                    c->pre_seq[e.pair] = 0;
                }
                c->rec_pre[e.pair] = 1;
                if (persistent) { c->on_dev[e.tensor] = 1; c->dev_addr[e.tensor] = al.address; c->in_host1[e.tensor] = 0; }
                h2d += pr.bytes;
            }
            ++nmig;
        }
        for (int q : p.kernel_wait_pre[k]) if (c->rec_pre[q]) {
            if (c->pre_seq[q]) if (MigrationEngine *eq = engine_of(c, p.pairs[q].tier)) eq->wait_prefetch_recorded(q, c->pre_seq[q]);
            HIPCHK(hipStreamWaitEvent(c->sc, c->ev_pre[q], 0));
        }
        for (int q : p.kernel_wait_off[k]) if (c->rec_off[q]) {
            if (c->off_seq[q]) if (MigrationEngine *eq = engine_of(c, p.pairs[q].tier)) eq->wait_offload_recorded(q, c->off_seq[q]);
            HIPCHK(hipStreamWaitEvent(c->sc, c->ev_off[q], 0));
        }
        if (capture && c->prog.kernels[k].op == OP_ADAMW) capture_grad(c, k);
        if (timing) HIPCHK(hipEventRecord(c->ev_t0[k], c->sc));
        launch(c, k);
        if (timing) HIPCHK(hipEventRecord(c->ev_t1[k], c->sc));
        // the scalar loss lives only until later kernels reuse its range: copy it out in stream order
        if (c->prog.kernels[k].op == OP_LOSS_REDUCE)
            HIPCHK(hipMemcpyAsync(c->loss_pinned, c->arena + c->ptrs[k][1], 4, hipMemcpyDeviceToHost, c->sc));
        if (p.kernel_needs_event[k]) { HIPCHK(hipEventRecord(c->ev_kernel[k], c->sc)); c->rec_kernel[k] = 1; }
    }
    HIPCHK(hipStreamSynchronize(c->sc));
    if (c->ft) c->ft->check();
    if (c->pp0) c->pp0->check();
    if (c->pp1) c->pp1->check();
    const float loss = *c->loss_pinned;
    const auto w1 = std::chrono::steady_clock::now();
    c->step += 1;
    if (tl) {
        sync_all(c);
        auto rel = [&](hipEvent_t e) { float ms = 0.f; HIPCHK(hipEventElapsedTime(&ms, c->ev_step0, e)); return (int64_t)std::llround((double)ms * 1e6); };
        c->tl_k0.assign(N, 0); c->tl_k1.assign(N, 0);
        c->tl_c0.assign(p.entries.size(), -1); c->tl_c1.assign(p.entries.size(), -1);
        for (int k = 0; k < N; ++k) { c->tl_k0[k] = rel(c->ev_t0[k]); c->tl_k1[k] = rel(c->ev_t1[k]); }
        for (size_t i = 0; i < p.entries.size(); ++i) if (issued[i]) { c->tl_c0[i] = rel(c->ev_c0[i]); c->tl_c1[i] = rel(c->ev_c1[i]); }
    }
    if (timing) {
        timing->assign(N, 0);
        for (int k = 0; k < N; ++k) {
            float ms = 0.f;
            HIPCHK(hipEventElapsedTime(&ms, c->ev_t0[k], c->ev_t1[k]));
            (*timing)[k] = std::max<int64_t>(1, (int64_t)std::llround((double)ms * 1e6));
        }
    }
    if (st) {
        std::memset(st, 0, sizeof(*st));
        st->loss = loss;
        st->step = c->step;
        st->wall_ns = std::chrono::duration_cast<std::chrono::nanoseconds>(w1 - w0).count();
        st->d2h_bytes = d2h; st->h2d_bytes = h2d;
        st->n_kernels = N; st->n_migrations = nmig;
        if (timing) for (int64_t x : *timing) st->kernel_ns += x;
        if (tl)
            for (size_t i = 0; i < p.entries.size(); ++i)
                if (issued[i]) (p.entries[i].kind == TIO_OFFLOAD ? st->d2h_busy_ns : st->h2d_busy_ns) += c->tl_c1[i] - c->tl_c0[i];
    }
}

// An error after the first launch leaves tensors half updated and transfers in flight: the context refuses further
// steps from then on.
void run_step(tio_ctx *c, const int32_t *tokens, const int32_t *labels, bool capture, std::vector<int64_t> *timing,
              tio_step_stats *st) {
    try {
        run_step_body(c, tokens, labels, capture, timing, st);
    } catch (...) {
        c->failed = true;
        throw;
    }
}

// ids are validated, and a context that failed earlier is refused, before anything is touched
void step_preconditions(const tio_ctx *c, const int32_t *tokens, const int32_t *labels) {
    if (c->failed) throw PlanError{TIO_ERR_HIP, "an earlier step on this context stopped with an error: destroy the context"};
    check_ids(c, tokens, labels);
}

const Plan &uncapped_plan(tio_ctx *c) {
    if (!c->have_uncapped) {
        tio_plan_opts o{1, 0, 0, UINT64_MAX};
        c->uncapped = build_plan(c->trace, c->life, UINT64_MAX / 2, 0, o);
        c->uncapped.serial = UINT64_MAX;
        c->have_uncapped = true;
    }
    return c->uncapped;
}

void ensure_plan(tio_ctx *c, const tio_plan *plan) {
    const Plan &want = plan ? plan->p : uncapped_plan(c);
    if (!c->installed || c->params_dirty || c->plan.serial != want.serial) install_plan(c, want);
}

}  // namespace

#define TIO_RT_BEGIN try {
#define TIO_RT_END                                                                                              \
    } catch (const PlanError &e) { return fail(e.code, e.msg);                                                  \
    } catch (const HipError &e) { return fail(TIO_ERR_HIP, std::string(e.what) + ": " + hipGetErrorString(e.e)); \
    } catch (const EngineError &e) { return fail(TIO_ERR_IO, e.msg);                                            \
    } catch (const std::exception &e) { return fail(TIO_ERR_INVALID_ARG, e.what()); }

extern "C" {

int tio_ctx_create(const tio_model_cfg *cfg, const tio_runtime_cfg *rt, tio_ctx **out) {
    if (!cfg || !rt || !out) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_RT_BEGIN
    const bool file_tier = rt->slow_tier_file != nullptr;
    if (!rt->arena || (!rt->host_pool && !file_tier) || rt->arena_bytes < (1u << 16))
        return fail(TIO_ERR_INVALID_ARG, "arena and slow-tier pool (or file) are required");
    if (file_tier && (rt->host_pool || rt->pool_on_device)) return fail(TIO_ERR_INVALID_ARG, "the slow tier is either a pool or a file");
    if (((uintptr_t)rt->arena & 255) || ((uintptr_t)rt->host_pool & 255)) return fail(TIO_ERR_INVALID_ARG, "arena and pool must be 256-byte aligned");
    const int dh = cfg->d_model / std::max(1, cfg->n_heads);
    if (dh != 32 && dh != 64 && dh != 128) return fail(TIO_ERR_INVALID_ARG, "head dimension must be 32, 64 or 128");
    if (((int64_t)cfg->batch * cfg->seq_len) % 8) return fail(TIO_ERR_INVALID_ARG, "batch * seq_len must be a multiple of 8");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(TIO_ERR_HIP, "no HIP device");
    tio_ctx *c = new tio_ctx();
    c->cfg = *cfg; c->rt = *rt;
    c->prog = build_program(*cfg);
    c->trace = trace_from_program(c->prog);
    c->life = analyze(c->trace);
    c->sc = (hipStream_t)rt->compute_stream; c->sd = (hipStream_t)rt->d2h_stream; c->sh = (hipStream_t)rt->h2d_stream;
    c->arena = (uint8_t *)rt->arena; c->host = (uint8_t *)rt->host_pool;
    c->arena_usable = (rt->arena_bytes - kReservedTail) / 256 * 256;
    c->bw = rt->slow_tier_bw;
    c->pool_dev = rt->pool_on_device != 0;
    c->host1 = (uint8_t *)rt->host_tier_pool;
    c->sd1 = (hipStream_t)rt->host_tier_d2h_stream; c->sh1 = (hipStream_t)rt->host_tier_h2d_stream;
    c->bw1 = rt->host_tier_bw;
    if (c->host1 && ((uintptr_t)c->host1 & 255)) { delete c; return fail(TIO_ERR_INVALID_ARG, "host-memory tier pool must be 256-byte aligned"); }
    uint64_t h = 0;
    c->home.assign(c->prog.n_persistent, 0);
    for (int t = 0; t < c->prog.n_persistent; ++t) { c->home[t] = h; h += c->prog.tensors[t].bytes; }
    c->home_bytes = h;
    if (file_tier) {                                     // every range of the file starts on a direct-I/O boundary
        uint64_t f = 0;
        c->home_file.assign(c->prog.n_persistent, 0);
        for (int t = 0; t < c->prog.n_persistent; ++t) {
            c->home_file[t] = f;
            f += (c->prog.tensors[t].bytes + FileTier::kAlign - 1) / FileTier::kAlign * FileTier::kAlign;
        }
        c->home_file_bytes = h = f;
    }
    if (h > rt->host_bytes) { delete c; return fail(TIO_ERR_OOM_HOST, "slow-tier pool smaller than the persistent tensors"); }
    c->loaded.assign(c->prog.params.size(), 0);
    c->reloaded.assign(c->prog.params.size(), 0);
    if (hipHostMalloc((void **)&c->loss_pinned, 4096, hipHostMallocDefault) != hipSuccess) { delete c; return fail(TIO_ERR_HIP, "hipHostMalloc failed"); }
    if (file_tier) {
        try {
            c->ft.reset(new FileTier(rt->slow_tier_file, rt->staging, rt->staging_bytes, rt->file_chunk_bytes, c->sd, c->sh, rt->file_buffered_io != 0));
            c->ft->resize(c->home_file_bytes);
        } catch (...) { tio_ctx_destroy(c); throw; }
    } else {
        try { c->pp0.reset(new PacedPool(c->sd, c->sh, c->bw, c->pool_dev)); } catch (...) { tio_ctx_destroy(c); throw; }
    }
    if (c->host1 && c->sd1 && c->sh1) {
        try { c->pp1.reset(new PacedPool(c->sd1, c->sh1, c->bw1)); } catch (...) { tio_ctx_destroy(c); throw; }
    }
    if (rt->poison_freed)
        for (MigrationEngine *e : {(MigrationEngine *)c->ft.get(), (MigrationEngine *)c->pp0.get(), (MigrationEngine *)c->pp1.get()})
            if (e) e->set_poison(poison_range);
    *out = c;
    return TIO_OK;
    TIO_RT_END
}

int tio_ctx_destroy(tio_ctx *c) {
    if (!c) return TIO_OK;
    try { sync_all(c); } catch (...) {}
    (void)hipStreamSynchronize(c->sc); (void)hipStreamSynchronize(c->sd); (void)hipStreamSynchronize(c->sh);
    c->ft.reset();                                       // joins the engines' threads before their events go
    c->pp0.reset();
    c->pp1.reset();
    destroy_events(c->ev_req);
    destroy_events(c->ev_kernel); destroy_events(c->ev_off); destroy_events(c->ev_pre);
    destroy_events(c->ev_t0); destroy_events(c->ev_t1);
    destroy_events(c->ev_c0); destroy_events(c->ev_c1);
    if (c->ev_step0) (void)hipEventDestroy(c->ev_step0);
    if (c->loss_pinned) (void)hipHostFree(c->loss_pinned);
    delete c;
    return TIO_OK;
}

int tio_params_load(tio_ctx *c, int32_t index, const float *v, int64_t numel) {
    if (!c || !v) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_RT_BEGIN
    if (index < 0 || index >= (int)c->prog.params.size()) return fail(TIO_ERR_INVALID_ARG, "parameter index out of range");
    const ParamInfo &p = c->prog.params[index];
    if (numel != p.rows * p.cols) return fail(TIO_ERR_INVALID_ARG, "element count differs from the parameter's shape");
    if (!c->params_dirty) {            // keep the other parameters' latest values, then treat the arena as empty
        gather_to_home(c);
        c->params_dirty = true;
        c->installed = false;
    }
    const bool bf = c->cfg.precision == TIO_PREC_BF16;
    const bool staged = c->pool_dev || c->ft;
    uint8_t *hw = staged ? nullptr : c->host + c->home[p.w], *hm = staged ? nullptr : c->host + c->home[p.m];
    uint8_t *hv = staged ? nullptr : c->host + c->home[p.v];
    uint8_t *hms = bf && !staged ? c->host + c->home[p.master] : nullptr;
    std::vector<uint8_t> stage;
    if (staged) {                                        // the CPU cannot write the pool: convert into a host buffer first
        const size_t wb = (size_t)numel * (bf ? 2 : 4);
        stage.resize(wb + (bf ? (size_t)numel * 4 : 0));
        hw = stage.data();
        hms = bf ? stage.data() + wb : nullptr;
        hm = hv = nullptr;
    }
    auto fill = [=](int64_t i0, int64_t i1) {
        if (bf) {
            uint16_t *w = (uint16_t *)hw;
            float *ms = (float *)hms;
            for (int64_t i = i0; i < i1; ++i) { w[i] = host_f32_to_bf16(v[i]); ms[i] = host_bf16_to_f32(w[i]); }
        } else {
            std::memcpy(hw + i0 * 4, v + i0, (size_t)(i1 - i0) * 4);
        }
        if (hm) {
            std::memset(hm + i0 * 4, 0, (size_t)(i1 - i0) * 4);
            std::memset(hv + i0 * 4, 0, (size_t)(i1 - i0) * 4);
        }
    };
    const int nthr = numel >= (1 << 22) ? 8 : 1;          // large tensors: split the conversion over host threads
    if (nthr == 1) fill(0, numel);
    else {
        std::vector<std::thread> th;
        const int64_t per = (numel + nthr - 1) / nthr;
        for (int t = 0; t < nthr; ++t) th.emplace_back(fill, t * per, std::min(numel, (t + 1) * per));
        for (auto &x : th) x.join();
    }
    if (c->ft) {
        home_from_host(c, p.w, hw, (uint64_t)numel * (bf ? 2 : 4));
        if (bf) home_from_host(c, p.master, hms, (uint64_t)numel * 4);
        c->ft->zero(c->home_file[p.m], (uint64_t)numel * 4);
        c->ft->zero(c->home_file[p.v], (uint64_t)numel * 4);
    } else if (c->pool_dev) {
        HIPCHK(hipMemcpy(c->host + c->home[p.w], hw, (size_t)numel * (bf ? 2 : 4), hipMemcpyHostToDevice));
        if (bf) HIPCHK(hipMemcpy(c->host + c->home[p.master], hms, (size_t)numel * 4, hipMemcpyHostToDevice));
        HIPCHK(hipMemset(c->host + c->home[p.m], 0, (size_t)numel * 4));
        HIPCHK(hipMemset(c->host + c->home[p.v], 0, (size_t)numel * 4));
        HIPCHK(hipDeviceSynchronize());
    }
    c->loaded[index] = 1;
    // the step counter (AdamW's bias correction) restarts once every parameter has been loaded anew; reloading some of
    // them leaves it, and the moments of the others, as they are
    if (!c->reloaded[index]) { c->reloaded[index] = 1; ++c->n_reloaded; }
    if (c->n_reloaded == c->reloaded.size()) {
        c->step = 0;
        c->reloaded.assign(c->reloaded.size(), 0);
        c->n_reloaded = 0;
    }
    return TIO_OK;
    TIO_RT_END
}

int tio_params_read(tio_ctx *c, int32_t index, int32_t which, float *dst, int64_t numel) {
    if (!c || !dst) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_RT_BEGIN
    if (index < 0 || index >= (int)c->prog.params.size()) return fail(TIO_ERR_INVALID_ARG, "parameter index out of range");
    const ParamInfo &p = c->prog.params[index];
    if (numel != p.rows * p.cols) return fail(TIO_ERR_INVALID_ARG, "element count differs from the parameter's shape");
    const int t = which == 0 ? p.w : which == 1 ? p.master : which == 2 ? p.m : which == 3 ? p.v : -1;
    if (t < 0) return fail(TIO_ERR_INVALID_ARG, "no such state tensor for this precision");
    sync_all(c);
    const bool half = which == 0 && c->cfg.precision == TIO_PREC_BF16;
    const uint64_t nbytes = (uint64_t)numel * (half ? 2 : 4);
    std::vector<uint8_t> tmp(nbytes);
    if (c->installed && !c->params_dirty && c->on_dev[t]) HIPCHK(hipMemcpy(tmp.data(), c->arena + c->dev_addr[t], nbytes, hipMemcpyDeviceToHost));
    else if (c->installed && !c->params_dirty && c->in_host1[t]) std::memcpy(tmp.data(), c->host1 + c->host1_off[t], nbytes);
    else home_to_host(c, t, tmp.data(), nbytes);
    if (half) for (int64_t i = 0; i < numel; ++i) dst[i] = host_bf16_to_f32(((uint16_t *)tmp.data())[i]);
    else std::memcpy(dst, tmp.data(), nbytes);
    return TIO_OK;
    TIO_RT_END
}

int tio_grads_read(tio_ctx *c, int32_t index, float *dst, int64_t numel) {
    if (!c || !dst) return fail(TIO_ERR_INVALID_ARG, "null argument");
    if (index < 0 || index >= (int)c->grads.size() || (int64_t)c->grads[index].size() != numel)
        return fail(TIO_ERR_INVALID_ARG, "no captured gradient of that size (run a step with capture_grads)");
    std::memcpy(dst, c->grads[index].data(), numel * 4);
    return TIO_OK;
}

int tio_file_tier_info(tio_ctx *c, tio_file_tier_stats *out) {
    if (!c || !out) return fail(TIO_ERR_INVALID_ARG, "null argument");
    if (!c->ft) return fail(TIO_ERR_INVALID_ARG, "the context has no file tier");
    TIO_RT_BEGIN
    sync_all(c);
    out->direct_io = c->ft->direct() ? 1 : 0;
    out->file_bytes = c->ft->file_bytes();
    out->bytes_written = c->ft->bytes_written();
    out->bytes_read = c->ft->bytes_read();
    return TIO_OK;
    TIO_RT_END
}

int tio_set_slow_tier_bw(tio_ctx *c, uint64_t bw) {
    if (!c) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_RT_BEGIN
    sync_all(c);                                         // the change may move the tier between plain copies and its paced engine
    c->bw = bw;
    if (c->pp0) c->pp0->set_bandwidth(bw);
    return TIO_OK;
    TIO_RT_END
}

int tio_engine_choose(const uint8_t *ready, const uint8_t *urgent, int32_t n, int32_t urgent_first, int32_t ready_queue) {
    if (n < 0 || (n > 0 && (!ready || !urgent))) return fail(TIO_ERR_INVALID_ARG, "null argument");
    return PacedPool::choose(std::vector<uint8_t>(ready, ready + n), std::vector<uint8_t>(urgent, urgent + n), urgent_first != 0,
                             ready_queue != 0);
}

int tio_set_engine_policy(tio_ctx *c, uint64_t chunk_bytes, int32_t urgent_first, int32_t ready_queue) {
    if (!c) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_RT_BEGIN
    sync_all(c);
    if (c->pp0) c->pp0->set_policy(chunk_bytes, urgent_first != 0, ready_queue != 0);
    if (c->pp1) c->pp1->set_policy(chunk_bytes, urgent_first != 0, ready_queue != 0);
    return TIO_OK;
    TIO_RT_END
}

int tio_train_step(tio_ctx *c, const int32_t *tokens, const int32_t *labels, const tio_plan *plan, int32_t flags,
                   tio_step_stats *out) {
    if (!c || !tokens || !labels) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_RT_BEGIN
    for (size_t i = 0; i < c->loaded.size(); ++i)
        if (!c->loaded[i]) return fail(TIO_ERR_INVALID_ARG, "parameter " + c->prog.params[i].name + " was never loaded");
    step_preconditions(c, tokens, labels);
    ensure_plan(c, plan);
    c->timeline = (flags & TIO_STEP_TIMELINE) != 0;
    run_step(c, tokens, labels, (flags & TIO_STEP_CAPTURE_GRADS) != 0,
             (flags & (TIO_STEP_TIME_KERNELS | TIO_STEP_TIMELINE)) ? &c->last_times : nullptr, out);
    c->timeline = false;
    return TIO_OK;
    TIO_RT_END
}

int tio_kernel_times(tio_ctx *c, int64_t *out_ns, int32_t n) {
    if (!c || !out_ns) return fail(TIO_ERR_INVALID_ARG, "null argument");
    if (n != (int32_t)c->last_times.size()) return fail(TIO_ERR_INVALID_ARG, "no timed step, or wrong kernel count");
    std::memcpy(out_ns, c->last_times.data(), (size_t)n * 8);
    return TIO_OK;
}

int tio_profile_iteration(tio_ctx *c, const int32_t *tokens, const int32_t *labels, int mode, tio_trace **out) {
    if (!c || !out) return fail(TIO_ERR_INVALID_ARG, "null argument");
    TIO_RT_BEGIN
    tio_trace *h = new tio_trace{c->trace};
    if (mode == TIO_PROFILE_MEASURED || mode == TIO_PROFILE_OFFLOADED) {
        if (!tokens || !labels) { delete h; return fail(TIO_ERR_INVALID_ARG, "null argument"); }
        for (size_t i = 0; i < c->loaded.size(); ++i)
            if (!c->loaded[i]) { delete h; return fail(TIO_ERR_INVALID_ARG, "parameter " + c->prog.params[i].name + " was never loaded"); }
        try {
            step_preconditions(c, tokens, labels);
            tio_plan under_cap;
            if (mode == TIO_PROFILE_OFFLOADED) {
                // the iteration does not fit the arena: run it under a plan made from the modelled times
                const tio_plan_opts o{1, 24, 0, 0, 0, 0};
                under_cap.p = build_plan(c->trace, c->life, c->arena_usable, c->bw, o);
                static uint64_t serial = (uint64_t)1 << 62;      // apart from the serials of plans built by callers
                under_cap.p.serial = serial++;
                ensure_plan(c, &under_cap);
            } else
            ensure_plan(c, nullptr);
            const int N = c->trace.n_kernels;
            std::vector<std::vector<int64_t>> runs(3);
            run_step(c, tokens, labels, false, nullptr, nullptr);          // warm-up
            for (auto &r : runs) run_step(c, tokens, labels, false, &r, nullptr);
            for (int k = 0; k < N; ++k) {
                int64_t a = runs[0][k], b = runs[1][k], d = runs[2][k];
                h->t.tau[k] = std::max(std::min(a, b), std::min(std::max(a, b), d));   // median of three
            }
        } catch (...) { delete h; throw; }
    }
    *out = h;
    return TIO_OK;
    TIO_RT_END
}

int tio_op_gemm(void *stream, int32_t dtype, int32_t a_km, int32_t b_km, int64_t M, int64_t N, int64_t K, const void *A,
                int64_t lda, const void *B, int64_t ldb, const void *bias, const void *resid, int64_t ldr, void *C, int64_t ldc,
                void *rowsum, void *workspace, int32_t splits) {
    TIO_RT_BEGIN
    if (!A || !B || !C) return fail(TIO_ERR_INVALID_ARG, "null argument");
    const int64_t al = dtype == TIO_PREC_BF16 ? 8 : 4;
    if (lda % al || ldb % al || ldc % 4 || (resid && ldr % 4)) return fail(TIO_ERR_INVALID_ARG, "leading dimensions must be multiples of 8 elements");
    if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C | (uintptr_t)bias | (uintptr_t)resid) & 15) return fail(TIO_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    const int64_t ka = (K + al - 1) / al * al, ma = (M + al - 1) / al * al, na = (N + al - 1) / al * al;
    if (splits < 1 || splits > 64 || (splits > 1 && (!workspace || ((uintptr_t)workspace & 15))))
        return fail(TIO_ERR_INVALID_ARG, "splits > 1 needs a 16-byte aligned fp32 workspace of splits*(M*N+M) floats");
    if ((a_km ? lda < ma : lda < ka) || (b_km ? ldb < na : ldb < ka) || ldc < N)
        return fail(TIO_ERR_INVALID_ARG, "leading dimension smaller than the (8-element padded) extent");
    k::gemm((hipStream_t)stream, dtype, a_km != 0, b_km != 0, M, N, K, A, lda, B, ldb, bias, resid, ldr, C, ldc, rowsum, workspace, splits);
    HIPCHK(hipGetLastError());
    return TIO_OK;
    TIO_RT_END
}

// ---- split-contraction product for callers that cannot allocate ------------------------------------------------
// The fp32 partial tiles go to a fixed array in device memory instead of a workspace from the caller.  In host
// code the array's name is only a handle for hipGetSymbolAddress: every device has its own copy at its own address,
// looked up once per device (with that device current) and kept.
namespace {
constexpr uint64_t kStaticWsBytes = (uint64_t)64 << 20;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];
namespace {
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device
void *static_workspace() {
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) throw PlanError{TIO_ERR_HIP, "device ordinal beyond the table of static workspaces"};
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) throw PlanError{TIO_ERR_HIP, "hipGetSymbolAddress returned no address for the static workspace"};
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int tio_op_gemm_static_ws(void *stream, int32_t dtype, int32_t a_km, int32_t b_km, int64_t M, int64_t N, int64_t K,
                                     const void *A, int64_t lda, const void *B, int64_t ldb, void *C, int64_t ldc, void *rowsum,
                                     int32_t splits) {
    TIO_RT_BEGIN
    if (M < 1 || N < 1 || K < 1) return fail(TIO_ERR_INVALID_ARG, "non-positive dimension");
    if (splits < 1 || splits > 64) return fail(TIO_ERR_INVALID_ARG, "splits must be in 1..64");
    // the same layout tio_op_gemm asks of its workspace: splits * (M*N + M) floats
    const unsigned __int128 need = (unsigned __int128)splits * ((unsigned __int128)M * N + M) * 4;
    if (splits > 1 && need > kStaticWsBytes)
        return fail(TIO_ERR_INVALID_ARG, "splits*(M*N+M) floats exceed the static workspace of " + std::to_string(kStaticWsBytes) +
                                             " bytes: use tio_op_gemm with a workspace of the caller's");
    void *ws = splits > 1 ? static_workspace() : nullptr;
    return tio_op_gemm(stream, dtype, a_km, b_km, M, N, K, A, lda, B, ldb, nullptr, nullptr, 0, C, ldc, rowsum, ws, splits);
    TIO_RT_END
}

int tio_step_timeline(tio_ctx *c, int64_t *k0, int64_t *k1, int32_t n_kernels, int64_t *c0, int64_t *c1, int32_t n_entries) {
    if (!c || !k0 || !k1 || (n_entries > 0 && (!c0 || !c1))) return fail(TIO_ERR_INVALID_ARG, "null argument");
    if (n_kernels != (int32_t)c->tl_k0.size() || n_entries != (int32_t)c->tl_c0.size())
        return fail(TIO_ERR_INVALID_ARG, "no step was run in timeline mode, or the counts differ");
    std::memcpy(k0, c->tl_k0.data(), (size_t)n_kernels * 8); std::memcpy(k1, c->tl_k1.data(), (size_t)n_kernels * 8);
    if (n_entries) { std::memcpy(c0, c->tl_c0.data(), (size_t)n_entries * 8); std::memcpy(c1, c->tl_c1.data(), (size_t)n_entries * 8); }
    return TIO_OK;
}

int tio_op_attention(void *stream, int32_t dtype, int64_t B, int64_t T, int64_t H, int64_t dh, const void *qkv, void *o,
                     float *lse, const void *dO, float *delta, void *dqkv) {
    TIO_RT_BEGIN
    if (!qkv || !o || !lse) return fail(TIO_ERR_INVALID_ARG, "null argument");
    if (dh != 32 && dh != 64 && dh != 128) return fail(TIO_ERR_INVALID_ARG, "head dimension must be 32, 64 or 128");
    if (B < 1 || T < 1 || H < 1) return fail(TIO_ERR_INVALID_ARG, "non-positive dimension");
    if (((uintptr_t)qkv | (uintptr_t)o | (uintptr_t)dO | (uintptr_t)dqkv) & 15) return fail(TIO_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    k::attn_fwd(s, dtype, qkv, o, lse, B, T, H, dh);
    if (dO) {
        if (!delta || !dqkv) return fail(TIO_ERR_INVALID_ARG, "backward needs delta and dqkv");
        k::attn_bwd_pre(s, dtype, dO, o, delta, B, T, H, dh);
        k::attn_bwd(s, dtype, dO, qkv, lse, delta, dqkv, B, T, H, dh);
    }
    HIPCHK(hipGetLastError());
    return TIO_OK;
    TIO_RT_END
}

int tio_op_bench(tio_ctx *c, int32_t kernel_index, int32_t reps, double *out_avg_ns) {
    if (!c || !out_avg_ns || reps < 1) return fail(TIO_ERR_INVALID_ARG, "bad argument");
    TIO_RT_BEGIN
    if (kernel_index < 0 || kernel_index >= c->trace.n_kernels) return fail(TIO_ERR_INVALID_ARG, "kernel index out of range");
    ensure_plan(c, nullptr);
    hipEvent_t e0, e1;
    HIPCHK(hipEventCreate(&e0)); HIPCHK(hipEventCreate(&e1));
    launch(c, kernel_index);                                  // warm-up
    HIPCHK(hipEventRecord(e0, c->sc));
    for (int i = 0; i < reps; ++i) launch(c, kernel_index);
    HIPCHK(hipEventRecord(e1, c->sc));
    HIPCHK(hipEventSynchronize(e1));
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    *out_avg_ns = (double)ms * 1e6 / reps;
    return TIO_OK;
    TIO_RT_END
}

}  // extern "C"
