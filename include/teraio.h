/*
 * teraio.h -- C ABI of the MI355X-native lifetime-aware tensor offloading library.
 *
 * The calls follow the pipeline of the paper (arXiv 2506.06472, Section 3, system overview):
 *   profile one iteration -> tensor access trace and kernel times   (Section 3.1, tracking tensors)
 *   analyse lifetimes     -> inactive periods and memory demand M   (Section 3.1, analysing activity)
 *   build a plan          -> offload / prefetch entries              (Section 3.2, Algorithm 1)
 *   run training steps under the plan                               (Section 3.3, migration engine)
 *
 * Conventions
 *   - every function returns 0 on success or a negative tio_status; out-parameters are written
 *     only on success; tio_last_error() gives a thread-local message for the last failure.
 *   - handles (tio_ctx, tio_trace, tio_lifetimes, tio_plan) are owned by the library and released
 *     by their _free / _destroy call; pointers inside a *_view stay valid until then.
 *   - "host" pointers are ordinary host memory borrowed for the duration of the call;
 *     "device" pointers are GPU memory owned by the caller for the lifetime of the context.
 *   - no exceptions cross this boundary; nothing here allocates GPU memory: the caller hands
 *     over the arena (GPU) and the slow-tier pool (pinned host) when the context is created.
 */
#ifndef TERAIO_H
#define TERAIO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tio_status {
    TIO_OK = 0,
    TIO_ERR_INVALID_ARG = -1,
    TIO_ERR_OOM_HOST = -2,            /* slow-tier pool too small */
    TIO_ERR_ACTIVE_SET_EXCEEDS_CAP = -3, /* one kernel's operands alone exceed the capacity */
    TIO_ERR_PLAN_INVALID = -4,
    TIO_ERR_PLAN_STALE = -5,          /* plan was built from a different trace */
    TIO_ERR_HIP = -6,
    TIO_ERR_ARENA_TOO_SMALL = -7,     /* address assignment does not fit the arena */
    TIO_ERR_NO_GPU_CODE = -8,
    TIO_ERR_IO = -9                   /* the slow-tier file could not be opened, grown, read or written */
} tio_status;

enum { TIO_ARCH_GPT = 0, TIO_ARCH_LLAMA = 1 };
enum { TIO_PREC_FP32 = 0, TIO_PREC_BF16 = 1 };
enum { TIO_PROFILE_MEASURED = 0, TIO_PROFILE_MODELLED = 1, TIO_PROFILE_OFFLOADED = 2 };
enum { TIO_OFFLOAD = 0, TIO_PREFETCH = 1 };

/* Model and optimizer shape.  GPT: LayerNorm, GELU (tanh form), biases, learned positions.
 * Llama: RMSNorm, RoPE on adjacent pairs, SwiGLU, no biases.  The LM head is untied. */
typedef struct tio_model_cfg {
    int32_t arch, n_layers, d_model, n_heads, d_ff, vocab, seq_len, batch;
    int32_t precision;               /* TIO_PREC_* : element type of weights, activations, gradients */
    float lr, beta1, beta2, adam_eps, weight_decay, norm_eps, rope_theta;
    int32_t micro_batches;           /* 0 or 1: the whole batch in one pass; n > 1: the batch (a multiple of n) is run as
                                        n groups of batch/n sequences with gradient accumulation, one AdamW update per step
                                        (the paper trains with micro-batches, Sections 4.1 and 4.2) */
} tio_model_cfg;

typedef struct tio_runtime_cfg {
    void *arena;                     /* device, 256-byte aligned; every tensor lives here */
    uint64_t arena_bytes;
    void *host_pool;                 /* slow tier, stands in for the paper's SSD tier: pinned host memory, or
                                        (pool_on_device) a second device buffer outside the capped arena */
    uint64_t host_bytes;
    void *compute_stream, *d2h_stream, *h2d_stream; /* hipStream_t, default priority; d2h may equal h2d */
    uint64_t slow_tier_bw;           /* emulated bandwidth of the slow tier, bytes/s per direction (one shared channel when
                                        d2h_stream == h2d_stream): a transfer counts as complete bytes/bandwidth after the
                                        later of "its dependencies are met" and "the channel is free"; 0 = unthrottled */
    int32_t poison_freed;            /* debug: every arena range vacated by an offload is overwritten with NaN
                                        patterns once its copy has left, so a kernel that read it would show */
    int32_t pool_on_device;          /* 1: host_pool is device memory (hosts that cannot pin enough memory) */
    /* Optional second destination (plans built with a host-memory tier, tio_plan_opts.host_bw / host_budget):
     * pinned host memory with its own two copy streams.  All NULL / 0 when no such plan will be run. */
    void *host_tier_pool;            /* pinned host memory, 256-byte aligned */
    uint64_t host_tier_bytes;
    void *host_tier_d2h_stream, *host_tier_h2d_stream;   /* hipStream_t, default priority */
    uint64_t host_tier_bw;           /* emulated bandwidth of that tier, bytes/s per direction; 0 = unthrottled */
    /* Optional: the slow tier is a file (the paper's storage tier, Section 3.3) instead of a memory pool.  Then
     * host_pool is NULL, pool_on_device 0, and host_bytes is the largest size the file may grow to.  The file is
     * created if missing, opened for direct I/O where the file system supports it, grown as plans need and never
     * deleted by the library.  Transfers go through `staging` in chunks (there is no direct storage-to-GPU path on
     * this platform); slow_tier_bw is ignored for this tier: the file system sets the pace. */
    const char *slow_tier_file;      /* host, NUL-terminated path, read only during tio_ctx_create; NULL = no file tier */
    void *staging;                   /* pinned host memory, 4096-byte aligned, owned by the caller for the context's lifetime */
    uint64_t staging_bytes;          /* at least 4 chunks (two per direction) */
    uint64_t file_chunk_bytes;       /* multiple of 4096; 0 = 8 MiB */
    int32_t file_buffered_io;        /* 1: go through the page cache even where direct I/O is available */
} tio_runtime_cfg;

typedef struct tio_ctx tio_ctx;
typedef struct tio_trace tio_trace;
typedef struct tio_lifetimes tio_lifetimes;
typedef struct tio_plan tio_plan;

/* ---- flat read-only views for element-by-element comparison ------------------------------- */
typedef struct tio_trace_view {
    int32_t n_kernels, n_tensors, n_persistent, n_operands;
    const int32_t *op;               /* [n_kernels] operator code */
    const int32_t *operand_off;      /* [n_kernels+1] into the two arrays below */
    const int32_t *operand_tensor;   /* sorted by tensor id within a kernel */
    const int32_t *operand_flags;    /* bit0 read, bit1 written */
    const int64_t *flops;            /* [n_kernels] */
    const int64_t *tau_ns;           /* [n_kernels] kernel times used for planning */
    const uint64_t *tensor_bytes;    /* [n_tensors] payload rounded up to 256 */
    const int32_t *tensor_kind;      /* [n_tensors] 0 weight 1 master 2 m 3 v 4 input 5 activation 6 gradient 7 parameter gradient */
} tio_trace_view;

typedef struct tio_lifetimes_view {
    int32_t n_kernels, n_periods;
    const uint64_t *M;               /* [n_kernels] bytes live at each kernel (Algorithm 1, input M) */
    const int32_t *tensor;           /* [n_periods] the set I: (t, s, start, end) */
    const uint64_t *bytes;
    const int32_t *start, *end;      /* bounding active kernels; end >= n_kernels wraps into the next iteration */
} tio_lifetimes_view;

typedef struct tio_plan_entry {
    int32_t tensor, kind;            /* TIO_OFFLOAD / TIO_PREFETCH */
    int32_t trigger, deadline;       /* unrolled kernel indices, see tio_build_plan */
    int32_t urgent, pair;
} tio_plan_entry;

typedef struct tio_alloc {
    int32_t tensor;
    int32_t first_kernel, last_kernel; /* residency interval, unrolled (last may be >= n_kernels) */
    uint64_t address;                /* byte offset in the arena */
} tio_alloc;

typedef struct tio_plan_view {
    int32_t n_kernels, n_entries, n_greedy, n_forced, n_allocs, reserved;
    const tio_plan_entry *entries;   /* issue order */
    const uint64_t *Mp;              /* [n_kernels] planned residency M' */
    const tio_alloc *allocs;
    uint64_t cap_bytes;              /* capacity asked for */
    uint64_t planning_cap_bytes;     /* capacity Algorithm 1 was run with (<= cap_bytes, lowered until the layout fits) */
    uint64_t arena_bytes_needed;     /* highest address used + size */
    uint64_t host_bytes_needed;
    uint64_t bytes_per_direction;    /* sum of sizes of migrated periods */
    /* host-memory tier (all zero / tier 0 everywhere when the plan was built without one) */
    int32_t n_pairs, reserved2;
    const int32_t *pair_tier;        /* [n_pairs] destination of each selected period (entry.pair): 0 slow tier, 1 host tier */
    uint64_t host_tier_bytes_needed; /* pool size of the host-memory tier (slots are reused over time) */
    uint64_t host_tier_peak_bytes;   /* most bytes the planner counts in host memory at any kernel (<= the budget) */
    uint64_t host_tier_bw;
    int32_t retime_pass, reserved3;  /* run of the re-timing loop whose plan this is (0: the first, on the kernel times) */
} tio_plan_view;

typedef struct tio_plan_opts {
    int32_t duplex;                  /* 1: offload and prefetch channels are independent (default); 0: one channel */
    int32_t layout_retries;          /* how many times the planning capacity may be lowered (default 24) */
    uint64_t min_bytes;              /* periods of smaller tensors are candidates of last resort only (default 0) */
    uint64_t arena_bytes;            /* arena the layout must fit; 0 = cap_bytes */
    /* Destination choice (Section 3.2, "Decide offloading destination"): a second, faster tier in host memory
     * with its own two channels.  The slow tier stays the preferred destination; a period goes to the host tier
     * when the transfers already planned on the slow tier displace it (the slow tier is saturated for it), the
     * host tier gives the larger benefit, and the bytes held in host memory stay within host_budget during its
     * whole inactive period.  Forced (urgent) evictions go to the host tier while the budget has room.
     * host_bw = 0 or host_budget = 0: no host tier (default). */
    uint64_t host_bw;                /* bytes/s per direction of the host-memory tier */
    uint64_t host_budget;            /* most bytes host memory may hold for migrated tensors */
    /* Benefit of a candidate (Section 3.2, "Quantify the benefit and cost").  0 (default): the formula of Algorithm 1,
     * B = s * (sum of tau over the kernels of the absent region that are over capacity).  1: the prose form, in which a
     * kernel counts only with the bytes it is over capacity, B = sum of min(s, M'[k] - capacity) * tau[k].  Candidates
     * are ranked by B / s, compared exactly. */
    int32_t clamp_benefit;
    /* Re-timing (an extension beyond the paper, default 0 = plan once as the paper does).  n > 0: Algorithm 1 and the
     * urgent pass are run 2n more times, each time on a timeline of the iteration as the performance model
     * (tio_plan_simulate) predicts it under the previous run's plan: a kernel takes its own time plus the stall in
     * front of it.  Runs 1..n stretch every kernel that way; runs n+1..2n (a second chain from the same start) only the
     * kernels from the first kernel of largest memory demand on.  Every run's plan is simulated on the true kernel
     * times; the runs are ranked by predicted iteration (the earlier run first among equals, the paper's plan is run 0)
     * and the best one whose address layout fits the arena is kept.  Where the best run's layout does not fit, the
     * search over planning capacities (2 % steps down from the cap) goes on for up to two more steps and keeps the
     * plan predicted fastest among those that fit: a plan whose layout fits at a slightly lower planning capacity
     * can beat, by more than its extra bytes cost, the first one that fits at the full capacity; and the plan built
     * without re-timing for the same arena replaces the result when it is predicted faster, so the result is never
     * predicted slower than that plan.  Helps where
     * migration takes longer than compute: the stalled iteration gives the channels several times the compute time,
     * which the first run cannot see.  tio_plan_view.retime_pass and planning_cap say what was kept. */
    int32_t retime_passes;
} tio_plan_opts;

typedef struct tio_step_stats {
    float loss;
    int32_t step;
    int64_t wall_ns;                 /* host clock, launch of the first kernel to completion of the last */
    int64_t kernel_ns;               /* sum of kernel times (only when measured) */
    uint64_t d2h_bytes, h2d_bytes;
    int64_t d2h_busy_ns, h2d_busy_ns;/* sum over the step's offloads / prefetches of begin-to-end time, pacing
                                        included (only with TIO_STEP_TIMELINE) */
    int32_t n_kernels, n_migrations;
} tio_step_stats;

const char *tio_last_error(void);
const char *tio_version(void);

/* ---- model description (pure CPU) ---------------------------------------------------------- */
/* Parameter list in parameter-list order (embeddings, layer 0..L-1, final norm, head). */
int tio_param_count(const tio_model_cfg *cfg, int32_t *out_n);
int tio_param_info(const tio_model_cfg *cfg, int32_t index, char *name_buf, size_t name_cap,
                   int64_t *out_rows, int64_t *out_cols);

/* ---- Section 3.1: trace and lifetimes (pure CPU unless measured) ------------------------------ */
/* Structural trace of one iteration with modelled kernel times; needs no GPU. */
int tio_trace_build(const tio_model_cfg *cfg, tio_trace **out);
/* Trace from caller-supplied arrays (synthetic traces for planner tests). view is copied. */
int tio_trace_import(const tio_trace_view *view, tio_trace **out);
/* Replaces the kernel times (host array of n_kernels int64 ns). */
int tio_trace_set_tau(tio_trace *trace, const int64_t *tau_ns, int32_t n);
int tio_trace_export(const tio_trace *trace, tio_trace_view *out);
void tio_trace_free(tio_trace *trace);

/* Runs iterations of the real kernels (uncapped layout: the arena must hold the whole
 * iteration), marks every operand of every launch active and times each launch with HIP events;
 * tau = median of three iterations.  tokens/labels: host int32 [batch, seq_len].
 * mode TIO_PROFILE_MODELLED skips the GPU and equals tio_trace_build.
 * mode TIO_PROFILE_OFFLOADED is for iterations that need more memory than the arena has (Section 2 of the
 * paper profiles such models by offloading tensors the current kernel does not need): the library plans
 * from the modelled times with the arena as the capacity and the context's slow-tier bandwidth, runs the
 * same measurement under that plan, and returns the measured times; plan again with them. */
int tio_profile_iteration(tio_ctx *ctx, const int32_t *tokens, const int32_t *labels, int mode,
                          tio_trace **out);

/* Inactive periods and memory demand per kernel. */
int tio_analyze_lifetimes(const tio_trace *trace, tio_lifetimes **out);
int tio_lifetimes_export(const tio_lifetimes *life, tio_lifetimes_view *out);
void tio_lifetimes_free(tio_lifetimes *life);

/* ---- Section 3.2: Algorithm 1 + urgent pass + address assignment (pure CPU) ------------------- */
/* mem_cap_bytes: M_GPU.  slow_tier_bw: bytes/s of each migration channel (0 = unlimited).
 * An entry is issued just before kernel (trigger mod N) is launched, once kernel trigger-1 has
 * completed.  An offload must be complete before kernel `deadline` reuses the memory; a prefetch
 * before kernel `deadline` (the tensor's next use) runs.  The tensor is counted out of GPU memory
 * at kernels [offload.deadline, prefetch.trigger-1].  Returning 0 with forced (urgent) entries
 * is not an error: the engine stalls kernels as the paper describes.  opts may be NULL. */
int tio_build_plan(const tio_trace *trace, const tio_lifetimes *life, uint64_t mem_cap_bytes,
                   uint64_t slow_tier_bw, const tio_plan_opts *opts, tio_plan **out);
int tio_plan_export(const tio_plan *plan, tio_plan_view *out);
/* Structural re-check of a plan against trace and lifetimes: residency of every operand,
 * residency <= cap at every kernel, non-overlapping addresses. */
int tio_plan_validate(const tio_trace *trace, const tio_lifetimes *life, const tio_plan *plan);
/* Performance model of the migration engine for a plan (Section 2.2 of the paper studies throughput against
 * migration bandwidth with such a model): kernel k takes the trace's tau[k]; each direction moves bytes at
 * slow_tier_bw bytes/s (0 = instantly; duplex = 0: one shared channel) in the plan's issue order; an entry is
 * issued when the kernel before its trigger completes; a prefetch also waits for its own offload and for the
 * offloads whose deadline has passed; a kernel starts when its predecessor and the migrations due at it have
 * completed.  `iterations` >= 1 consecutive iterations are simulated; out_step_ns receives the duration of the
 * last one (the steady state), out_compute_ns the sum of tau.  Pure CPU, integer arithmetic. */
int tio_plan_simulate(const tio_trace *trace, const tio_plan *plan, uint64_t slow_tier_bw, int32_t duplex,
                      int32_t iterations, int64_t *out_step_ns, int64_t *out_compute_ns);
/* The same model for the engine as the runtime runs it on tiers with an emulated bandwidth (Section 3.2, "Minimize
 * kernel stalls": urgent migrations go ahead of the other pending ones; Section 3.3): each channel moves one chunk of at
 * most chunk_bytes at a time (0: whole tensors), ceil(bytes * 1e9 / bandwidth) ns per chunk; a request is ready once it
 * has been issued and, for a prefetch, once its own offload and every offload whose deadline had been reached at its
 * issue are complete; a free channel takes the next chunk of the first ready urgent request in issue order, else of the
 * first ready request (urgent_first = 0: ready requests in issue order, no priority); a kernel starts when its
 * predecessor, the prefetches due at it and every offload whose deadline is that kernel or an earlier one are complete. */
int tio_plan_simulate_engine(const tio_trace *trace, const tio_plan *plan, uint64_t slow_tier_bw, int32_t duplex,
                             int32_t iterations, uint64_t chunk_bytes, int32_t urgent_first, int64_t *out_step_ns,
                             int64_t *out_compute_ns);
void tio_plan_free(tio_plan *plan);

/* ---- Section 3.3: runtime ---------------------------------------------------------------------- */
int tio_ctx_create(const tio_model_cfg *cfg, const tio_runtime_cfg *rt, tio_ctx **out);
int tio_ctx_destroy(tio_ctx *ctx);
/* Loads parameter `index` from host fp32 values (rounded to the compute precision; fp32 master
 * copy kept in bf16 mode); its moments are zeroed.  The step counter of the context (AdamW's bias correction) restarts
 * at the call that completes a reload of every parameter; reloading only some of them leaves the counter and the other
 * parameters' moments as they are. */
int tio_params_load(tio_ctx *ctx, int32_t index, const float *host_values, int64_t numel);
/* which: 0 compute weight, 1 master copy (bf16 mode only), 2 first moment, 3 second moment;
 * values are returned as fp32 wherever the tensor currently lives (GPU or slow tier). */
int tio_params_read(tio_ctx *ctx, int32_t index, int32_t which, float *host_dst, int64_t numel);
/* Gradient of parameter `index` as captured during the last step run with TIO_STEP_CAPTURE_GRADS. */
int tio_grads_read(tio_ctx *ctx, int32_t index, float *host_dst, int64_t numel);
/* State of the file-backed slow tier (Section 3.3): whether direct I/O is in use, the current file size, and the
 * payload bytes written to and read from the file by migrations since the context was created (it waits for
 * the transfers in flight).  TIO_ERR_INVALID_ARG if the context has no file tier. */
typedef struct tio_file_tier_stats {
    int32_t direct_io;
    uint64_t file_bytes, bytes_written, bytes_read;
} tio_file_tier_stats;
int tio_file_tier_info(tio_ctx *ctx, tio_file_tier_stats *out);
/* Bandwidth enforced on the copy streams from the next step on (0 = unthrottled). */
int tio_set_slow_tier_bw(tio_ctx *ctx, uint64_t bytes_per_s);

/* How the engine of a tier with an emulated bandwidth serves its requests (Section 3.2, "Minimize kernel stalls": urgent
 * migrations go ahead of the other pending ones).  Default: chunks of 16 MiB, urgent_first = 1, ready_queue = 1: whenever a
 * direction's channel is free it takes the next chunk of the first urgent request whose dependencies are met, else of the
 * first request whose dependencies are met, in the order submitted.  chunk_bytes = 0 moves whole tensors (nothing can
 * overtake a transfer in progress); urgent_first = 0 ignores the mark; ready_queue = 0 serves strictly in the order
 * submitted, waiting for the dependencies of the oldest request.  Waits for the transfers in flight; applies from the
 * next step on.  Tiers without an emulated bandwidth and the file tier serve in the order submitted and ignore this. */
int tio_set_engine_policy(tio_ctx *ctx, uint64_t chunk_bytes, int32_t urgent_first, int32_t ready_queue);

/* Testing aid (pure CPU): the choice a free channel of that engine makes.  ready[i] / urgent[i] (host, n bytes each)
 * describe the queued requests in the order submitted; returns the index served next, -1 if none may go (no error code
 * is negative one: a null array with n > 0 returns TIO_ERR_INVALID_ARG = -1 as well, so pass valid arrays). */
int tio_engine_choose(const uint8_t *ready, const uint8_t *urgent, int32_t n, int32_t urgent_first, int32_t ready_queue);

/* One training iteration: forward, backward, AdamW, with the plan's migrations on the copy
 * streams.  plan == NULL runs the uncapped layout with no migration.  tokens/labels: host int32.
 * flags: TIO_STEP_CAPTURE_GRADS keeps a host copy of every parameter gradient (debug: it
 * synchronises before each optimizer launch); TIO_STEP_TIME_KERNELS brackets every launch with HIP
 * events on the compute stream (see tio_kernel_times); TIO_STEP_TIMELINE additionally stamps every
 * migration (see tio_step_timeline).
 * Blocks until the compute stream has finished the iteration (copies may still be in flight).
 * Errors found before the first launch (null or out-of-vocabulary ids, a parameter never loaded, a plan that is
 * stale, invalid or too large for the arena or the pools) leave the context as it was.  TIO_ERR_HIP or TIO_ERR_IO
 * from inside the iteration leaves tensors half updated: every later step on the context returns TIO_ERR_HIP and
 * the caller destroys it. */
enum { TIO_STEP_CAPTURE_GRADS = 1, TIO_STEP_TIME_KERNELS = 2, TIO_STEP_TIMELINE = 4 };
int tio_train_step(tio_ctx *ctx, const int32_t *tokens, const int32_t *labels,
                   const tio_plan *plan, int32_t flags, tio_step_stats *out);
/* Per-launch durations (ns, HIP events) of the last step run with TIO_STEP_TIME_KERNELS;
 * n must equal the kernel count of the trace. */
int tio_kernel_times(tio_ctx *ctx, int64_t *out_ns, int32_t n);
/* Timeline of the last step run with TIO_STEP_TIMELINE (it synchronises all streams before and
 * after the step): begin and end of every kernel and of every plan entry's copy, in ns from the
 * start of the step (HIP events on the stream the work ran on); -1 for entries not issued. */
int tio_step_timeline(tio_ctx *ctx, int64_t *kernel_begin, int64_t *kernel_end, int32_t n_kernels,
                      int64_t *copy_begin, int64_t *copy_end, int32_t n_entries);

/* ---- single operators on caller-provided device buffers (kernel parity tests, benchmarks) ---- */
/* C[M,N] = A . B^T (+ bias[N]) (+ resid[M,N]); a_kmajor/b_kmajor: operand stored [K, rows]
 * instead of [rows, K].  dtype TIO_PREC_*.  All leading dimensions in elements, multiples of 8
 * and at least the 8-element padded extent; device pointers, 16-byte aligned; stream is a
 * hipStream_t (NULL = default stream).  rowsum (optional, device, [M] elements): receives
 * sum_k A[m][k] from the same launch (the bias gradient when A = dY^T).
 * splits > 1 (bf16, no bias/resid, N multiple of 4) cuts the contraction into `splits` ranges:
 * workspace (device, fp32, splits*(M*N+M) floats) receives the partial tiles and a second launch
 * adds them in range order; splits = 1 ignores workspace. */
int tio_op_gemm(void *stream, int32_t dtype, int32_t a_kmajor, int32_t b_kmajor,
                int64_t M, int64_t N, int64_t K,
                const void *A, int64_t lda, const void *B, int64_t ldb,
                const void *bias, const void *resid, int64_t ldr, void *C, int64_t ldc, void *rowsum,
                void *workspace, int32_t splits);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): tio_op_gemm without bias / residual, whose split-contraction partial tiles go to a
 * fixed 64 MiB (67108864-byte) array in the library's device image instead of a caller workspace.  It allocates
 * nothing; every GPU the library runs on holds its own copy of that array until the process ends.
 * TIO_ERR_INVALID_ARG when splits > 1 and splits*(M*N+M) floats exceed the array, otherwise the arguments,
 * the checks and the result are those of tio_op_gemm (bit for bit: the same kernels run).  Nothing in the array
 * has to start at zero (every partial tile is written before the reduction launch reads it) and its contents
 * after the call are unspecified.  All calls on one GPU share the array: calls whose launches may overlap on
 * that GPU (different streams, different threads) race; serialise them on one stream. */
int tio_op_gemm_static_ws(void *stream, int32_t dtype, int32_t a_kmajor, int32_t b_kmajor,
                          int64_t M, int64_t N, int64_t K,
                          const void *A, int64_t lda, const void *B, int64_t ldb,
                          void *C, int64_t ldc, void *rowsum, int32_t splits);
/* Causal self-attention on a packed qkv buffer [B*T, 3*H*dh] (q | k | v, heads side by side):
 * o [B*T, H*dh] = softmax(q k^T / sqrt(dh)) v per head, lse [B*H*T] fp32 = log-sum-exp of the scaled
 * scores.  With dO != NULL also the backward pass: delta [B*H*T] fp32 (work buffer, receives
 * rowsum(dO * o)) and dqkv [B*T, 3*H*dh].  Device pointers, 16-byte aligned; dh in {32, 64, 128}. */
int tio_op_attention(void *stream, int32_t dtype, int64_t B, int64_t T, int64_t H, int64_t dh,
                     const void *qkv, void *o, float *lse, const void *dO, float *delta, void *dqkv);
/* Measuring aid: launch number kernel_index of the schedule, repeated reps times on the compute stream with the
 * uncapped layout (the arena must hold it) and whatever the arena contains, HIP events around the repetitions;
 * returns average ns per launch.  It overwrites that launch's outputs, and a launch that updates its operands in place
 * (AdamW, gradient accumulation of later micro-batches, RoPE, cross entropy) applies its update reps + 1 times: weights
 * and optimizer state are not what training left.  Not for use between training steps; reload the parameters afterwards. */
int tio_op_bench(tio_ctx *ctx, int32_t kernel_index, int32_t reps, double *out_avg_ns);

#ifdef __cplusplus
}
#endif
#endif /* TERAIO_H */
