// Memory-bound kernels of the training step: embedding, LayerNorm / RMSNorm, GELU, SwiGLU, RoPE,
// fused softmax cross-entropy, bias gradient, AdamW, plus small utilities.  All are bound by HBM:
// 16-byte coalesced accesses, fp32 arithmetic, wavefront (64-lane) reductions, fixed summation
// orders (no floating-point atomics) so that results do not depend on timing or addresses.
#include <stdexcept>

#include <cstdlib>
#include "../../include/teraio.h"
#include "device_common.h"
#include "kernels.h"

namespace tio {
namespace k {

namespace {

constexpr int TPB = 256;
inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

// ---------------------------------------------------------------- embedding
template <typename T>
__global__ void __launch_bounds__(TPB) embed_fwd_k(const int32_t *__restrict__ tok, const T *__restrict__ wte,
                                                   const T *__restrict__ wpe, T *__restrict__ x, int64_t S,
                                                   int64_t d, int64_t Tn) {
    constexpr int V = Vec16<T>::N;
    const int64_t cpr = d / V;
    const int64_t idx = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (idx >= S * cpr) return;
    const int64_t row = idx / cpr, c = idx % cpr;
    Vec16<T> a;
    a.load(wte + (int64_t)tok[row] * d + c * V);
    if (wpe) {
        Vec16<T> p;
        p.load(wpe + (row % Tn) * d + c * V);
        float fa[V], fp[V];
        a.get(fa); p.get(fp);
#pragma unroll
        for (int i = 0; i < V; ++i) fa[i] += fp[i];
        a.set(fa);
    }
    a.store(x + row * d + c * V);
}

// The gradient table is zero-filled by a separate launch; then workgroup s, if position s holds the first
// occurrence of its token id, adds the rows of all occurrences of that id in position order and writes
// the sum: one writer per row, a fixed order, no atomics.  All threads scan the token array together
// (a contiguous range each); the occurrences found are collected in LDS in position order.
template <typename T>
__global__ void __launch_bounds__(TPB) embed_bwd_k(const T *__restrict__ dx, const int32_t *__restrict__ tok,
                                                   T *__restrict__ dw, int64_t S, int64_t d, bool accumulate) {
    constexpr int V = Vec16<T>::N;
    constexpr int CAP = 1024;                              // occurrences handled per round
    __shared__ int cnt[TPB + 1];
    __shared__ int list[CAP];
    const int64_t cpr = d / V;
    const int64_t blk = blockIdx.x;
    const int32_t id = tok[blk];
    const int tid = threadIdx.x;
    const int64_t per = ((S + TPB - 1) / TPB + 3) / 4 * 4;       // a multiple of 4: 16-byte loads of token ids
    const int64_t lo = tid * per, hi = lo + per < S ? lo + per : S;
    int n = 0, earlier = 0;
    {
        int64_t i = lo;
        for (; i + 4 <= hi; i += 4) {
            const int4 t4 = *reinterpret_cast<const int4 *>(tok + i);
            const int hit = (t4.x == id) + (t4.y == id) + (t4.z == id) + (t4.w == id);
            n += hit;
            earlier |= (hit != 0) & ((t4.x == id ? i : t4.y == id ? i + 1 : t4.z == id ? i + 2 : i + 3) < blk);
        }
        for (; i < hi; ++i)
            if (tok[i] == id) { ++n; earlier |= (i < blk); }
    }
    if (__syncthreads_or(earlier)) return;
    cnt[tid] = n;
    __syncthreads();
    if (tid == 0) {                                        // exclusive prefix over the threads' counts
        int run = 0;
        for (int t = 0; t < TPB; ++t) { const int c = cnt[t]; cnt[t] = run; run += c; }
        cnt[TPB] = run;
    }
    __syncthreads();
    const int total = cnt[TPB], first = cnt[tid];
    constexpr int NC = 2;                                  // column chunks a thread owns per pass
    for (int64_t cb0 = 0; cb0 < cpr; cb0 += (int64_t)NC * TPB) {
        float acc[NC][V];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
#pragma unroll
            for (int e = 0; e < V; ++e) acc[c][e] = 0.f;
            const int64_t ch = cb0 + tid + (int64_t)c * TPB;
            if (accumulate && ch < cpr) { Vec16<T> o; o.load(dw + (int64_t)id * d + ch * V); o.get(acc[c]); }   // earlier micro-batches
        }
        for (int base = 0; base < total; base += CAP) {
            if (total > CAP || cb0 == 0) {                 // (re)build the list of this round's occurrences
                __syncthreads();
                int rank = first;
                for (int64_t i = lo; i < hi; ++i)
                    if (tok[i] == id) {
                        if (rank >= base && rank < base + CAP) list[rank - base] = (int)i;
                        ++rank;
                    }
                __syncthreads();
            }
            const int m = total - base < CAP ? total - base : CAP;
            for (int k = 0; k < m; ++k) {
                const int64_t row = list[k];
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int64_t ch = cb0 + tid + (int64_t)c * TPB;
                    if (ch < cpr) {
                        Vec16<T> gvec; gvec.load(dx + row * d + ch * V);
                        float fv[V]; gvec.get(fv);
#pragma unroll
                        for (int e = 0; e < V; ++e) acc[c][e] += fv[e];
                    }
                }
            }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int64_t ch = cb0 + tid + (int64_t)c * TPB;
            if (ch < cpr) { Vec16<T> o; o.set(acc[c]); o.store(dw + (int64_t)id * d + ch * V); }
        }
    }
}

template <typename T>
__global__ void __launch_bounds__(TPB) posemb_bwd_k(const T *__restrict__ dx, T *__restrict__ dw, int64_t B,
                                                    int64_t Tn, int64_t d, bool accumulate) {
    constexpr int V = Vec16<T>::N;
    const int64_t cpr = d / V;
    const int64_t idx = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (idx >= Tn * cpr) return;
    const int64_t t = idx / cpr, c = idx % cpr;
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;
    if (accumulate) { Vec16<T> o; o.load(dw + t * d + c * V); o.get(acc); }      // earlier micro-batches
    for (int64_t b = 0; b < B; ++b) {
        Vec16<T> g;
        g.load(dx + (b * Tn + t) * d + c * V);
        float f[V];
        g.get(f);
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] += f[i];
    }
    Vec16<T> o;
    o.set(acc);
    o.store(dw + t * d + c * V);
}

// ---------------------------------------------------------------- norms
// one wavefront per row; the row is re-read from cache for the second and third pass
template <typename T, bool RMS>
__global__ void __launch_bounds__(TPB) norm_fwd_k(const T *__restrict__ x, const T *__restrict__ g,
                                                  const T *__restrict__ b, T *__restrict__ y,
                                                  float *__restrict__ stats, int64_t S, int64_t d, float eps) {
    constexpr int V = Vec16<T>::N;
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * (TPB / 64) + (threadIdx.x >> 6);
    if (row >= S) return;
    const int64_t cpr = d / V;
    const T *xr = x + row * d;
    float mean = 0.f;
    if (!RMS) {
        float s = 0.f;
        for (int64_t c = lane; c < cpr; c += 64) {
            Vec16<T> v; v.load(xr + c * V);
            float f[V]; v.get(f);
#pragma unroll
            for (int i = 0; i < V; ++i) s += f[i];
        }
        mean = wave_sum(s) / (float)d;
    }
    float q = 0.f;
    for (int64_t c = lane; c < cpr; c += 64) {
        Vec16<T> v; v.load(xr + c * V);
        float f[V]; v.get(f);
#pragma unroll
        for (int i = 0; i < V; ++i) { const float t = f[i] - mean; q += t * t; }
    }
    const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
    if (lane == 0) {
        if (RMS) stats[row] = rstd;
        else { stats[2 * row] = mean; stats[2 * row + 1] = rstd; }
    }
    for (int64_t c = lane; c < cpr; c += 64) {
        Vec16<T> v, gv; v.load(xr + c * V); gv.load(g + c * V);
        float f[V], gf[V], bf[V];
        v.get(f); gv.get(gf);
        if (!RMS) { Vec16<T> bv; bv.load(b + c * V); bv.get(bf); }
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float xh = (f[i] - mean) * rstd;
            f[i] = RMS ? xh * gf[i] : xh * gf[i] + bf[i];
        }
        Vec16<T> o; o.set(f); o.store(y + row * d + c * V);
    }
}

// Same contract as norm_fwd_k, for rows of at most 64*NCH 16-byte chunks: a wavefront owns a row and keeps it in
// registers, so the row is read once and all of its loads are in flight together.
template <typename T, bool RMS, int NCH>
__global__ void __launch_bounds__(TPB) norm_fwd_wave_k(const T *__restrict__ x, const T *__restrict__ g,
                                                       const T *__restrict__ b, T *__restrict__ y,
                                                       float *__restrict__ stats, int64_t S, int64_t d, float eps) {
    constexpr int V = Vec16<T>::N;
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * (TPB / 64) + (threadIdx.x >> 6);
    if (row >= S) return;
    const int cpr = (int)(d / V);
    const T *xr = x + row * d;
    Vec16<T> a[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i)
        if (lane + 64 * i < cpr) a[i].load(xr + (lane + 64 * i) * V);
    const float inv_d = 1.0f / (float)d;
    float mean = 0.f;
    if (!RMS) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < NCH; ++i)
            if (lane + 64 * i < cpr) {
                float f[V]; a[i].get(f);
#pragma unroll
                for (int e = 0; e < V; ++e) s += f[e];
            }
        mean = wave_sum(s) * inv_d;
    }
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i)
        if (lane + 64 * i < cpr) {
            float f[V]; a[i].get(f);
#pragma unroll
            for (int e = 0; e < V; ++e) { const float t = f[e] - mean; q += t * t; }
        }
    const float rstd = 1.0f / sqrtf(wave_sum(q) * inv_d + eps);
    if (lane == 0) {
        if (RMS) stats[row] = rstd;
        else { stats[2 * row] = mean; stats[2 * row + 1] = rstd; }
    }
#pragma unroll
    for (int i = 0; i < NCH; ++i)
        if (lane + 64 * i < cpr) {
            Vec16<T> gv; gv.load(g + (lane + 64 * i) * V);
            float f[V], gf[V], bf[V];
            a[i].get(f); gv.get(gf);
            if (!RMS) { Vec16<T> bv; bv.load(b + (lane + 64 * i) * V); bv.get(bf); }
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float xh = (f[e] - mean) * rstd;
                f[e] = RMS ? xh * gf[e] : xh * gf[e] + bf[e];
            }
            Vec16<T> o; o.set(f); o.store(y + row * d + (lane + 64 * i) * V);
        }
}

// one workgroup per rows_per_blk rows, rows in order; column sums for the gain / bias gradients are
// kept in LDS, each column owned by one thread, and written out as one partial row per workgroup
template <typename T, bool RMS>
__global__ void __launch_bounds__(TPB) norm_bwd_k(const T *__restrict__ dy, const T *__restrict__ x,
                                                  const float *__restrict__ stats, const T *__restrict__ g,
                                                  const T *__restrict__ dres, T *__restrict__ dx,
                                                  float *__restrict__ part, int64_t S, int64_t d, int rows_per_blk) {
    constexpr int V = Vec16<T>::N;
    constexpr int NP = RMS ? 1 : 2;
    extern __shared__ float lds[];          // NP*d accumulators, then 16 floats for reductions
    float *acc = lds;
    float *red = lds + NP * d;
    const int64_t cpr = d / V;
    for (int64_t i = threadIdx.x; i < NP * d; i += TPB) acc[i] = 0.f;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_blk;
    const int64_t r1 = r0 + rows_per_blk < S ? r0 + rows_per_blk : S;
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    for (int64_t row = r0; row < r1; ++row) {
        const float mean = RMS ? 0.f : stats[2 * row];
        const float rstd = RMS ? stats[row] : stats[2 * row + 1];
        float s1 = 0.f, s2 = 0.f;
        for (int64_t c = threadIdx.x; c < cpr; c += TPB) {
            Vec16<T> a, b, gv; a.load(dy + row * d + c * V); b.load(x + row * d + c * V); gv.load(g + c * V);
            float fa[V], fb[V], fg[V]; a.get(fa); b.get(fb); gv.get(fg);
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const float xh = (fb[i] - mean) * rstd, dxh = fa[i] * fg[i];
                s1 += dxh; s2 += dxh * xh;
            }
        }
        s1 = wave_sum(s1); s2 = wave_sum(s2);
        __syncthreads();
        if (l == 0) { red[w] = s1; red[4 + w] = s2; }
        __syncthreads();
        s1 = (red[0] + red[1] + red[2] + red[3]) / (float)d;
        s2 = (red[4] + red[5] + red[6] + red[7]) / (float)d;
        if (RMS) s1 = 0.f;
        for (int64_t c = threadIdx.x; c < cpr; c += TPB) {
            Vec16<T> a, b, gv; a.load(dy + row * d + c * V); b.load(x + row * d + c * V); gv.load(g + c * V);
            float fa[V], fb[V], fg[V], fr[V], out[V]; a.get(fa); b.get(fb); gv.get(fg);
            if (dres) { Vec16<T> r; r.load(dres + row * d + c * V); r.get(fr); }
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const float xh = (fb[i] - mean) * rstd, dxh = fa[i] * fg[i];
                out[i] = rstd * (dxh - s1 - xh * s2) + (dres ? fr[i] : 0.f);
                acc[c * V + i] += fa[i] * xh;
                if (!RMS) acc[d + c * V + i] += fa[i];
            }
            Vec16<T> o; o.set(out); o.store(dx + row * d + c * V);
        }
    }
    __syncthreads();
    float *p = part + (int64_t)blockIdx.x * NP * d;
    for (int64_t i = threadIdx.x; i < NP * d; i += TPB) p[i] = acc[i];
}

// Same contract as norm_bwd_k, for rows of at most 64*NCH 16-byte chunks: a wavefront owns a row and
// keeps it in registers between the statistics pass and the output pass (one read of dy and x, no
// barriers per row); the wavefronts of a workgroup take its rows round-robin, each adds its rows'
// contributions to the gain / bias gradients in registers in row order, and the four register sets
// are then added through LDS in wavefront order.
template <typename T, bool RMS, int NCH>
__global__ void __launch_bounds__(TPB) norm_bwd_wave_k(const T *__restrict__ dy, const T *__restrict__ x,
                                                       const float *__restrict__ stats, const T *__restrict__ g,
                                                       const T *__restrict__ dres, T *__restrict__ dx,
                                                       float *__restrict__ part, int64_t S, int64_t d, int rows_per_blk) {
    constexpr int V = Vec16<T>::N;
    constexpr int NP = RMS ? 1 : 2, NW = TPB / 64;
    extern __shared__ float lds[];          // NP*d accumulators
    const int cpr = (int)(d / V);
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_blk;
    const int64_t r1 = r0 + rows_per_blk < S ? r0 + rows_per_blk : S;
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    constexpr bool KEEP_G = NCH <= 8;       // wider rows re-read the gain (it stays in cache) to save registers
    float cg[NCH][V], cb[RMS ? 1 : NCH][V];
    Vec16<T> gv[KEEP_G ? NCH : 1];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        if (KEEP_G && l + 64 * i < cpr) gv[i].load(g + (l + 64 * i) * V);
#pragma unroll
        for (int e = 0; e < V; ++e) { cg[i][e] = 0.f; if (!RMS) cb[i][e] = 0.f; }
    }
    const float inv_d = 1.0f / (float)d;
    for (int64_t row = r0 + w; row < r1; row += NW) {
        const float mean = RMS ? 0.f : stats[2 * row];
        const float rstd = RMS ? stats[row] : stats[2 * row + 1];
        Vec16<T> a[NCH], b[NCH], rr[NCH];
        float s1 = 0.f, s2 = 0.f;
        // every load of the row goes out before the first use: dy, x and the residual gradient
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            if (l + 64 * i < cpr) {
                a[i].load(dy + row * d + (l + 64 * i) * V);
                b[i].load(x + row * d + (l + 64 * i) * V);
                if (dres) rr[i].load(dres + row * d + (l + 64 * i) * V);
            }
        }
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            if (l + 64 * i < cpr) {
                if (!KEEP_G) gv[0].load(g + (l + 64 * i) * V);
                float fa[V], fb[V], fg[V]; a[i].get(fa); b[i].get(fb); gv[KEEP_G ? i : 0].get(fg);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const float xh = (fb[e] - mean) * rstd, dxh = fa[e] * fg[e];
                    s1 += dxh; s2 += dxh * xh;
                }
            }
        }
        s1 = RMS ? 0.f : wave_sum(s1) * inv_d;
        s2 = wave_sum(s2) * inv_d;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            if (l + 64 * i < cpr) {
                if (!KEEP_G) gv[0].load(g + (l + 64 * i) * V);
                float fa[V], fb[V], fg[V], fr[V], out[V]; a[i].get(fa); b[i].get(fb); gv[KEEP_G ? i : 0].get(fg);
                if (dres) rr[i].get(fr);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const float xh = (fb[e] - mean) * rstd, dxh = fa[e] * fg[e];
                    out[e] = rstd * (dxh - s1 - xh * s2) + (dres ? fr[e] : 0.f);
                    cg[i][e] += fa[e] * xh;
                    if (!RMS) cb[i][e] += fa[e];
                }
                Vec16<T> o; o.set(out); o.store(dx + row * d + (l + 64 * i) * V);
            }
        }
    }
    for (int ww = 0; ww < NW; ++ww) {
        if (w == ww) {
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                if (l + 64 * i < cpr) {
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        const int col = (l + 64 * i) * V + e;
                        lds[col] = (ww ? lds[col] : 0.f) + cg[i][e];
                        if (!RMS) lds[d + col] = (ww ? lds[d + col] : 0.f) + cb[i][e];
                    }
                }
            }
        }
        __syncthreads();
    }
    float *p = part + (int64_t)blockIdx.x * NP * d;
    for (int64_t i = threadIdx.x; i < NP * d; i += TPB) p[i] = lds[i];
}

// Same contract as norm_bwd_k (one partial row of gain / bias gradient sums per workgroup, ROWS rows per workgroup),
// for rows of at most NT*NCH 16-byte chunks; which rows a workgroup takes differs (workgroup w takes rows w, w + G,
// w + 2G, ... of G workgroups, so the grid sweeps every tensor as one contiguous window), so the partial rows hold
// different subsets than norm_bwd_k's and their total is the same sum in another order.  A thread owns the same NCH
// chunks of every row, so a row is read once and the gradient sums of a thread's columns stay in its registers over
// all the rows and go straight to the partial row.  PF rows of dy, x, the residual gradient and the row statistics
// are in flight per workgroup: a row's registers are refilled with the row PF further on as soon as the row is done
// (one barrier per row; the two row sums go through LDS in wavefront order).  All row accesses go through buffer
// descriptors, so chunks past the row's end and rows past the last read zeros and write nothing: there is no branch
// around a memory operation, and the ROWS rows are unrolled into straight-line code, which lets the compiler count
// outstanding loads exactly (at a loop header it waits for all of them).
// What decides this kernel's rate is the number of independent workgroups per compute unit, not the loads in flight
// per workgroup: at d = 4096 in bf16, 8192 rows, on data that is not in any cache, 32 rows per workgroup (one
// workgroup per CU) gives 2.2 TB/s, 16 rows 3.3, 8 rows 4.8, 4 rows 4.7, whatever PF is and however the rows are
// assigned; eight rows per workgroup it is, at the price of a partial row per eight rows.
template <typename T, bool RMS, bool RES, int NCH, int PF, int ROWS, bool CYCLIC = true, int NT = TPB>
__global__ void __launch_bounds__(NT) norm_bwd_block_k(const T *__restrict__ dy, const T *__restrict__ x,
                                                        const float *__restrict__ stats, const T *__restrict__ g,
                                                        const T *__restrict__ dres, T *__restrict__ dx,
                                                        float *__restrict__ part, int64_t S, int64_t d, int rows_per_blk) {
    constexpr int V = Vec16<T>::N;
    constexpr int NP = RMS ? 1 : 2, NW = NT / 64;
    constexpr uint32_t OUTSIDE = 0x40000000u;
    __shared__ float red[2][2][NW];
    const int cpr = (int)(d / V);
    const uint32_t row_bytes = (uint32_t)(d * sizeof(T));
    // a descriptor per row and tensor: rows at or past S have size zero, so they read zeros and write nothing
    const int64_t G = gridDim.x;
    auto row_of = [&](int r) -> int64_t { return CYCLIC ? (int64_t)blockIdx.x + (int64_t)r * G : (int64_t)blockIdx.x * ROWS + r; };
    auto over_row = [&](const T *base, int r) { const int64_t row = row_of(r); return buffer_over(base + (row < S ? row : 0) * d, row < S ? row_bytes : 0u); };
    auto stats_row = [&](int r) { const int64_t row = row_of(r); return buffer_over(stats + (row < S ? row : 0) * NP, row < S ? (uint32_t)(NP * sizeof(float)) : 0u); };
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    uint32_t off[NCH];
    float cg[NCH][V], cb[RMS ? 1 : NCH][V];
    Vec16<T> gv[NCH], a[PF][NCH], b[PF][NCH], rr[RES ? PF : 1][NCH];
    float st_mean[PF], st_rstd[PF];
    auto fetch = [&](int j, int r) {
        const __amdgpu_buffer_rsrc_t rs_st = stats_row(r), rs_dy = over_row(dy, r), rs_x = over_row(x, r);
        if (RMS) { st_mean[j] = 0.f; st_rstd[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_st, 0, 0, 0)); }
        else {
            st_mean[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_st, 0, 0, 0));
            st_rstd[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_st, 4, 0, 0));
        }
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            buffer_load16(a[j][i], rs_dy, off[i]);
            buffer_load16(b[j][i], rs_x, off[i]);
            if (RES) buffer_load16(rr[j][i], over_row(dres, r), off[i]);
        }
    };
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = threadIdx.x + NT * i;
        off[i] = c < cpr ? (uint32_t)c * 16u : OUTSIDE;
        buffer_load16(gv[i], buffer_over(g, row_bytes), off[i]);
#pragma unroll
        for (int e = 0; e < V; ++e) { cg[i][e] = 0.f; if (!RMS) cb[i][e] = 0.f; }
    }
#pragma unroll
    for (int j = 0; j < PF; ++j) fetch(j, j);
    const float inv_d = 1.0f / (float)d;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {                  // rows at or past S (last rows of some workgroups): all zeros, nothing written
        const int j = r % PF, par = r & 1;
        const float mean = st_mean[j], rstd = st_rstd[j];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            float fa[V], fb[V], fg[V]; a[j][i].get(fa); b[j][i].get(fb); gv[i].get(fg);
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float xh = (fb[e] - mean) * rstd, dxh = fa[e] * fg[e];
                s1 += dxh; s2 += dxh * xh;
            }
        }
        s1 = wave_sum(s1); s2 = wave_sum(s2);
        if (l == 0) { red[par][0][w] = s1; red[par][1][w] = s2; }
        __syncthreads();
        s1 = 0.f; s2 = 0.f;
#pragma unroll
        for (int i = 0; i < NW; ++i) { s1 += red[par][0][i]; s2 += red[par][1][i]; }
        s1 = RMS ? 0.f : s1 * inv_d;
        s2 *= inv_d;
        const __amdgpu_buffer_rsrc_t rs_dx = over_row(dx, r);
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            float fa[V], fb[V], fg[V], fr[V], out[V]; a[j][i].get(fa); b[j][i].get(fb); gv[i].get(fg);
            if (RES) rr[j][i].get(fr);
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float xh = (fb[e] - mean) * rstd, dxh = fa[e] * fg[e];
                out[e] = rstd * (dxh - s1 - xh * s2) + (RES ? fr[e] : 0.f);
                cg[i][e] += fa[e] * xh;
                if (!RMS) cb[i][e] += fa[e];
            }
            Vec16<T> o; o.set(out);
            buffer_store16(o, rs_dx, off[i]);
        }
        if (r + PF < ROWS) fetch(j, r + PF);
    }
    float *p = part + (int64_t)blockIdx.x * NP * d;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = threadIdx.x + NT * i;
        if (c < cpr) {
#pragma unroll
            for (int e = 0; e < V; e += 4) {
                *reinterpret_cast<float4 *>(p + (int64_t)c * V + e) = make_float4(cg[i][e], cg[i][e + 1], cg[i][e + 2], cg[i][e + 3]);
                if (!RMS) *reinterpret_cast<float4 *>(p + d + (int64_t)c * V + e) = make_float4(cb[i][e], cb[i][e + 1], cb[i][e + 2], cb[i][e + 3]);
            }
        }
    }
}

// column sums of the per-workgroup partial rows: 32 columns x 8 row groups per workgroup, each
// thread adds its rows in order and the eight groups are combined in order
template <typename T, bool RMS>
__global__ void __launch_bounds__(TPB) norm_bwd_params_k(const float *__restrict__ part, T *__restrict__ dg,
                                                         T *__restrict__ db, int64_t nb, int64_t d, bool accumulate) {
    constexpr int NP = RMS ? 1 : 2;
    __shared__ float red[2][8][33];
    const int c = threadIdx.x & 31, rg = threadIdx.x >> 5;
    const int64_t col = (int64_t)blockIdx.x * 32 + c;
    float sg = 0.f, sb = 0.f;
    if (col < d) {
        // eight loads in flight per sum; the additions stay in row order
        int64_t b = rg;
        for (; b + 56 < nb; b += 64) {
            float tg[8], tb[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                tg[u] = part[(b + 8 * u) * NP * d + col];
                tb[u] = RMS ? 0.f : part[(b + 8 * u) * NP * d + d + col];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) { sg += tg[u]; sb += tb[u]; }
        }
        for (; b < nb; b += 8) {
            sg += part[b * NP * d + col];
            if (!RMS) sb += part[b * NP * d + d + col];
        }
    }
    red[0][rg][c] = sg;
    red[1][rg][c] = sb;
    __syncthreads();
    if (rg == 0 && col < d) {
        float tg = 0.f, tb = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) { tg += red[0][i][c]; tb += red[1][i][c]; }
        if (accumulate) { tg += to_f32(dg[col]); if (!RMS) tb += to_f32(db[col]); }      // earlier micro-batches
        dg[col] = from_f32<T>(tg);
        if (!RMS) db[col] = from_f32<T>(tb);
    }
}

// ---------------------------------------------------------------- activations
__device__ __forceinline__ float gelu_f(float x) {
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return 0.5f * x * (1.0f + tanhf(u));
}
__device__ __forceinline__ float gelu_grad_f(float x) {
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    const float t = tanhf(u);
    return 0.5f * (1.0f + t) + 0.5f * x * (1.0f - t * t) * 0.7978845608028654f * (1.0f + 3.0f * 0.044715f * x * x);
}

// The activation kernels give a thread ACT_UNROLL 16-byte chunks, a whole grid apart from one another, and issue all
// of their loads before the first use: with one chunk per thread too few bytes are in flight to fill the memory system.
constexpr int ACT_UNROLL = 4;

template <typename T>
__global__ void __launch_bounds__(TPB) gelu_fwd_k(const T *__restrict__ u, T *__restrict__ y, int64_t nvec) {
    constexpr int V = Vec16<T>::N;
    const int64_t i0 = (int64_t)blockIdx.x * TPB + threadIdx.x, stride = (int64_t)gridDim.x * TPB;
    Vec16<T> a[ACT_UNROLL];
#pragma unroll
    for (int k = 0; k < ACT_UNROLL; ++k) if (i0 + k * stride < nvec) a[k].load(u + (i0 + k * stride) * V);
#pragma unroll
    for (int k = 0; k < ACT_UNROLL; ++k) {
        if (i0 + k * stride >= nvec) continue;
        float f[V]; a[k].get(f);
#pragma unroll
        for (int j = 0; j < V; ++j) f[j] = gelu_f(f[j]);
        a[k].set(f); a[k].store(y + (i0 + k * stride) * V);
    }
}

template <typename T>
__global__ void __launch_bounds__(TPB) gelu_bwd_k(T *__restrict__ dact, const T *__restrict__ u, int64_t nvec) {
    constexpr int V = Vec16<T>::N;
    const int64_t i0 = (int64_t)blockIdx.x * TPB + threadIdx.x, stride = (int64_t)gridDim.x * TPB;
    Vec16<T> a[ACT_UNROLL], b[ACT_UNROLL];
#pragma unroll
    for (int k = 0; k < ACT_UNROLL; ++k)
        if (i0 + k * stride < nvec) { a[k].load(dact + (i0 + k * stride) * V); b[k].load(u + (i0 + k * stride) * V); }
#pragma unroll
    for (int k = 0; k < ACT_UNROLL; ++k) {
        if (i0 + k * stride >= nvec) continue;
        float fa[V], fb[V]; a[k].get(fa); b[k].get(fb);
#pragma unroll
        for (int j = 0; j < V; ++j) fa[j] *= gelu_grad_f(fb[j]);
        a[k].set(fa); a[k].store(dact + (i0 + k * stride) * V);
    }
}

// element index -> (row, chunk in the row): one division per thread, 32-bit whenever the tensor allows it (a 64-bit
// division by a run-time value is some hundred instructions and was a third of these kernels' work)
__device__ __forceinline__ void split_row(int64_t idx, int64_t cpr, int64_t n, int64_t &row, int64_t &c) {
    if (n <= 0x7fffffff) { const uint32_t r = (uint32_t)idx / (uint32_t)cpr; row = r; c = (uint32_t)idx - r * (uint32_t)cpr; }
    else { row = idx / cpr; c = idx - row * cpr; }
}
// logistic function; in bf16 the hardware's exponential and reciprocal (relative error about 1e-6, against the 4e-3
// of the output's rounding), in fp32 the library's
template <typename T>
__device__ __forceinline__ float sigmoid_f(float x) {
    if (sizeof(T) == 2) return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
    return 1.0f / (1.0f + expf(-x));
}

template <typename T>
__global__ void __launch_bounds__(TPB) swiglu_fwd_k(const T *__restrict__ gu, T *__restrict__ y, int64_t S, int64_t f) {
    constexpr int V = Vec16<T>::N;
    const int64_t cpr = f / V, n = S * cpr;
    const int64_t i0 = (int64_t)blockIdx.x * TPB + threadIdx.x, stride = (int64_t)gridDim.x * TPB;
    Vec16<T> a[ACT_UNROLL], b[ACT_UNROLL];
    int64_t row[ACT_UNROLL], c[ACT_UNROLL];
#pragma unroll
    for (int k = 0; k < ACT_UNROLL; ++k) {
        const int64_t idx = i0 + k * stride;
        if (idx < n) {
            split_row(idx, cpr, n, row[k], c[k]);
            a[k].load(gu + row[k] * 2 * f + c[k] * V); b[k].load(gu + row[k] * 2 * f + f + c[k] * V);
        }
    }
#pragma unroll
    for (int k = 0; k < ACT_UNROLL; ++k) {
        if (i0 + k * stride >= n) continue;
        float fg[V], fu[V]; a[k].get(fg); b[k].get(fu);
#pragma unroll
        for (int j = 0; j < V; ++j) fg[j] = fg[j] * sigmoid_f<T>(fg[j]) * fu[j];
        a[k].set(fg); a[k].store(y + row[k] * f + c[k] * V);
    }
}

template <typename T>
__global__ void __launch_bounds__(TPB) swiglu_bwd_k(const T *__restrict__ dy, const T *__restrict__ gu,
                                                    T *__restrict__ dgu, int64_t S, int64_t f) {
    constexpr int V = Vec16<T>::N;
    const int64_t cpr = f / V, n = S * cpr;
    const int64_t i0 = (int64_t)blockIdx.x * TPB + threadIdx.x, stride = (int64_t)gridDim.x * TPB;
    Vec16<T> a[ACT_UNROLL], b[ACT_UNROLL], e[ACT_UNROLL];
    int64_t row[ACT_UNROLL], c[ACT_UNROLL];
#pragma unroll
    for (int k = 0; k < ACT_UNROLL; ++k) {
        const int64_t idx = i0 + k * stride;
        if (idx < n) {
            split_row(idx, cpr, n, row[k], c[k]);
            a[k].load(gu + row[k] * 2 * f + c[k] * V); b[k].load(gu + row[k] * 2 * f + f + c[k] * V);
            e[k].load(dy + row[k] * f + c[k] * V);
        }
    }
#pragma unroll
    for (int k = 0; k < ACT_UNROLL; ++k) {
        if (i0 + k * stride >= n) continue;
        float fg[V], fu[V], fd[V]; a[k].get(fg); b[k].get(fu); e[k].get(fd);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const float sg = sigmoid_f<T>(fg[j]);
            const float dg = fd[j] * fu[j] * (sg + fg[j] * sg * (1.0f - sg));
            fu[j] = fd[j] * fg[j] * sg;
            fg[j] = dg;
        }
        a[k].set(fg); a[k].store(dgu + row[k] * 2 * f + c[k] * V);
        b[k].set(fu); b[k].store(dgu + row[k] * 2 * f + f + c[k] * V);
    }
}

// rotation of adjacent pairs of q and k, in place; angle = pos * theta^(-2i/dh).  A thread owns one
// 16-byte column chunk for ROPE_ROWS consecutive rows: the inverse frequencies of its pairs are computed
// once, in double; per row the angle is formed and reduced to [-pi, pi] in double (two operations), and
// sine / cosine of the reduced angle are evaluated in float.
constexpr int ROPE_ROWS = 16;
template <typename T>
__global__ void __launch_bounds__(TPB) rope_k(T *__restrict__ qkv, int64_t S, int64_t Tn, int64_t d, int64_t dh,
                                              double log_theta, float sign) {
    constexpr int V = Vec16<T>::N;
    const int64_t cpr = 2 * d / V;                         // q and k columns only
    const int64_t c = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (c >= cpr) return;
    const int64_t col = c * V;                             // column in [0, 2d)
    double inv[V / 2];
#pragma unroll
    for (int j = 0; j < V; j += 2) {
        const int64_t i = ((col + j) % dh) / 2;
        inv[j / 2] = exp(-2.0 * (double)i / (double)dh * log_theta);
    }
    const int64_t r0 = (int64_t)blockIdx.y * ROPE_ROWS;
    const int64_t r1 = r0 + ROPE_ROWS < S ? r0 + ROPE_ROWS : S;
    constexpr double TWO_PI = 6.283185307179586476925, INV_TWO_PI = 0.15915494309189533577;
    for (int64_t row = r0; row < r1; ++row) {
        T *p = qkv + row * 3 * d + col;
        Vec16<T> a; a.load(p);
        float f[V]; a.get(f);
        const double pos = (double)(row % Tn);
#pragma unroll
        for (int j = 0; j < V; j += 2) {
            const double ang = pos * inv[j / 2];
            const float r = (float)fma(-TWO_PI, rint(ang * INV_TWO_PI), ang);
            float sn, cs;
            sincosf(r, &sn, &cs);
            const float cf = cs, sf = sign * sn;
            const float x0 = f[j], x1 = f[j + 1];
            f[j] = x0 * cf - x1 * sf;
            f[j + 1] = x0 * sf + x1 * cf;
        }
        a.set(f); a.store(p);
    }
}

// ---------------------------------------------------------------- cross entropy
// one workgroup per row: online max / sum-of-exponentials, then dlogits written in place.  Two exponentials per
// logit make the kernel as much an ALU as a memory problem at a 50k vocabulary, so they are the hardware's
// base-2 exponential of x*log2(e) (relative error about 1e-6 for |x| up to 20, far inside the loss and gradient bars).
__device__ __forceinline__ float ce_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }
template <typename T>
__global__ void __launch_bounds__(TPB) ce_k(T *__restrict__ logits, const int32_t *__restrict__ labels,
                                            float *__restrict__ losses, int64_t S, int64_t Vn, int64_t ld, int64_t S_total) {
    constexpr int V = Vec16<T>::N;
    __shared__ float red[8];
    const int64_t row = blockIdx.x;
    T *xr = logits + row * ld;
    const int64_t nchunk = ld / V;
    float m = -INFINITY, s = 0.f;
    for (int64_t c = threadIdx.x; c < nchunk; c += TPB) {
        if (c * V >= Vn) break;
        Vec16<T> a; a.load(xr + c * V);
        float f[V]; a.get(f);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            if (c * V + j < Vn) {
                const float x = f[j];
                if (x > m) { s = s * ce_exp(m - x) + 1.0f; m = x; }
                else s += ce_exp(x - m);
            }
        }
    }
    const float M = block_max<TPB / 64>(m, red);
    const float tot = block_sum<TPB / 64>(m == -INFINITY ? 0.f : s * ce_exp(m - M), red);
    const float lse = M + logf(tot);
    const int32_t lab = labels[row];
    if (threadIdx.x == 0) losses[row] = lse - to_f32(xr[lab]);
    __syncthreads();                                       // the label logit is read before it is overwritten
    const float invS = 1.0f / (float)S_total;          // the loss is the mean over the whole batch
    for (int64_t c = threadIdx.x; c < nchunk; c += TPB) {
        Vec16<T> a; a.load(xr + c * V);
        float f[V]; a.get(f);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const int64_t col = c * V + j;
            f[j] = col < Vn ? (ce_exp(f[j] - lse) - (col == lab ? 1.0f : 0.0f)) * invS : 0.0f;
        }
        a.set(f); a.store(xr + c * V);
    }
}

// Same contract as ce_k, for rows of at most TPB*NCH 16-byte chunks: the workgroup keeps its row in registers, so
// the logits are read once with all of a thread's loads in flight together, and maximum, sum and gradient are three
// passes over registers.
template <typename T, int NCH>
__global__ void __launch_bounds__(TPB) ce_reg_k(T *__restrict__ logits, const int32_t *__restrict__ labels,
                                                float *__restrict__ losses, int64_t S, int64_t Vn, int64_t ld, int64_t S_total) {
    constexpr int V = Vec16<T>::N;
    __shared__ float red[8];
    const int64_t row = blockIdx.x;
    T *xr = logits + row * ld;
    const int nchunk = (int)(ld / V), nv = (int)Vn;
    Vec16<T> a[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = threadIdx.x + TPB * i;
        if (c < nchunk) a[i].load(xr + (int64_t)c * V);
    }
    const int32_t lab = labels[row];
    const float x_lab = threadIdx.x == 0 ? to_f32(xr[lab]) : 0.f;      // read long before the row is overwritten
    // only the last chunk that holds logits can be partly padding: the others take the paths without column tests
    constexpr float L2E = 1.4426950408889634f;
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = threadIdx.x + TPB * i;
        if (c < nchunk) {
            float f[V]; a[i].get(f);
            if ((c + 1) * V <= nv) {
#pragma unroll
                for (int j = 0; j < V; ++j) m = fmaxf(m, f[j]);
            } else {
#pragma unroll
                for (int j = 0; j < V; ++j) if (c * V + j < nv) m = fmaxf(m, f[j]);
            }
        }
    }
    const float M = block_max<TPB / 64>(m, red);
    const float kM = -M * L2E;
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = threadIdx.x + TPB * i;
        if (c < nchunk) {
            float f[V]; a[i].get(f);
            if ((c + 1) * V <= nv) {
#pragma unroll
                for (int j = 0; j < V; ++j) sum += __builtin_amdgcn_exp2f(fmaf(f[j], L2E, kM));
            } else {
#pragma unroll
                for (int j = 0; j < V; ++j) if (c * V + j < nv) sum += __builtin_amdgcn_exp2f(fmaf(f[j], L2E, kM));
            }
        }
    }
    const float tot = block_sum<TPB / 64>(sum, red);
    const float lse = M + logf(tot);
    if (threadIdx.x == 0) losses[row] = lse - x_lab;
    // gradient of the mean loss over the whole batch: exp(x - lse) / S_total as one exponential, the 1/S_total folded
    // into the exponent; the label's column is corrected in the one chunk that holds it
    const float invS = 1.0f / (float)S_total;
    const float kL = -lse * L2E - log2f((float)S_total);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = threadIdx.x + TPB * i;
        if (c < nchunk) {
            float f[V]; a[i].get(f);
#pragma unroll
            for (int j = 0; j < V; ++j) f[j] = __builtin_amdgcn_exp2f(fmaf(f[j], L2E, kL));
            if (lab >= c * V && lab < (c + 1) * V) {
#pragma unroll
                for (int j = 0; j < V; ++j) if (c * V + j == lab) f[j] -= invS;
            }
            if ((c + 1) * V > nv) {
#pragma unroll
                for (int j = 0; j < V; ++j) if (c * V + j >= nv) f[j] = 0.f;
            }
            a[i].set(f); a[i].store(xr + (int64_t)c * V);
        }
    }
}

__global__ void __launch_bounds__(TPB) loss_reduce_k(const float *__restrict__ losses, float *__restrict__ loss, int64_t S,
                                                     int64_t S_total, bool accumulate) {
    __shared__ float red[8];
    float s = 0.f;
    for (int64_t i = threadIdx.x; i < S; i += TPB) s += losses[i];
    const float t = block_sum<TPB / 64>(s, red);
    if (threadIdx.x == 0) loss[0] = (accumulate ? loss[0] : 0.f) + t / (float)S_total;
}

// ---------------------------------------------------------------- AdamW
// reads g, theta (fp32 master), m, v; writes theta, m, v and, in bf16 mode, the bf16 compute weight
template <typename T>
__global__ void __launch_bounds__(TPB) adamw_k(const T *__restrict__ g, T *__restrict__ w, float *__restrict__ master,
                                               float *__restrict__ m, float *__restrict__ v, int64_t n, float lr,
                                               float b1, float b2, float eps, float wd, float inv_bc1, float inv_bc2) {
    const int64_t i0 = ((int64_t)blockIdx.x * TPB + threadIdx.x) * 4;
    if (i0 >= n) return;
    float *theta = master ? master : reinterpret_cast<float *>(w);
    if (i0 + 4 <= n) {
        float gg[4];
        if (sizeof(T) == 4) {
            const float4 t = *reinterpret_cast<const float4 *>(g + i0);
            gg[0] = t.x; gg[1] = t.y; gg[2] = t.z; gg[3] = t.w;
        } else {
            const uint2 t = *reinterpret_cast<const uint2 *>(g + i0);
            gg[0] = __uint_as_float(t.x << 16); gg[1] = __uint_as_float(t.x & 0xffff0000u);
            gg[2] = __uint_as_float(t.y << 16); gg[3] = __uint_as_float(t.y & 0xffff0000u);
        }
        float4 th = *reinterpret_cast<float4 *>(theta + i0), mm = *reinterpret_cast<float4 *>(m + i0),
               vv = *reinterpret_cast<float4 *>(v + i0);
        float *pt = &th.x, *pm = &mm.x, *pv = &vv.x;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            pm[j] = b1 * pm[j] + (1.0f - b1) * gg[j];
            pv[j] = b2 * pv[j] + (1.0f - b2) * gg[j] * gg[j];
            pt[j] = pt[j] - lr * (pm[j] * inv_bc1 / (sqrtf(pv[j] * inv_bc2) + eps) + wd * pt[j]);
        }
        *reinterpret_cast<float4 *>(theta + i0) = th;
        *reinterpret_cast<float4 *>(m + i0) = mm;
        *reinterpret_cast<float4 *>(v + i0) = vv;
        if (master) {
            uint2 o;
            o.x = pack_bf16x2(pt[0], pt[1]);
            o.y = pack_bf16x2(pt[2], pt[3]);
            *reinterpret_cast<uint2 *>(w + i0) = o;
        }
    } else {
        for (int64_t i = i0; i < n; ++i) {
            const float gi = to_f32(g[i]);
            const float mi = b1 * m[i] + (1.0f - b1) * gi;
            const float vi = b2 * v[i] + (1.0f - b2) * gi * gi;
            const float ti = theta[i] - lr * (mi * inv_bc1 / (sqrtf(vi * inv_bc2) + eps) + wd * theta[i]);
            m[i] = mi; v[i] = vi; theta[i] = ti;
            if (master) w[i] = from_f32<T>(ti);
        }
    }
}

// ---------------------------------------------------------------- utilities
__global__ void __launch_bounds__(TPB) fill_u32_k(uint32_t *p, uint32_t value, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n) p[i] = value;
}
// 16-byte stores, four per thread (p 16-byte aligned, n16 chunks)
__global__ void __launch_bounds__(TPB) fill_u128_k(uint4 *p, uint32_t value, int64_t n16) {
    const uint4 v = make_uint4(value, value, value, value);
    const int64_t base = (int64_t)blockIdx.x * TPB * 4 + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t i = base + (int64_t)u * TPB;
        if (i < n16) p[i] = v;
    }
}

template <typename T>
__global__ void __launch_bounds__(TPB) convert_k(const float *__restrict__ src, T *__restrict__ dst, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n) dst[i] = from_f32<T>(src[i]);
}

}  // namespace

#define TIO_DISPATCH(dtype, ...)                                  \
    do {                                                          \
        if ((dtype) == TIO_PREC_BF16) { using T = bf16_t; __VA_ARGS__; } \
        else { using T = float; __VA_ARGS__; }                    \
    } while (0)

void embed_fwd(hipStream_t s, int dtype, const int32_t *tok, const void *wte, const void *wpe, void *x, int64_t S,
               int64_t d, int64_t Tn) {
    TIO_DISPATCH(dtype, {
        const int64_t n = S * (d / Vec16<T>::N);
        embed_fwd_k<T><<<blocks_for(n, TPB), TPB, 0, s>>>(tok, (const T *)wte, (const T *)wpe, (T *)x, S, d, Tn);
    });
}

void embed_bwd(hipStream_t s, int dtype, const void *dx, const int32_t *tok, void *dwte, int64_t S, int64_t d, int64_t V,
               bool accumulate) {
    // rows of ids that do not occur stay zero (or, when accumulating over micro-batches, what they were)
    const int64_t words = V * d * (dtype == TIO_PREC_BF16 ? 2 : 4) / 4;
    if (!accumulate) fill_u32(s, dwte, 0u, words);
    TIO_DISPATCH(dtype, { embed_bwd_k<T><<<(unsigned)S, TPB, 0, s>>>((const T *)dx, tok, (T *)dwte, S, d, accumulate); });
}

void posemb_bwd(hipStream_t s, int dtype, const void *dx, void *dwpe, int64_t B, int64_t Tn, int64_t d, bool accumulate) {
    TIO_DISPATCH(dtype, {
        const int64_t n = Tn * (d / Vec16<T>::N);
        posemb_bwd_k<T><<<blocks_for(n, TPB), TPB, 0, s>>>((const T *)dx, (T *)dwpe, B, Tn, d, accumulate);
    });
}

void norm_fwd(hipStream_t s, int dtype, bool rms, const void *x, const void *g, const void *b, void *y, float *stats,
              int64_t S, int64_t d, float eps) {
#define TIO_NORM_FWD_WAVE(NCH)                                                                                              \
    do {                                                                                                                \
        if (rms) norm_fwd_wave_k<T, true, NCH><<<nb, TPB, 0, s>>>((const T *)x, (const T *)g, nullptr, (T *)y, stats, S, d, eps); \
        else norm_fwd_wave_k<T, false, NCH><<<nb, TPB, 0, s>>>((const T *)x, (const T *)g, (const T *)b, (T *)y, stats, S, d, eps); \
    } while (0)
    TIO_DISPATCH(dtype, {
        const unsigned nb = blocks_for(S, TPB / 64);
        const int64_t chunks = d / Vec16<T>::N;          // 16-byte chunks per row; 64 lanes take NCH each
        if (chunks <= 64 * 2) TIO_NORM_FWD_WAVE(2);
        else if (chunks <= 64 * 8) TIO_NORM_FWD_WAVE(8);
        else if (chunks <= 64 * 16) TIO_NORM_FWD_WAVE(16);
        else if (rms) norm_fwd_k<T, true><<<nb, TPB, 0, s>>>((const T *)x, (const T *)g, nullptr, (T *)y, stats, S, d, eps);
        else norm_fwd_k<T, false><<<nb, TPB, 0, s>>>((const T *)x, (const T *)g, (const T *)b, (T *)y, stats, S, d, eps);
    });
#undef TIO_NORM_FWD_WAVE
}

// rows per workgroup the unrolled kernel is built for (what the training program asks for); other counts take the loop kernel
constexpr int NORM_BLOCK_ROWS = 8;
#define TIO_NORM_BWD_ARGS (const T *)dy, (const T *)x, stats, (const T *)g, (const T *)dres, (T *)dx, part, S, d, rows
#define TIO_NORM_BWD_BLOCK(NCH, PF)                                                                              \
    do {                                                                                                         \
        if (rms && dres) norm_bwd_block_k<T, true, true, NCH, PF, NORM_BLOCK_ROWS><<<(unsigned)nb, TPB, 0, s>>>(TIO_NORM_BWD_ARGS);  \
        else if (rms) norm_bwd_block_k<T, true, false, NCH, PF, NORM_BLOCK_ROWS><<<(unsigned)nb, TPB, 0, s>>>(TIO_NORM_BWD_ARGS);    \
        else if (dres) norm_bwd_block_k<T, false, true, NCH, PF, NORM_BLOCK_ROWS><<<(unsigned)nb, TPB, 0, s>>>(TIO_NORM_BWD_ARGS);   \
        else norm_bwd_block_k<T, false, false, NCH, PF, NORM_BLOCK_ROWS><<<(unsigned)nb, TPB, 0, s>>>(TIO_NORM_BWD_ARGS);            \
    } while (0)

void norm_bwd(hipStream_t s, int dtype, bool rms, const void *dy, const void *x, const float *stats, const void *g,
              const void *dres, void *dx, float *part, int64_t S, int64_t d, int64_t nb) {
    const int rows = (int)((S + nb - 1) / nb);
    const size_t lds = ((rms ? 1 : 2) * d + 16) * sizeof(float);
    TIO_DISPATCH(dtype, {
        const int64_t chunks = d / Vec16<T>::N;          // 16-byte chunks per row
        const bool block_ok = rows == NORM_BLOCK_ROWS;
        if (chunks <= 64 * 2) {                          // a wavefront per row
            if (rms) norm_bwd_wave_k<T, true, 2><<<(unsigned)nb, TPB, lds, s>>>(TIO_NORM_BWD_ARGS);
            else norm_bwd_wave_k<T, false, 2><<<(unsigned)nb, TPB, lds, s>>>(TIO_NORM_BWD_ARGS);
        }
        else if (block_ok && chunks <= TPB) TIO_NORM_BWD_BLOCK(1, 4);         // a workgroup per row, rows in flight: 4
        else if (block_ok && chunks <= TPB * 2) TIO_NORM_BWD_BLOCK(2, 4);
        else if (block_ok && chunks <= TPB * 4) TIO_NORM_BWD_BLOCK(4, 2);
        else if (block_ok && chunks <= TPB * 8) TIO_NORM_BWD_BLOCK(8, 1);
        else if (rms) norm_bwd_k<T, true><<<(unsigned)nb, TPB, lds, s>>>(TIO_NORM_BWD_ARGS);
        else norm_bwd_k<T, false><<<(unsigned)nb, TPB, lds, s>>>(TIO_NORM_BWD_ARGS);
    });
}
#undef TIO_NORM_BWD_BLOCK
#undef TIO_NORM_BWD_ARGS

void norm_bwd_params(hipStream_t s, int dtype, bool rms, const float *part, void *dg, void *db, int64_t nb, int64_t d,
                     bool accumulate) {
    TIO_DISPATCH(dtype, {
        if (rms) norm_bwd_params_k<T, true><<<blocks_for(d, 32), TPB, 0, s>>>(part, (T *)dg, nullptr, nb, d, accumulate);
        else norm_bwd_params_k<T, false><<<blocks_for(d, 32), TPB, 0, s>>>(part, (T *)dg, (T *)db, nb, d, accumulate);
    });
}

void gelu_fwd(hipStream_t s, int dtype, const void *u, void *y, int64_t n) {
    TIO_DISPATCH(dtype, {
        const int64_t nv = n / Vec16<T>::N;
        gelu_fwd_k<T><<<blocks_for(nv, TPB * ACT_UNROLL), TPB, 0, s>>>((const T *)u, (T *)y, nv);
    });
}

void gelu_bwd(hipStream_t s, int dtype, void *dact, const void *u, int64_t n) {
    TIO_DISPATCH(dtype, {
        const int64_t nv = n / Vec16<T>::N;
        gelu_bwd_k<T><<<blocks_for(nv, TPB * ACT_UNROLL), TPB, 0, s>>>((T *)dact, (const T *)u, nv);
    });
}

void swiglu_fwd(hipStream_t s, int dtype, const void *gu, void *y, int64_t S, int64_t f) {
    TIO_DISPATCH(dtype, {
        const int64_t n = S * (f / Vec16<T>::N);
        swiglu_fwd_k<T><<<blocks_for(n, TPB * ACT_UNROLL), TPB, 0, s>>>((const T *)gu, (T *)y, S, f);
    });
}

void swiglu_bwd(hipStream_t s, int dtype, const void *dact, const void *gu, void *dgu, int64_t S, int64_t f) {
    TIO_DISPATCH(dtype, {
        const int64_t n = S * (f / Vec16<T>::N);
        swiglu_bwd_k<T><<<blocks_for(n, TPB * ACT_UNROLL), TPB, 0, s>>>((const T *)dact, (const T *)gu, (T *)dgu, S, f);
    });
}

void rope(hipStream_t s, int dtype, void *qkv, int64_t B, int64_t Tn, int64_t H, int64_t dh, float theta, bool inverse) {
    const int64_t S = B * Tn, d = H * dh;
    TIO_DISPATCH(dtype, {
        const dim3 grid(blocks_for(2 * d / Vec16<T>::N, TPB), (unsigned)((S + ROPE_ROWS - 1) / ROPE_ROWS));
        rope_k<T><<<grid, TPB, 0, s>>>((T *)qkv, S, Tn, d, dh, log((double)theta), inverse ? -1.0f : 1.0f);
    });
}

void ce_fwd_bwd(hipStream_t s, int dtype, void *logits, const int32_t *labels, float *losses, int64_t S, int64_t V,
                int64_t ld, int64_t S_total) {
#define TIO_CE_REG(NCH) ce_reg_k<T, NCH><<<(unsigned)S, TPB, 0, s>>>((T *)logits, labels, losses, S, V, ld, S_total)
    TIO_DISPATCH(dtype, {
        const int64_t chunks = ld / Vec16<T>::N;         // 16-byte chunks per row; TPB threads take NCH each
        if (chunks <= TPB * 4) TIO_CE_REG(4);
        else if (chunks <= TPB * 8) TIO_CE_REG(8);
        else if (chunks <= TPB * 16) TIO_CE_REG(16);
        else if (chunks <= TPB * 32) TIO_CE_REG(32);
        else ce_k<T><<<(unsigned)S, TPB, 0, s>>>((T *)logits, labels, losses, S, V, ld, S_total);
    });
#undef TIO_CE_REG
}

void loss_reduce(hipStream_t s, const float *losses, float *loss, int64_t S, int64_t S_total, bool accumulate) {
    loss_reduce_k<<<1, TPB, 0, s>>>(losses, loss, S, S_total, accumulate);
}

void adamw(hipStream_t s, int dtype, const void *g, void *w, float *master, float *m, float *v, int64_t n, float lr,
           float beta1, float beta2, float eps, float wd, float bc1, float bc2) {
    TIO_DISPATCH(dtype, {
        adamw_k<T><<<blocks_for(n, TPB * 4), TPB, 0, s>>>((const T *)g, (T *)w, master, m, v, n, lr, beta1, beta2, eps, wd,
                                                          1.0f / bc1, 1.0f / bc2);
    });
}

void fill_u32(hipStream_t s, void *p, uint32_t value, int64_t n_words) {
    if (n_words <= 0) return;
    int64_t done = 0;
    if ((reinterpret_cast<uintptr_t>(p) & 15) == 0 && n_words >= 1024) {
        const int64_t n16 = n_words / 4;
        fill_u128_k<<<blocks_for(n16, TPB * 4), TPB, 0, s>>>((uint4 *)p, value, n16);
        done = n16 * 4;
    }
    if (done < n_words) fill_u32_k<<<blocks_for(n_words - done, TPB), TPB, 0, s>>>((uint32_t *)p + done, value, n_words - done);
}

void convert_from_f32(hipStream_t s, int dtype, const float *src, void *dst, int64_t n) {
    TIO_DISPATCH(dtype, { convert_k<T><<<blocks_for(n, TPB), TPB, 0, s>>>(src, (T *)dst, n); });
}

}  // namespace k
}  // namespace tio
