// Causal self-attention, forward and backward, on the packed [S, 3d] q|k|v layout (no head
// transposes ever touch HBM).  This file holds the fp32-ALU formulation used by the fp32 workloads and
// by head dimension 32; bf16 with head dimension 64 or 128 runs on the matrix cores
// (kernels_attn_mfma.hip).  Row-parallel formulation: a query row (forward, dQ) or a key row
// (dK, dV) is owned by G = dh/32 adjacent lanes, each holding a 32-wide slice of the head dimension
// in registers; the opposite side streams through LDS in tiles of 32 rows.  Softmax statistics are
// fp32 (row maximum and log-sum-exp saved for the backward pass); every sum has a fixed order, so
// the result does not depend on scheduling.  The backward pass recomputes the probabilities from
// the saved log-sum-exp; dQ and dK/dV are produced by two launches so that no atomics are needed.
#include "../../include/teraio.h"
#include "device_common.h"
#include "kernels.h"

namespace tio {
namespace k {

namespace {

constexpr int TPB = 256;
constexpr int TJ = 32;           // rows of the streamed side per LDS tile

template <int G> __device__ __forceinline__ float group_sum(float v) {
#pragma unroll
    for (int o = 1; o < G; o <<= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// loads `n` rows (starting at row r0 of this batch element, clipped to T) of a [.., DH] head slice
// into LDS as fp32, zero filling rows past the end
template <typename T, int DH>
__device__ __forceinline__ void load_tile(float *lds, const T *base, int64_t row_stride, int64_t r0, int64_t Tn) {
    constexpr int V = Vec16<T>::N;
    constexpr int CPR = DH / V;
    for (int c = threadIdx.x; c < TJ * CPR; c += TPB) {
        const int r = c / CPR, cc = c % CPR;
        float f[V];
        if (r0 + r < Tn) {
            Vec16<T> v;
            v.load(base + (r0 + r) * row_stride + cc * V);
            v.get(f);
        } else {
#pragma unroll
            for (int i = 0; i < V; ++i) f[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < V; ++i) lds[r * DH + cc * V + i] = f[i];
    }
}

template <typename T> __device__ __forceinline__ void load_slice(float *dst, const T *src) {   // 32 elements
    constexpr int V = Vec16<T>::N;
#pragma unroll
    for (int c = 0; c < 32 / V; ++c) {
        Vec16<T> v;
        v.load(src + c * V);
        v.get(dst + c * V);
    }
}
template <typename T> __device__ __forceinline__ void store_slice(T *dst, const float *src) {
    constexpr int V = Vec16<T>::N;
#pragma unroll
    for (int c = 0; c < 32 / V; ++c) {
        Vec16<T> v;
        v.set(src + c * V);
        v.store(dst + c * V);
    }
}

__device__ __forceinline__ float dot32(const float *a, const float *lds_row) {
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 32; e += 4) {
        const float4 kv = *reinterpret_cast<const float4 *>(lds_row + e);
        s = fmaf(a[e], kv.x, s); s = fmaf(a[e + 1], kv.y, s); s = fmaf(a[e + 2], kv.z, s); s = fmaf(a[e + 3], kv.w, s);
    }
    return s;
}
__device__ __forceinline__ void axpy32(float *acc, float a, const float *lds_row) {
#pragma unroll
    for (int e = 0; e < 32; e += 4) {
        const float4 v = *reinterpret_cast<const float4 *>(lds_row + e);
        acc[e] = fmaf(a, v.x, acc[e]); acc[e + 1] = fmaf(a, v.y, acc[e + 1]);
        acc[e + 2] = fmaf(a, v.z, acc[e + 2]); acc[e + 3] = fmaf(a, v.w, acc[e + 3]);
    }
}

// ---------------------------------------------------------------- forward
template <typename T, int DH>
__global__ void __launch_bounds__(TPB) attn_fwd_k(const T *__restrict__ qkv, T *__restrict__ o, float *__restrict__ lse,
                                                  int64_t Tn, int64_t H, float scale) {
    constexpr int G = DH / 32, R = TPB / G;
    __shared__ __attribute__((aligned(16))) float Ks[TJ * DH];
    __shared__ __attribute__((aligned(16))) float Vs[TJ * DH];
    const int64_t d = H * DH;
    const int64_t bh = blockIdx.y, b = bh / H, h = bh % H;
    const int g = threadIdx.x % G;
    const int64_t i0 = (int64_t)blockIdx.x * R;
    const int64_t i = i0 + threadIdx.x / G;                  // query position within the sequence
    const bool live = i < Tn;
    const T *base = qkv + b * Tn * 3 * d + h * DH;
    float q[32], acc[32];
    if (live) load_slice<T>(q, base + i * 3 * d + g * 32);
#pragma unroll
    for (int e = 0; e < 32; ++e) { q[e] = live ? q[e] * scale : 0.f; acc[e] = 0.f; }
    float m = -INFINITY, l = 0.f;
    const int64_t jmax = (i0 + R - 1 < Tn - 1) ? i0 + R - 1 : Tn - 1;   // last key any row of the block sees
    for (int64_t j0 = 0; j0 <= jmax; j0 += TJ) {
        __syncthreads();
        load_tile<T, DH>(Ks, base + d, 3 * d, j0, Tn);
        load_tile<T, DH>(Vs, base + 2 * d, 3 * d, j0, Tn);
        __syncthreads();
        float s[TJ];
        float tmax = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < TJ; ++jj) {
            float t = group_sum<G>(dot32(q, Ks + jj * DH + g * 32));
            t = (live && j0 + jj <= i) ? t : -INFINITY;
            s[jj] = t;
            tmax = fmaxf(tmax, t);
        }
        if (tmax == -INFINITY) continue;                     // nothing visible in this tile (uniform per group)
        const float mn = fmaxf(m, tmax);
        const float corr = expf(m - mn);
        l *= corr;
#pragma unroll
        for (int e = 0; e < 32; ++e) acc[e] *= corr;
#pragma unroll
        for (int jj = 0; jj < TJ; ++jj) {
            const float p = expf(s[jj] - mn);                // exp(-inf) = 0 for masked keys
            l += p;
            axpy32(acc, p, Vs + jj * DH + g * 32);
        }
        m = mn;
    }
    if (live) {
        const float inv = 1.0f / l;
#pragma unroll
        for (int e = 0; e < 32; ++e) acc[e] *= inv;
        store_slice<T>(o + (b * Tn + i) * d + h * DH + g * 32, acc);
        if (g == 0) lse[bh * Tn + i] = m + logf(l);
    }
}

// ---------------------------------------------------------------- backward
// delta[b,h,t] = sum_e dO[s,h,e] * O[s,h,e].  dh / (elements per 16 bytes) consecutive lanes share one (s, h):
// the wavefront reads consecutive 16-byte chunks, and the partial sums meet in a fixed xor-shuffle order.
template <typename T>
__global__ void __launch_bounds__(TPB) attn_bwd_pre_k(const T *__restrict__ dO, const T *__restrict__ O,
                                                      float *__restrict__ delta, int64_t Bn, int64_t Tn, int64_t H, int64_t dh) {
    constexpr int V = Vec16<T>::N;
    const int G = (int)(dh / V);                                     // lanes per (s, h): a power of two, at most 64
    const int64_t idx = (int64_t)blockIdx.x * TPB + threadIdx.x;    // chunk index = ((s * H + h) * G + g)
    const bool ok = idx < Bn * Tn * H * G;
    float sum = 0.f;
    if (ok) {
        Vec16<T> x, y; x.load(dO + idx * V); y.load(O + idx * V);
        float fx[V], fy[V]; x.get(fx); y.get(fy);
#pragma unroll
        for (int i = 0; i < V; ++i) sum = fmaf(fx[i], fy[i], sum);
    }
    for (int o = 1; o < G; o <<= 1) sum += __shfl_xor(sum, o, 64);
    if (ok && idx % G == 0) {
        const int64_t sh = idx / G, s = sh / H, h = sh % H;
        const int64_t b = s / Tn, t = s % Tn;
        delta[(b * H + h) * Tn + t] = sum;
    }
}

// dQ: a query row per lane group, keys and values stream through LDS
template <typename T, int DH>
__global__ void __launch_bounds__(TPB) attn_bwd_dq_k(const T *__restrict__ dO, const T *__restrict__ qkv,
                                                     const float *__restrict__ lse, const float *__restrict__ delta,
                                                     T *__restrict__ dqkv, int64_t Tn, int64_t H, float scale) {
    constexpr int G = DH / 32, R = TPB / G;
    __shared__ __attribute__((aligned(16))) float Ks[TJ * DH];
    __shared__ __attribute__((aligned(16))) float Vs[TJ * DH];
    const int64_t d = H * DH;
    const int64_t bh = blockIdx.y, b = bh / H, h = bh % H;
    const int g = threadIdx.x % G;
    const int64_t i0 = (int64_t)blockIdx.x * R;
    const int64_t i = i0 + threadIdx.x / G;
    const bool live = i < Tn;
    const T *base = qkv + b * Tn * 3 * d + h * DH;
    float q[32], go[32], dq[32];
    if (live) { load_slice<T>(q, base + i * 3 * d + g * 32); load_slice<T>(go, dO + (b * Tn + i) * d + h * DH + g * 32); }
#pragma unroll
    for (int e = 0; e < 32; ++e) { if (!live) { q[e] = 0.f; go[e] = 0.f; } dq[e] = 0.f; }
    const float li = live ? lse[bh * Tn + i] : 0.f, di = live ? delta[bh * Tn + i] : 0.f;
    const int64_t jmax = (i0 + R - 1 < Tn - 1) ? i0 + R - 1 : Tn - 1;
    for (int64_t j0 = 0; j0 <= jmax; j0 += TJ) {
        __syncthreads();
        load_tile<T, DH>(Ks, base + d, 3 * d, j0, Tn);
        load_tile<T, DH>(Vs, base + 2 * d, 3 * d, j0, Tn);
        __syncthreads();
#pragma unroll 4
        for (int jj = 0; jj < TJ; ++jj) {
            const float s = group_sum<G>(dot32(q, Ks + jj * DH + g * 32)) * scale;
            const float dp = group_sum<G>(dot32(go, Vs + jj * DH + g * 32));
            const float p = (live && j0 + jj <= i) ? expf(s - li) : 0.f;
            axpy32(dq, p * (dp - di) * scale, Ks + jj * DH + g * 32);
        }
    }
    if (live) store_slice<T>(dqkv + (b * Tn + i) * 3 * d + h * DH + g * 32, dq);
}

// dK, dV: a key row per lane group, queries and output gradients stream through LDS
template <typename T, int DH>
__global__ void __launch_bounds__(TPB) attn_bwd_dkv_k(const T *__restrict__ dO, const T *__restrict__ qkv,
                                                      const float *__restrict__ lse, const float *__restrict__ delta,
                                                      T *__restrict__ dqkv, int64_t Tn, int64_t H, float scale) {
    constexpr int G = DH / 32, R = TPB / G;
    __shared__ __attribute__((aligned(16))) float Qs[TJ * DH];
    __shared__ __attribute__((aligned(16))) float Gs[TJ * DH];
    __shared__ float Ls[TJ], Ds[TJ];
    const int64_t d = H * DH;
    const int64_t bh = blockIdx.y, b = bh / H, h = bh % H;
    const int g = threadIdx.x % G;
    const int64_t j0 = (int64_t)blockIdx.x * R;
    const int64_t j = j0 + threadIdx.x / G;                  // key position
    const bool live = j < Tn;
    const T *base = qkv + b * Tn * 3 * d + h * DH;
    float kk[32], vv[32], dk[32], dv[32];
    if (live) { load_slice<T>(kk, base + j * 3 * d + d + g * 32); load_slice<T>(vv, base + j * 3 * d + 2 * d + g * 32); }
#pragma unroll
    for (int e = 0; e < 32; ++e) { if (!live) { kk[e] = 0.f; vv[e] = 0.f; } dk[e] = 0.f; dv[e] = 0.f; }
    for (int64_t i0 = j0 / TJ * TJ; i0 < Tn; i0 += TJ) {     // queries at or after the first key of the block
        __syncthreads();
        load_tile<T, DH>(Qs, base, 3 * d, i0, Tn);
        load_tile<T, DH>(Gs, dO + b * Tn * d + h * DH, d, i0, Tn);
        if (threadIdx.x < TJ) {
            const bool ok = i0 + threadIdx.x < Tn;
            Ls[threadIdx.x] = ok ? lse[bh * Tn + i0 + threadIdx.x] : 0.f;
            Ds[threadIdx.x] = ok ? delta[bh * Tn + i0 + threadIdx.x] : 0.f;
        }
        __syncthreads();
#pragma unroll 4
        for (int ii = 0; ii < TJ; ++ii) {
            const float s = group_sum<G>(dot32(kk, Qs + ii * DH + g * 32)) * scale;
            const float dp = group_sum<G>(dot32(vv, Gs + ii * DH + g * 32));
            const float p = (live && i0 + ii >= j && i0 + ii < Tn) ? expf(s - Ls[ii]) : 0.f;
            axpy32(dv, p, Gs + ii * DH + g * 32);
            axpy32(dk, p * (dp - Ds[ii]) * scale, Qs + ii * DH + g * 32);
        }
    }
    if (live) {
        store_slice<T>(dqkv + (b * Tn + j) * 3 * d + d + h * DH + g * 32, dk);
        store_slice<T>(dqkv + (b * Tn + j) * 3 * d + 2 * d + h * DH + g * 32, dv);
    }
}

}  // namespace

#define TIO_ATTN_DISPATCH(dtype, dh, ...)                                                         \
    do {                                                                                          \
        if ((dtype) == TIO_PREC_BF16) {                                                           \
            using T = bf16_t;                                                                     \
            if ((dh) == 32) { constexpr int DH = 32; __VA_ARGS__; }                               \
            else if ((dh) == 64) { constexpr int DH = 64; __VA_ARGS__; }                          \
            else { constexpr int DH = 128; __VA_ARGS__; }                                         \
        } else {                                                                                  \
            using T = float;                                                                      \
            if ((dh) == 32) { constexpr int DH = 32; __VA_ARGS__; }                               \
            else if ((dh) == 64) { constexpr int DH = 64; __VA_ARGS__; }                          \
            else { constexpr int DH = 128; __VA_ARGS__; }                                         \
        }                                                                                         \
    } while (0)

void attn_fwd(hipStream_t s, int dtype, const void *qkv, void *o, float *lse, int64_t B, int64_t Tn, int64_t H, int64_t dh) {
    if (attn_mfma_supported(dtype, Tn, H, dh)) { attn_fwd_mfma(s, qkv, o, lse, B, Tn, H, dh); return; }
    const float scale = 1.0f / sqrtf((float)dh);
    TIO_ATTN_DISPATCH(dtype, dh, {
        constexpr int R = TPB / (DH / 32);
        const dim3 grid((unsigned)((Tn + R - 1) / R), (unsigned)(B * H));
        attn_fwd_k<T, DH><<<grid, TPB, 0, s>>>((const T *)qkv, (T *)o, lse, Tn, H, scale);
    });
}

void attn_bwd_pre(hipStream_t s, int dtype, const void *dO, const void *O, float *delta, int64_t B, int64_t Tn, int64_t H,
                  int64_t dh) {
    const int64_t n = B * Tn * H * (dh / (dtype == TIO_PREC_BF16 ? 8 : 4));
    if (dtype == TIO_PREC_BF16)
        attn_bwd_pre_k<bf16_t><<<(unsigned)((n + TPB - 1) / TPB), TPB, 0, s>>>((const bf16_t *)dO, (const bf16_t *)O, delta, B, Tn, H, dh);
    else
        attn_bwd_pre_k<float><<<(unsigned)((n + TPB - 1) / TPB), TPB, 0, s>>>((const float *)dO, (const float *)O, delta, B, Tn, H, dh);
}

void attn_bwd(hipStream_t s, int dtype, const void *dO, const void *qkv, const float *lse, const float *delta, void *dqkv,
              int64_t B, int64_t Tn, int64_t H, int64_t dh) {
    if (attn_mfma_supported(dtype, Tn, H, dh)) { attn_bwd_mfma(s, dO, qkv, lse, delta, dqkv, B, Tn, H, dh); return; }
    const float scale = 1.0f / sqrtf((float)dh);
    TIO_ATTN_DISPATCH(dtype, dh, {
        constexpr int R = TPB / (DH / 32);
        const dim3 grid((unsigned)((Tn + R - 1) / R), (unsigned)(B * H));
        attn_bwd_dq_k<T, DH><<<grid, TPB, 0, s>>>((const T *)dO, (const T *)qkv, lse, delta, (T *)dqkv, Tn, H, scale);
        attn_bwd_dkv_k<T, DH><<<grid, TPB, 0, s>>>((const T *)dO, (const T *)qkv, lse, delta, (T *)dqkv, Tn, H, scale);
    });
}

}  // namespace k
}  // namespace tio
