// Device-side helpers shared by the kernels: bf16 storage type, 16-byte vector access, wavefront
// (64 lanes) and workgroup reductions.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace tio {

struct bf16_t { uint16_t v; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
// two floats -> two bf16 in one word (lo in bits 15:0), round to nearest even, NaN stays NaN: gfx950 converts a pair
// in one instruction (v_cvt_pk_bf16_f32); doing it by hand costs about a dozen integer operations per pair, which made
// the bf16 elementwise kernels instruction-bound rather than memory-bound
typedef __bf16 tio_bf16x2 __attribute__((ext_vector_type(2)));
typedef float tio_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const tio_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, tio_bf16x2));
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.f) & 0xffffu; }

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_bits_to_f32(x.v); }
template <typename T> __device__ __forceinline__ T from_f32(float f);
template <> __device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) { return bf16_t{(uint16_t)f32_to_bf16_bits(f)}; }

// 16-byte vectors: 4 floats or 8 bf16
template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    float4 raw;
    __device__ __forceinline__ void load(const float *p) { raw = *reinterpret_cast<const float4 *>(p); }
    __device__ __forceinline__ void store(float *p) const { *reinterpret_cast<float4 *>(p) = raw; }
    __device__ __forceinline__ void get(float *f) const { f[0] = raw.x; f[1] = raw.y; f[2] = raw.z; f[3] = raw.w; }
    __device__ __forceinline__ void set(const float *f) { raw = make_float4(f[0], f[1], f[2], f[3]); }
};
template <> struct Vec16<bf16_t> {
    static constexpr int N = 8;
    uint4 raw;
    __device__ __forceinline__ void load(const bf16_t *p) { raw = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void store(bf16_t *p) const { *reinterpret_cast<uint4 *>(p) = raw; }
    __device__ __forceinline__ void get(float *f) const {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
    }
    __device__ __forceinline__ void set(const float *f) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(f[2 * i], f[2 * i + 1]);
        raw = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// 16-byte accesses through a buffer descriptor: an access whose offset lies at or beyond the descriptor's size reads
// zeros / is dropped by the hardware, which lets a kernel guard ragged edges without branches around its memory operations
typedef uint32_t tio_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_over(const void *base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ void buffer_load16(Vec16<float> &v, __amdgpu_buffer_rsrc_t r, uint32_t off) {
    const tio_u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
    v.raw = make_float4(__uint_as_float(t.x), __uint_as_float(t.y), __uint_as_float(t.z), __uint_as_float(t.w));
}
__device__ __forceinline__ void buffer_load16(Vec16<bf16_t> &v, __amdgpu_buffer_rsrc_t r, uint32_t off) {
    const tio_u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
    v.raw = make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void buffer_store16(const Vec16<float> &v, __amdgpu_buffer_rsrc_t r, uint32_t off) {
    const tio_u32x4 t = {__float_as_uint(v.raw.x), __float_as_uint(v.raw.y), __float_as_uint(v.raw.z), __float_as_uint(v.raw.w)};
    __builtin_amdgcn_raw_buffer_store_b128(t, r, (int)off, 0, 0);
}
__device__ __forceinline__ void buffer_store16(const Vec16<bf16_t> &v, __amdgpu_buffer_rsrc_t r, uint32_t off) {
    const tio_u32x4 t = {v.raw.x, v.raw.y, v.raw.z, v.raw.w};
    __builtin_amdgcn_raw_buffer_store_b128(t, r, (int)off, 0, 0);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Sum over a workgroup of NW wavefronts; every thread gets the result.  `red` is LDS of >= NW floats.
template <int NW> __device__ __forceinline__ float block_sum(float v, float *red) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    __syncthreads();
    if (l == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) t += red[i];
    return t;
}
template <int NW> __device__ __forceinline__ float block_max(float v, float *red) {
    v = wave_max(v);
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    __syncthreads();
    if (l == 0) red[w] = v;
    __syncthreads();
    float t = red[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) t = fmaxf(t, red[i]);
    return t;
}

}  // namespace tio
