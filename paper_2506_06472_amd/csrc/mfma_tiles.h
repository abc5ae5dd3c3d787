// Building blocks shared by the MFMA kernels (GEMM, attention): vector types of the
// v_mfma_f32_32x32x16_bf16 operands and the staging of operand tiles global -> registers -> LDS.
//
// Operand layout of the instruction D[32x32] += A[32x16] . B[16x32]: lane l supplies row (A) or column (B)
// l%32 and the eight contraction slots 8*(l/32) .. +7; D: lane l owns column l%32 and rows
// 8*(r/4) + 4*(l/32) + r%4 for register r = 0..15.  Any assignment of contraction elements to slots is
// valid as long as A and B use the same one.
#pragma once
#include "device_common.h"

namespace tio {
namespace k {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int LDS_PAD = 8;     // bf16 elements (16 bytes) appended to every LDS row

union Frag {
    uint4 u;
    bf16x8 v;
};

// ---- tiles from global memory straight into LDS
// One wavefront-wide 16-byte-per-lane load from a buffer straight into LDS: lane i's bytes land at
// lds_addr + 16 i.  Written as inline assembly so that the compiler does not order the wavefront's later LDS reads
// behind it (it would wait for every outstanding load before each read of LDS): the kernel waits for these loads
// itself, with s_waitcnt vmcnt before the barrier that publishes a stage.  M0 holds the LDS address; one wait
// state separates its write from the load.
// (The compiler notes that M0 is a reserved register and that it does not track the clobber; it has no use of M0 of its
// own in these kernels: no indirect register indexing, no message or GDS instructions.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds_b128(i32x4 rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory", "m0");
}
#pragma clang diagnostic pop

// buffer descriptor over [base, base + bytes): raw (stride 0) addressing, out-of-range lanes read zero
__device__ __forceinline__ i32x4 make_rsrc(const void *base, uint32_t bytes) {
    const uint64_t a = (uint64_t)(uintptr_t)base;
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32) & 0xffff);
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

__device__ __forceinline__ uint32_t lds_address(const void *p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char *)p;
}

// byte offsets of valid lanes stay below 2^30; a lane that must read zeros adds this and leaves the descriptor's range
constexpr uint32_t DL_OOB = 0x40000000u;

// ---- staging of one operand tile: global -> registers -> LDS ([row][k], row stride BK+LDS_PAD)
template <int ROWS, int BK, int NT, bool KM> struct Stage;

// contraction index contiguous in memory: 16-byte chunks along k
template <int ROWS, int BK, int NT> struct Stage<ROWS, BK, NT, false> {
    static constexpr int CPR = BK / 8, TOTAL = ROWS * CPR, PER = (TOTAL + NT - 1) / NT;
    uint4 r[PER];
    __device__ __forceinline__ void load(const uint16_t *__restrict__ base, int64_t ld, int64_t row0, int64_t rows,
                                         int64_t k0, int64_t K, int tid) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + i * NT;
            const int row = c / CPR, kc = c % CPR;
            const int64_t gr = row0 + row, gk = k0 + kc * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (c < TOTAL && gr < rows && gk < K) {
                v = *reinterpret_cast<const uint4 *>(base + gr * ld + gk);
                if (gk + 8 > K) {                       // ragged end of the contraction: zero the tail
                    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (gk + j >= K) w[j >> 1] &= (j & 1) ? 0x0000ffffu : 0xffff0000u;
                    v = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
            r[i] = v;
        }
    }
    __device__ __forceinline__ void store(uint16_t *lds, int tid) const {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + i * NT;
            if (c < TOTAL) {
                const int row = c / CPR, kc = c % CPR;
                *reinterpret_cast<uint4 *>(lds + row * (BK + LDS_PAD) + kc * 8) = r[i];
            }
        }
    }
};

// contraction index is the slow dimension: 8(k) x 8(rows) blocks, transposed in registers
template <int ROWS, int BK, int NT> struct Stage<ROWS, BK, NT, true> {
    // consecutive lanes take consecutive k-blocks of one row block: with the 144-byte LDS row pitch the
    // sixteen 16-byte stores of a quarter wavefront then fall into sixteen different bank groups
    static constexpr int RB = ROWS / 8, KB = BK / 8, TOTAL = RB * KB, PER = (TOTAL + NT - 1) / NT;
    uint4 r[PER][8];
    __device__ __forceinline__ void load(const uint16_t *__restrict__ base, int64_t ld, int64_t row0, int64_t rows,
                                         int64_t k0, int64_t K, int tid) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + i * NT;
            const int kb = c % KB, rb = c / KB;
            const int64_t gr = row0 + rb * 8;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int64_t gk = k0 + kb * 8 + j;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (c < TOTAL && gr < rows && gk < K) v = *reinterpret_cast<const uint4 *>(base + gk * ld + gr);
                r[i][j] = v;
            }
        }
    }
    __device__ __forceinline__ void store(uint16_t *lds, int tid) const {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + i * NT;
            if (c < TOTAL) {
                const int kb = c % KB, rb = c / KB;
#pragma unroll
                for (int rr = 0; rr < 8; ++rr) {       // output row rr of the 8x8 block: k = 0..7
                    uint32_t w[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint4 &lo = r[i][2 * j], &hi = r[i][2 * j + 1];
                        const uint32_t a = rr < 2 ? lo.x : rr < 4 ? lo.y : rr < 6 ? lo.z : lo.w;
                        const uint32_t b = rr < 2 ? hi.x : rr < 4 ? hi.y : rr < 6 ? hi.z : hi.w;
                        // even row: low halves; odd row: high halves
                        w[j] = (rr & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0x0000ffffu) | (b << 16));
                    }
                    *reinterpret_cast<uint4 *>(lds + (rb * 8 + rr) * (BK + LDS_PAD) + kb * 8) = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
        }
    }
};

}  // namespace k
}  // namespace tio
