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

constexpr int LDS_PAD = 8;     // bf16 elements (16 bytes) appended to every LDS row

union Frag {
    uint4 u;
    bf16x8 v;
};

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
