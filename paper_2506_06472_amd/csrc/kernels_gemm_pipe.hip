// Pipelined bf16 MFMA GEMM for gfx950: C[M,N] = A . B^T (+bias) (+residual), fp32 accumulate.
//
// Differences from the plain tiled kernel in kernels_gemm.hip:
//  * operand tiles are fetched with raw buffer loads: a lane whose chunk lies outside the operand gets an
//    offset beyond the descriptor's range and the hardware returns zeros, so the steady-state loop has no
//    branches and the compiler can interleave loads, LDS traffic and MFMAs freely;
//  * two operand tile pairs in LDS and two sets of MFMA fragments in registers: while the MFMAs of
//    contraction step s run, the fragments of step s+1 are read from LDS; the last step of a tile runs
//    after the barrier, so the first fragment reads of the next tile are covered by its MFMAs;
//  * an operand stored with the contraction index as the slow dimension ("k-major") is kept in LDS as it
//    is in memory, [k][row], and turned into MFMA fragments by the transposing LDS read
//    (ds_read_b64_tr_b16): within 16 lanes, lane i receives element i%4 of the four 8-byte words
//    addressed by lanes i/4, i/4+4, i/4+8, i/4+12.  Lanes 4j..4j+3 therefore point at k-row j, columns
//    0..15, and lane i ends up with column i of k-rows 0..3: four consecutive contraction slots.
//    No register transposes, and the global loads of a k-major operand are whole 512-byte rows.
#include "../../include/teraio.h"
#include "device_common.h"
#include "kernels.h"
#include "mfma_tiles.h"

namespace tio {
namespace k {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

// byte offsets handed to the buffer loads stay below 2^30 for every valid lane; a lane or a tile that
// must read as zero adds this, which pushes the offset beyond any descriptor range used here
constexpr uint32_t OOB = 0x40000000u;

__device__ __forceinline__ u32x4 buf_load(__amdgpu_buffer_rsrc_t rsrc, uint32_t off) {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
}

// zeroes the bf16 elements j >= keep of an 8-element chunk (keep in 0..8)
__device__ __forceinline__ u32x4 keep_first(u32x4 v, int keep) {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const int left = keep - 2 * d;                      // elements of this dword that stay
        const uint32_t m = left >= 2 ? 0xffffffffu : left == 1 ? 0x0000ffffu : 0u;
        v[d] &= m;
    }
    return v;
}

template <int ROWS, int BK, int NT, bool KM> struct Operand;

// contraction index contiguous: LDS holds [row][BK + pad]
template <int ROWS, int BK, int NT> struct Operand<ROWS, BK, NT, false> {
    static constexpr int LS = BK + LDS_PAD;
    static constexpr int LDS_ELEMS = ROWS * LS;
    static constexpr int CPR = BK / 8, TOTAL = ROWS * CPR, PER = TOTAL / NT;
    static_assert(TOTAL % NT == 0, "tile chunks must divide over the threads");
    uint32_t off[PER];
    u32x4 r[PER];
    __device__ __forceinline__ void init(int64_t ld, int rows_valid, int tid) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + i * NT, row = c / CPR, kc = c % CPR;
            off[i] = row < rows_valid ? (uint32_t)(((int64_t)row * ld + kc * 8) * 2) : OOB;
        }
    }
    static __device__ __forceinline__ uint32_t tile_step(int64_t) { return BK * 2; }
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, uint32_t kb) {
#pragma unroll
        for (int i = 0; i < PER; ++i) r[i] = buf_load(rsrc, off[i] + kb);
    }
    // last, partial tile: only the first kvalid contraction elements exist
    __device__ __forceinline__ void load_tail(__amdgpu_buffer_rsrc_t rsrc, uint32_t kb, int kvalid, int tid) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int kc = (tid + i * NT) % CPR;
            const int keep = kvalid - kc * 8;
            r[i] = keep_first(buf_load(rsrc, keep > 0 ? off[i] + kb : OOB), keep < 0 ? 0 : keep > 8 ? 8 : keep);
        }
    }
    __device__ __forceinline__ void store(uint16_t *lds, int tid) const {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + i * NT, row = c / CPR, kc = c % CPR;
            *reinterpret_cast<u32x4 *>(lds + row * LS + kc * 8) = r[i];
        }
    }
    // per-lane part of the fragment address
    static __device__ __forceinline__ int lane_base(int row0, int lane) { return (row0 + (lane & 31)) * LS + (lane >> 5) * 8; }
    static __device__ __forceinline__ bf16x8 frag(const uint16_t *lds, int base, int sub, int ks) {
        Frag f;
        f.u = *reinterpret_cast<const uint4 *>(lds + base + sub * 32 * LS + ks * 16);
        return f.v;
    }
    // sum over the tile's contraction elements [part*BK/TPR, (part+1)*BK/TPR) of row `row`
    template <int TPR> static __device__ __forceinline__ float row_partial(const uint16_t *lds, int row, int part) {
        float s = 0.f;
        const uint16_t *p = lds + row * LS + part * (BK / TPR);
#pragma unroll
        for (int c = 0; c < BK / TPR; c += 8) {
            const uint4 v = *reinterpret_cast<const uint4 *>(p + c);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) s += __uint_as_float(w[e] << 16) + __uint_as_float(w[e] & 0xffff0000u);
        }
        return s;
    }
};

// contraction index is the slow dimension: LDS holds [k][ROWS + pad], fragments come from transposing reads.
// The pad makes the row pitch 64 bytes modulo 256, so the four k-rows a 16-lane group reads, and the two
// 32-byte column groups of a 32-lane half, fall into different banks.
template <int ROWS, int BK, int NT> struct Operand<ROWS, BK, NT, true> {
    static constexpr int P = ROWS + 32;
    static constexpr int LDS_ELEMS = BK * P;
    static constexpr int CPK = ROWS / 8, TOTAL = BK * CPK, PER = TOTAL / NT;
    static_assert(TOTAL % NT == 0 && (ROWS * 2) % 256 == 0, "tile chunks must divide over the threads");
    uint32_t off[PER];
    u32x4 r[PER];
    __device__ __forceinline__ void init(int64_t ld, int rows_valid, int tid) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + i * NT, kk = c / CPK, rc = c % CPK;
            off[i] = rc * 8 < rows_valid ? (uint32_t)(((int64_t)kk * ld + rc * 8) * 2) : OOB;
        }
    }
    static __device__ __forceinline__ uint32_t tile_step(int64_t ld) { return (uint32_t)(BK * ld * 2); }
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, uint32_t kb) {
#pragma unroll
        for (int i = 0; i < PER; ++i) r[i] = buf_load(rsrc, off[i] + kb);
    }
    __device__ __forceinline__ void load_tail(__amdgpu_buffer_rsrc_t rsrc, uint32_t kb, int kvalid, int tid) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int kk = (tid + i * NT) / CPK;
            r[i] = buf_load(rsrc, kk < kvalid ? off[i] + kb : OOB);
        }
    }
    __device__ __forceinline__ void store(uint16_t *lds, int tid) const {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + i * NT, kk = c / CPK, rc = c % CPK;
            *reinterpret_cast<u32x4 *>(lds + kk * P + rc * 8) = r[i];
        }
    }
    static __device__ __forceinline__ int lane_base(int row0, int lane) {
        return ((lane >> 5) * 8 + ((lane & 15) >> 2)) * P + row0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
    }
    static __device__ __forceinline__ bf16x8 frag(const uint16_t *lds, int base, int sub, int ks) {
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const uint16_t *p = lds + base + sub * 32 + ks * 16 * P;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * P));
        union { s16x4 h[2]; bf16x8 v; } f;
        f.h[0] = lo;
        f.h[1] = hi;
        return f.v;
    }
    template <int TPR> static __device__ __forceinline__ float row_partial(const uint16_t *lds, int row, int part) {
        float s = 0.f;
#pragma unroll 8
        for (int kk = 0; kk < BK / TPR; ++kk) s += bf16_bits_to_f32(lds[(part * (BK / TPR) + kk) * P + row]);
        return s;
    }
};

template <int BM, int BN, int BK, int WGM, int WGN, bool AKM, bool BKM>
__global__ void __launch_bounds__(WGM *WGN * 64)
    gemm_bf16_pipe_k(const uint16_t *__restrict__ A, int64_t lda, const uint16_t *__restrict__ B, int64_t ldb,
                     const uint16_t *__restrict__ bias, const uint16_t *__restrict__ resid, int64_t ldr,
                     uint16_t *__restrict__ C, int64_t ldc, int64_t M, int64_t N, int64_t K, int tiles_m, int tiles_n,
                     uint16_t *__restrict__ rowsum, float *__restrict__ ws, int64_t k_chunk, int rowsum_acc, int xsplits) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int TPR = NT / BM;           // threads that share one row of the A tile for the row sums
    static_assert(NT % BM == 0 && (TPR & (TPR - 1)) == 0 && TPR <= 64 && BK % (8 * TPR) == 0, "row-sum mapping");
    constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32, KS = BK / 16;
    static_assert(KS % 2 == 0, "fragment double buffering needs an even number of contraction steps");
    using OpA = Operand<BM, BK, NT, AKM>;
    using OpB = Operand<BN, BK, NT, BKM>;
    constexpr int TILE = OpA::LDS_ELEMS + OpB::LDS_ELEMS;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    // tile order: see gemm_bf16_k (each XCD works on one contiguous eighth of the tile sequence).  With 2, 4 or 8
    // contraction ranges (xsplits, one-dimensional grid) an XCD owns one range and one part of the tile sequence,
    // so that its L2 fetches only that range of the two operands.
    const int tid = threadIdx.x;
    const int total_tiles = tiles_m * tiles_n;
    int split, nsplit, bid;
    if (xsplits) {
        const int x = (int)(blockIdx.x % 8), i = (int)(blockIdx.x / 8);
        const int parts = 8 / xsplits, chunk = (total_tiles + parts - 1) / parts;
        nsplit = xsplits;
        split = x % xsplits;
        if (i >= chunk) return;
        bid = (x / xsplits) * chunk + i;
    } else {
        nsplit = (int)gridDim.y;
        split = (int)blockIdx.y;
        bid = (int)(blockIdx.x % 8) * ((total_tiles + 7) / 8) + (int)(blockIdx.x / 8);
    }
    if (bid >= total_tiles) return;
    constexpr int GROUP = 8;
    const int per_group = GROUP * tiles_n;
    const int g = bid / per_group;
    const int gm0 = g * GROUP;
    const int gsz = tiles_m - gm0 < GROUP ? tiles_m - gm0 : GROUP;
    const int tm = gm0 + (bid % per_group) % gsz;
    const int tn = (bid % per_group) / gsz;
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, lhi = lane >> 5;

    const int64_t kbeg = (int64_t)split * k_chunk;
    const int64_t kend = (ws != nullptr && kbeg + k_chunk < K) ? kbeg + k_chunk : K;
    const int kspan = kend > kbeg ? (int)(kend - kbeg) : 0;     // a trailing split may be empty
    const int nkf = kspan / BK, rem = kspan % BK, nk = nkf + (rem ? 1 : 0);

    const int rows_a = (int)(M - m0 < BM ? M - m0 : BM), rows_b = (int)(N - n0 < BN ? N - n0 : BN);
    // descriptors cover exactly the part of each operand this workgroup may touch
    const uint16_t *baseA = AKM ? A + kbeg * lda + m0 : A + m0 * lda + kbeg;
    const uint16_t *baseB = BKM ? B + kbeg * ldb + n0 : B + n0 * ldb + kbeg;
    // (rounded up to whole 16-byte chunks: leading dimensions are multiples of 8 elements)
    const int k8 = (kspan + 7) / 8 * 8;
    const int64_t recA = kspan == 0 ? 0 : AKM ? ((int64_t)(kspan - 1) * lda + (rows_a + 7) / 8 * 8) * 2 : ((int64_t)(rows_a - 1) * lda + k8) * 2;
    const int64_t recB = kspan == 0 ? 0 : BKM ? ((int64_t)(kspan - 1) * ldb + (rows_b + 7) / 8 * 8) * 2 : ((int64_t)(rows_b - 1) * ldb + k8) * 2;
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc((void *)baseA, 0, (int)recA, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc((void *)baseB, 0, (int)recB, 0x00020000);
    const uint32_t stepA = OpA::tile_step(lda), stepB = OpB::tile_step(ldb);

    OpA oa;
    OpB ob;
    oa.init(lda, rows_a, tid);
    ob.init(ldb, rows_b, tid);

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    auto load_tile = [&](int kt) {           // kt < nk
        if (kt < nkf) {
            oa.load(rsA, (uint32_t)kt * stepA);
            ob.load(rsB, (uint32_t)kt * stepB);
        } else {
            oa.load_tail(rsA, (uint32_t)kt * stepA, rem, tid);
            ob.load_tail(rsB, (uint32_t)kt * stepB, rem, tid);
        }
    };
    auto store_tile = [&](int buf) {
        oa.store(smem + buf * TILE, tid);
        ob.store(smem + buf * TILE + OpA::LDS_ELEMS, tid);
    };

    const int fa_base = OpA::lane_base(wm * WM, lane), fb_base = OpB::lane_base(wn * WN, lane);
    bf16x8 fa[2][TM], fb[2][TN];
    auto read_frags = [&](int set, int buf, int ks) {
        const uint16_t *As = smem + buf * TILE, *Bs = As + OpA::LDS_ELEMS;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[set][i] = OpA::frag(As, fa_base, i, ks);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[set][j] = OpB::frag(Bs, fb_base, j, ks);
    };
    auto mfmas = [&](int set) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                // first operand indexes the accumulator's register dimension (n), second its lane dimension (m)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0);
    };

    const bool do_rowsum = rowsum != nullptr && tn == 0;
    float rsum = 0.f;

    // prologue: tile 0 in LDS, tile 1 in registers, fragments of step 0 in registers
    load_tile(0);
    store_tile(0);
    if (nk > 1) load_tile(1);
    __syncthreads();
    read_frags(0, 0, 0);

    int kt = 0;
    // steady state: tiles kt+1 (registers) and kt+2 (to be fetched) both exist and kt+2 is a full tile
    for (; kt + 2 < nkf; ++kt) {
        const int cur = kt & 1, nxt = cur ^ 1;
        if (do_rowsum) rsum += OpA::template row_partial<TPR>(smem + cur * TILE, tid / TPR, tid % TPR);
        // Each operand's registers (tile kt+1) go to LDS and are refilled at once with tile kt+2, which
        // gives every global load a whole tile of MFMAs to arrive; both happen early in the tile so the
        // LDS stores have completed long before the barrier.
#pragma unroll
        for (int ks = 0; ks + 1 < KS; ++ks) {
            read_frags((ks + 1) & 1, cur, ks + 1);
            if (ks == 0) {
                oa.store(smem + nxt * TILE, tid);
                oa.load(rsA, (uint32_t)(kt + 2) * stepA);
            }
            if (ks == (KS > 2 ? 1 : 0)) {
                ob.store(smem + nxt * TILE + OpA::LDS_ELEMS, tid);
                ob.load(rsB, (uint32_t)(kt + 2) * stepB);
            }
            mfmas(ks & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
        read_frags(0, nxt, 0);
        mfmas((KS - 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
    }
    // the last (up to three) tiles: same steps, each guarded
    for (; kt < nk; ++kt) {
        const int cur = kt & 1, nxt = cur ^ 1;
        if (do_rowsum) rsum += OpA::template row_partial<TPR>(smem + cur * TILE, tid / TPR, tid % TPR);
#pragma unroll
        for (int ks = 0; ks + 1 < KS; ++ks) {
            read_frags((ks + 1) & 1, cur, ks + 1);
            mfmas(ks & 1);
        }
        if (kt + 1 < nk) store_tile(nxt);
        if (kt + 2 < nk) load_tile(kt + 2);
        __syncthreads();
        if (kt + 1 < nk) read_frags(0, nxt, 0);
        mfmas((KS - 1) & 1);
    }

    if (do_rowsum) {
#pragma unroll
        for (int o = 1; o < TPR; o <<= 1) rsum += __shfl_xor(rsum, o, 64);
        const int64_t m = m0 + tid / TPR;
        if (tid % TPR == 0 && m < M) {
            if (ws) ws[(int64_t)nsplit * M * N + (int64_t)split * M + m] = rsum;
            else rowsum[m] = (uint16_t)f32_to_bf16_bits(rsum + (rowsum_acc ? bf16_bits_to_f32(rowsum[m]) : 0.f));
        }
    }
    // epilogue: lane holds C[m][n .. n+3] for 4 groups of columns per 32x32 tile.
    // Results pass through LDS (the tile buffer that the last contraction tile did not use: every wavefront finished
    // reading it before the last barrier, so no further barrier is needed), one 32-row block of the wavefront's tile at
    // a time, as fp32: a lane then owns eight consecutive columns of one
    // row, so the bias and residual are read and the output is written in whole 16-byte chunks of full rows
    // (writing the accumulator layout directly touches 16 bytes of each of 32 rows per instruction).  The fp32 partial
    // tiles of a split contraction take the same route.
    {
        constexpr int SPF = WN + 4, CPR = WN / 8, PASSES = 32 * CPR / 64;
        static_assert((32 * CPR) % 64 == 0, "a 32-row block is a whole number of wavefront passes");
        const bool wide = (ldc % 8 == 0) && (resid == nullptr || ldr % 8 == 0);     // 16-byte aligned rows
        static_assert((size_t)TILE * 2 >= (size_t)WGM * WGN * 32 * SPF * 4, "the staging blocks fit one tile buffer");
        float *stage = reinterpret_cast<float *>(smem + (nk & 1) * TILE) + wave * (32 * SPF);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<float4 *>(stage + l32 * SPF + j * 32 + q * 8 + lhi * 4) =
                        make_float4(acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int c = p * 64 + lane, row = c / CPR, ch = c % CPR;
                const float4 x0 = *reinterpret_cast<const float4 *>(stage + row * SPF + ch * 8);
                const float4 x1 = *reinterpret_cast<const float4 *>(stage + row * SPF + ch * 8 + 4);
                const int64_t m = m0 + wm * WM + i * 32 + row, n = n0 + wn * WN + ch * 8;
                if (m >= M || n >= N) continue;
                if (ws) {                                   // N is a multiple of 4 in split mode
                    float *dst = ws + ((int64_t)split * M + m) * N + n;
                    *reinterpret_cast<float4 *>(dst) = x0;
                    if (n + 4 < N) *reinterpret_cast<float4 *>(dst + 4) = x1;
                    continue;
                }
                float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
                if (n + 8 <= N && wide) {
                    if (bias) {
                        const uint4 t = *reinterpret_cast<const uint4 *>(bias + n);
                        const uint32_t u[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(u[e] << 16); v[2 * e + 1] += __uint_as_float(u[e] & 0xffff0000u); }
                    }
                    if (resid) {
                        const uint4 t = *reinterpret_cast<const uint4 *>(resid + m * ldr + n);
                        const uint32_t u[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(u[e] << 16); v[2 * e + 1] += __uint_as_float(u[e] & 0xffff0000u); }
                    }
                    uint4 o;
                    o.x = pack_bf16x2(v[0], v[1]);
                    o.y = pack_bf16x2(v[2], v[3]);
                    o.z = pack_bf16x2(v[4], v[5]);
                    o.w = pack_bf16x2(v[6], v[7]);
                    *reinterpret_cast<uint4 *>(C + m * ldc + n) = o;
                } else {
                    for (int e = 0; e < 8 && n + e < N; ++e) {
                        float x = v[e];
                        if (bias) x += bf16_bits_to_f32(bias[n + e]);
                        if (resid) x += bf16_bits_to_f32(resid[m * ldr + n + e]);
                        C[m * ldc + n + e] = (uint16_t)f32_to_bf16_bits(x);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

template <int BM, int BN, int BK, int WGM, int WGN>
bool launch_pipe(hipStream_t s, bool a_km, bool b_km, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                 const void *B, int64_t ldb, const void *bias, const void *resid, int64_t ldr, void *C, int64_t ldc,
                 void *rowsum, float *ws, int splits, bool rowsum_acc) {
    const int64_t k_chunk = splits > 1 ? ((K + splits - 1) / splits + BK - 1) / BK * BK : K;
    // every byte offset a lane can form must stay below 2^30 (see OOB)
    const int64_t kspan = splits > 1 ? k_chunk : K;
    const int64_t spanA = a_km ? (kspan + 3 * BK) * lda * 2 : ((int64_t)BM * lda + kspan + 3 * BK) * 2;
    const int64_t spanB = b_km ? (kspan + 3 * BK) * ldb * 2 : ((int64_t)BN * ldb + kspan + 3 * BK) * 2;
    constexpr int64_t LIMIT = (int64_t)1 << 30;
    if (spanA >= LIMIT || spanB >= LIMIT) return false;
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    const int tiles = tiles_m * tiles_n;
    const int xsplits = (splits == 2 || splits == 4 || splits == 8) ? splits : 0;
    const dim3 grid = xsplits ? dim3((unsigned)(8 * ((tiles + 8 / xsplits - 1) / (8 / xsplits))))
                              : dim3((unsigned)(8 * ((tiles + 7) / 8)), (unsigned)(splits > 1 ? splits : 1));
    const dim3 block(WGM * WGN * 64);
    constexpr int NT = WGM * WGN * 64;
    const size_t lds = (size_t)2 * 2 * ((a_km ? Operand<BM, BK, NT, true>::LDS_ELEMS : Operand<BM, BK, NT, false>::LDS_ELEMS) +
                                        (b_km ? Operand<BN, BK, NT, true>::LDS_ELEMS : Operand<BN, BK, NT, false>::LDS_ELEMS));
    constexpr int lds_max = 2 * 2 * (Operand<BM, BK, NT, true>::LDS_ELEMS + Operand<BN, BK, NT, true>::LDS_ELEMS);
    static_assert(Operand<BM, BK, NT, true>::LDS_ELEMS >= Operand<BM, BK, NT, false>::LDS_ELEMS, "k-major layout is the larger one");
    static bool attr_done = false;
    if (!attr_done) {
        (void)hipFuncSetAttribute((const void *)gemm_bf16_pipe_k<BM, BN, BK, WGM, WGN, false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_max);
        (void)hipFuncSetAttribute((const void *)gemm_bf16_pipe_k<BM, BN, BK, WGM, WGN, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_max);
        (void)hipFuncSetAttribute((const void *)gemm_bf16_pipe_k<BM, BN, BK, WGM, WGN, true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_max);
        (void)hipFuncSetAttribute((const void *)gemm_bf16_pipe_k<BM, BN, BK, WGM, WGN, true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_max);
        attr_done = true;
    }
#define TIO_GEMM_ARGS (const uint16_t *)A, lda, (const uint16_t *)B, ldb, (const uint16_t *)bias, (const uint16_t *)resid, ldr, \
                      (uint16_t *)C, ldc, M, N, K, tiles_m, tiles_n, (uint16_t *)rowsum, ws, k_chunk, (int)rowsum_acc, xsplits
    if (!a_km && !b_km) gemm_bf16_pipe_k<BM, BN, BK, WGM, WGN, false, false><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
    else if (!a_km && b_km) gemm_bf16_pipe_k<BM, BN, BK, WGM, WGN, false, true><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
    else if (a_km && b_km) gemm_bf16_pipe_k<BM, BN, BK, WGM, WGN, true, true><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
    else gemm_bf16_pipe_k<BM, BN, BK, WGM, WGN, true, false><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
#undef TIO_GEMM_ARGS
    return true;
}

}  // namespace

bool gemm_bf16_pipelined(hipStream_t s, int cfg, bool a_km, bool b_km, int64_t M, int64_t N, int64_t K, const void *A,
                         int64_t lda, const void *B, int64_t ldb, const void *bias, const void *resid, int64_t ldr,
                         void *C, int64_t ldc, void *rowsum, float *ws, int splits, bool rowsum_accumulate) {
#define TIO_P(BM, BN, BK, WGM, WGN) launch_pipe<BM, BN, BK, WGM, WGN>(s, a_km, b_km, M, N, K, A, lda, B, ldb, bias, resid, ldr, C, ldc, rowsum, ws, splits, rowsum_accumulate)
    if (cfg == 1) return TIO_P(256, 256, 64, 2, 4);
    return TIO_P(128, 128, 64, 2, 2);
#undef TIO_P
}

}  // namespace k
}  // namespace tio
