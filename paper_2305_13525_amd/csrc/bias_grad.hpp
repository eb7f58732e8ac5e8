// Bias gradient: db[n] (+)= sum_t dY[t, n], dY bf16 row-major [M x Nl], db fp32.  Memory bound:
// it reads dY once (2 M Nl bytes) and writes Nl floats.
//
// One 1024-thread workgroup owns COLS columns (16, 32 or 64): COLS / 8 lanes across (8 columns =
// one 16-byte load each) by 1024 / (COLS / 8) lanes down the rows.  Every thread sums its rows
// t = r, r + ROWS, ... in fp32 (four loads in flight per thread), the partial sums of a column are
// added in a fixed tree through LDS, and lane (0, c) writes the result: no atomics, so the result
// does not depend on scheduling.  The host picks the widest COLS that still gives a quarter (64
// columns) or an eighth (32 columns) of the 256 CUs a workgroup: wide blocks read whole 128-byte
// lines, which matters more than filling every CU (measured on a 4096 x 6144 shard: 2.6 TB/s
// with 96 workgroups of 64 columns, 1.1 TB/s with 384 of 16; 5.2 TB/s on 4096 x 16384 with 256
// workgroups of 64).  Unrolling the row loop further (8 or 16 loads in flight per thread) was
// measured slower (2.2 TB/s) on the narrow shard and equal on the wide one.
#pragma once
#include "axo_common.hpp"

namespace axo {

constexpr int BG_THREADS = 1024;

struct BiasGradArgs {
    const bf16_t* dY; int64_t lddy;
    float* db;
    int M, Nl;
    int accumulate;  // 0: db = sums, 1: db += sums
};

// One strip of COLS columns, summed by a workgroup of THREADS threads (1024, or 512 inside the
// grouped GEMM launch); part: ROWS128 x (COLS + 1) floats of LDS.  The reduction has the shape of
// the 1024-thread one whatever THREADS is: 128 row lanes (1024 / 8 column lanes at COLS = 64), each
// summing rows t = r, r + 128, ..., then a binary tree over the row lanes; with 512 threads every
// thread plays row lanes r and r + 64 and adds the two sums itself, which is the tree's first
// level.  So both forms give the same bits.
template <int COLS, int THREADS>
__device__ __forceinline__ void bias_grad_strip(const BiasGradArgs& g, int strip, float* part_lds) {
    constexpr int CX = COLS / 8, LANES = BG_THREADS / CX;  // row lanes of the reference shape
    constexpr int ROWS = THREADS / CX;                     // row lanes this workgroup really has
    constexpr int FOLD = LANES / ROWS;                     // reference lanes per thread (1 or 2)
    static_assert(FOLD == 1 || FOLD == 2, "1024 or 512 threads");
    float(*part)[COLS + 1] = reinterpret_cast<float(*)[COLS + 1]>(part_lds);
    const int cx = threadIdx.x % CX, ry = threadIdx.x / CX;
    const int col = strip * COLS + cx * 8;
    const int valid = g.Nl - col;  // columns of this thread's chunk inside the matrix (may be <= 0 or >= 8)
    float s[FOLD][8];
#pragma unroll
    for (int f = 0; f < FOLD; ++f)
#pragma unroll
        for (int i = 0; i < 8; ++i) s[f][i] = 0.f;
#pragma unroll
    for (int f = 0; f < FOLD; ++f) {
        const int r0 = ry + f * ROWS;
        if (valid >= 8) {
#pragma unroll 4
            for (int t = r0; t < g.M; t += LANES) {
                const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(g.dY + (int64_t)t * g.lddy + col));
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    s[f][2 * i] += __uint_as_float(w[i] << 16);
                    s[f][2 * i + 1] += __uint_as_float(w[i] & 0xFFFF0000u);
                }
            }
        } else if (valid > 0) {  // ragged last chunk
            for (int t = r0; t < g.M; t += LANES)
                for (int i = 0; i < valid; ++i) s[f][i] += bf16_bits_to_f32(g.dY[(int64_t)t * g.lddy + col + i]);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) part[ry][cx * 8 + i] = FOLD == 2 ? s[0][i] + s[FOLD - 1][i] : s[0][i];
    __syncthreads();
    for (int half = ROWS / 2; half >= 1; half >>= 1) {  // fixed-shape tree over the row lanes
        if (ry < half) {
#pragma unroll
            for (int i = 0; i < 8; ++i) part[ry][cx * 8 + i] += part[ry + half][cx * 8 + i];
        }
        __syncthreads();
    }
    if (ry == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (col + i < g.Nl) {
                const float v = part[0][cx * 8 + i];
                g.db[col + i] = g.accumulate ? g.db[col + i] + v : v;
            }
    }
}

template <int COLS>
__global__ void __launch_bounds__(BG_THREADS) bias_grad_kernel(BiasGradArgs g) {
    __shared__ float part[(BG_THREADS / (COLS / 8)) * (COLS + 1)];
    bias_grad_strip<COLS, BG_THREADS>(g, blockIdx.x, part);
}

// ---- bias gradient with the rows split over workgroups ------------------------------------------
// The strip kernel above gives a 6144-column shard 96 workgroups for 256 CUs and is bound by memory
// latency (a third of the HBM rate).  Here a strip's rows are cut into S slices, one workgroup each
// (S chosen by the host from the shape alone, for a few hundred workgroups in all; plain loads:
// non-temporal ones were measured 5-10 % slower here);
// a workgroup writes the fp32 sums of its slice to scratch memory [S x Nl], counts itself in on
// its strip's arrival counter, and the workgroup that arrives last adds the S slices of the strip
// in ascending slice order and writes db.  Which workgroup does that addition depends on timing,
// what it computes does not: the result is a fixed function of the input (no floating-point
// atomics).  No workgroup waits for another.
//
// Scratch: `counters` (one uint32 per strip) must be zero when the kernel starts; the last
// workgroup of every strip sets its counter back to zero, so the kernel leaves them as it found
// them.  `partial` needs no initialisation.  Launches that share scratch memory must not overlap.
//
// A 512-thread workgroup is 8 column lanes (16 bytes = 8 columns each: one 128-byte line per row)
// by 64 row lanes; a thread's rows are 64 apart, their loads are issued eight at a time, summed in
// ascending order; the 8 row lanes of a wave are combined with lane exchanges, the 8 waves through
// LDS by wave 0, whose 64 lanes then own one column each.
constexpr int BGS_THREADS = 512;
constexpr int BGS_COLS = 64;
constexpr int BGS_ROW_LANES = BGS_THREADS / (BGS_COLS / 8);  // 64
constexpr int BGS_MAX_SPLIT = 32;

struct BiasGradSplitArgs {
    const bf16_t* dY; int64_t lddy;
    float* db;
    int M, Nl;
    int accumulate;      // 0: db = sums, 1: db += sums
    int S;               // row slices per strip (1: no scratch is touched)
    int rows_per_slice;  // a multiple of BGS_ROW_LANES
    float* partial;      // [S x Nl] fp32
    uint32_t* counters;  // [number of strips]
};

__global__ void __launch_bounds__(BGS_THREADS) bias_grad_split_kernel(BiasGradSplitArgs g) {
    __shared__ float part[BGS_THREADS / 64][BGS_COLS];
    const int strip = blockIdx.x / g.S, slice = blockIdx.x % g.S;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cx = lane & 7, ry = wave * 8 + (lane >> 3);
    const int col = strip * BGS_COLS + cx * 8;
    const int valid = g.Nl - col;  // columns of this thread's chunk inside the matrix (may be <= 0 or >= 8)
    const int row_end = min(g.M, (slice + 1) * g.rows_per_slice);
    float s[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) s[i] = 0.f;
    if (valid >= 8) {
        const bf16_t* base = g.dY + col;
        int t = slice * g.rows_per_slice + ry;
        for (; t + 7 * BGS_ROW_LANES < row_end; t += 8 * BGS_ROW_LANES) {  // eight loads in flight
            u32x4 w[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                w[j] = *(reinterpret_cast<const u32x4*>(base + (int64_t)(t + j * BGS_ROW_LANES) * g.lddy));
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    s[2 * i] += __uint_as_float(w[j][i] << 16);
                    s[2 * i + 1] += __uint_as_float(w[j][i] & 0xFFFF0000u);
                }
        }
        for (; t < row_end; t += BGS_ROW_LANES) {
            const u32x4 w = *(reinterpret_cast<const u32x4*>(base + (int64_t)t * g.lddy));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                s[2 * i] += __uint_as_float(w[i] << 16);
                s[2 * i + 1] += __uint_as_float(w[i] & 0xFFFF0000u);
            }
        }
    } else if (valid > 0) {  // ragged last chunk
        for (int t = slice * g.rows_per_slice + ry; t < row_end; t += BGS_ROW_LANES)
            for (int i = 0; i < valid; ++i) s[i] += bf16_bits_to_f32(g.dY[(int64_t)t * g.lddy + col + i]);
    }
    // the 8 row lanes of the wave (lane bits 3..5), in a fixed butterfly
#pragma unroll
    for (int m = 8; m < 64; m <<= 1)
#pragma unroll
        for (int i = 0; i < 8; ++i) s[i] += __shfl_xor(s[i], m, 64);
    if (lane < 8) {
#pragma unroll
        for (int i = 0; i < 8; ++i) part[wave][cx * 8 + i] = s[i];
    }
    __syncthreads();
    if (wave != 0) return;
    // wave 0: lane c owns column strip * 64 + c
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < BGS_THREADS / 64; ++w) v += part[w][lane];
    const int c = strip * BGS_COLS + lane;
    if (g.S == 1) {
        if (c < g.Nl) g.db[c] = g.accumulate ? g.db[c] + v : v;
        return;
    }
    // Publication without cache-wide fences.  Slice sums, counter and the reads of the last
    // workgroup are all device-scope atomic accesses: they go past the per-XCD L2 to the level all
    // XCDs share.  Order: the wave's stores are complete (acknowledged at that level) before its
    // lane 0 counts the slice in, and the last workgroup issues its reads only after the value of
    // its own count has come back.  (A release / acquire fence pair does the same by writing back
    // and invalidating the whole L2 per workgroup: measured three times slower than the strips.)
    if (c < g.Nl) __hip_atomic_store(g.partial + (int64_t)slice * g.Nl + c, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    uint32_t arrived = 0;
    if (lane == 0) arrived = __hip_atomic_fetch_add(g.counters + strip, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    arrived = __shfl(arrived, 0, 64);
    if (arrived != (uint32_t)(g.S - 1)) return;
    asm volatile("" ::: "memory");
    if (c < g.Nl) {
        float sum = 0.f;
        for (int k = 0; k < g.S; ++k)
            sum += __hip_atomic_load(g.partial + (int64_t)k * g.Nl + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        g.db[c] = g.accumulate ? g.db[c] + sum : sum;
    }
    if (lane == 0) __hip_atomic_store(g.counters + strip, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace axo
