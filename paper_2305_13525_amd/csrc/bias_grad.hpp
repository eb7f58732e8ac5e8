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

}  // namespace axo
