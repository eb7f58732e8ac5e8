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

template <int COLS>
__global__ void __launch_bounds__(BG_THREADS) bias_grad_kernel(BiasGradArgs g) {
    constexpr int CX = COLS / 8, ROWS = BG_THREADS / CX;
    __shared__ float part[ROWS][COLS + 1];
    const int cx = threadIdx.x % CX, ry = threadIdx.x / CX;
    const int col = blockIdx.x * COLS + cx * 8;
    const int valid = g.Nl - col;  // columns of this thread's chunk inside the matrix (may be <= 0 or >= 8)
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (valid >= 8) {
#pragma unroll 4
        for (int t = ry; t < g.M; t += ROWS) {
            const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(g.dY + (int64_t)t * g.lddy + col));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                s[2 * i] += __uint_as_float(w[i] << 16);
                s[2 * i + 1] += __uint_as_float(w[i] & 0xFFFF0000u);
            }
        }
    } else if (valid > 0) {  // ragged last chunk
        for (int t = ry; t < g.M; t += ROWS)
            for (int i = 0; i < valid; ++i) s[i] += bf16_bits_to_f32(g.dY[(int64_t)t * g.lddy + col + i]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) part[ry][cx * 8 + i] = s[i];
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

}  // namespace axo
