// General-shape bf16 MFMA GEMM for gfx950: any Mo, No, R (including ragged tails), both operand
// layouts.  This is the correctness-first kernel: it serves shapes the tuned kernel does not
// take.  128x128 output tile per 256-thread workgroup (4 waves in a 2x2 arrangement, 64x64 per
// wave = 2x2 MFMA 32x32x16 tiles), reduction step 32, one LDS buffer, operands staged
// global -> registers -> LDS with the reduction index contiguous in LDS for both operands.
#pragma once
#include "axo_common.hpp"

namespace axo {

constexpr int GEN_BM = 128, GEN_BN = 128, GEN_BK = 32;
constexpr int GEN_LDS_STRIDE = GEN_BK + 8;  // elements; 80 bytes keeps 16-byte alignment of chunks

// Load 8 consecutive elements starting at p, of which `valid` (0..8) lie inside the matrix;
// the rest read as zero.  p is 16-byte aligned whenever valid == 8.
__device__ __forceinline__ void load8(const bf16_t* p, int valid, bf16_t (&v)[8]) {
    if (valid >= 8) {
        u32x4 w = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) { v[2 * i] = (bf16_t)(w[i] & 0xFFFFu); v[2 * i + 1] = (bf16_t)(w[i] >> 16); }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (i < valid) ? p[i] : (bf16_t)0;
    }
}

// Stage one operand tile [128 outer x 32 reduction] into LDS as lds[outer][reduction].
template <int LAYOUT>
__device__ __forceinline__ void stage_tile(const bf16_t* __restrict__ src, int64_t ld, int outer0, int outer_n,
                                           int r0, int r_n, bf16_t* lds, int tid) {
    if (LAYOUT == KC) {
        // 128 rows x 4 chunks of 8 reduction elements
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            int c = tid + it * 256;
            int row = c >> 2, kc = (c & 3) * 8;
            int gi = outer0 + row, gr = r0 + kc;
            bf16_t v[8];
            int valid = (gi < outer_n) ? min(8, max(0, r_n - gr)) : 0;
            if (valid > 0) load8(src + (int64_t)gi * ld + gr, valid, v);
            else {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = 0;
            }
            u32x4 w;
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = (uint32_t)v[2 * i] | ((uint32_t)v[2 * i + 1] << 16);
            *reinterpret_cast<u32x4*>(lds + row * GEN_LDS_STRIDE + kc) = w;
        }
    } else {
        // 32 reduction rows x 16 chunks of 8 outer elements; transpose on the way into LDS
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            int c = tid + it * 256;
            int k = c >> 4, o = (c & 15) * 8;
            int gr = r0 + k, gi = outer0 + o;
            bf16_t v[8];
            int valid = (gr < r_n) ? min(8, max(0, outer_n - gi)) : 0;
            if (valid > 0) load8(src + (int64_t)gr * ld + gi, valid, v);
            else {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = 0;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) lds[(o + i) * GEN_LDS_STRIDE + k] = v[i];
        }
    }
}

template <int LA, int LB>
__global__ void __launch_bounds__(256) gemm_generic_kernel(GemmArgs g) {
    __shared__ __attribute__((aligned(16))) bf16_t As[GEN_BM * GEN_LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[GEN_BN * GEN_LDS_STRIDE];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i0 = blockIdx.y * GEN_BM, j0 = blockIdx.x * GEN_BN;

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    for (int r0 = 0; r0 < g.R; r0 += GEN_BK) {
        stage_tile<LA>(g.A, g.lda, i0, g.Mo, r0, g.R, As, tid);
        stage_tile<LB>(g.B, g.ldb, j0, g.No, r0, g.R, Bs, tid);
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GEN_BK; kk += 16) {
            bf16x8 fa[2], fb[2];
            const int koff = kk + 8 * (lane >> 5);
#pragma unroll
            for (int a = 0; a < 2; ++a)
                fa[a] = *reinterpret_cast<const bf16x8*>(As + (wm * 64 + a * 32 + (lane & 31)) * GEN_LDS_STRIDE + koff);
#pragma unroll
            for (int b = 0; b < 2; ++b)
                fb[b] = *reinterpret_cast<const bf16x8*>(Bs + (wn * 64 + b * 32 + (lane & 31)) * GEN_LDS_STRIDE + koff);
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
        __syncthreads();
    }

    // accumulator element e of a 32x32 tile: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int col = j0 + wn * 64 + b * 32 + (lane & 31);
            if (col >= g.No) continue;
            float bv = 0.0f;
            if (g.epilogue >= EPI_BIAS && g.epilogue <= EPI_BIAS_GELU_ERF && g.add_bias) bv = bf16_bits_to_f32(g.bias[col]);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = i0 + wm * 64 + a * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (row < g.Mo) {
                    float v = acc[a][b][e];
                    if (g.epilogue == EPI_ACC_F32) {
                        reinterpret_cast<float*>(g.C)[(int64_t)row * g.ldc + col] += v;
                        continue;
                    }
                    if (g.epilogue == EPI_MUL_DGELU_TANH || g.epilogue == EPI_MUL_DGELU_ERF)
                        v = apply_dact(v, bf16_bits_to_f32(g.aux[(int64_t)row * g.ldaux + col]), g.epilogue);
                    else if (g.epilogue != EPI_NONE)
                        v = apply_epilogue(v, bv, g.epilogue);
                    g.C[(int64_t)row * g.ldc + col] = f32_to_bf16_bits(v);
                }
            }
        }
}

}  // namespace axo
