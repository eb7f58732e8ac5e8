// Tuned bf16 MFMA GEMM for gfx950 (MI355X) for shapes that are whole multiples of the tile:
//   C[Mo x No] = sum_r A(i, r) * B(j, r),  Mo % BM == 0, No % BN == 0, R % 64 == 0.
//
// One 512-thread workgroup (8 waves, two per SIMD) owns a BM x BN output tile and walks the
// reduction in steps of 64.  Both operand tiles are copied global -> LDS by the direct-to-LDS
// load (16 bytes per lane, no register staging) into a double buffer; MFMA 32x32x16 fragments
// are read from LDS with ds_read_b128 when the reduction index is contiguous in memory (KC) and
// with the transposing ds_read_b64_tr_b16 when the output index is contiguous (MC), so no
// operand is ever transposed in global memory.  16-byte chunks are permuted on their way into
// LDS (the lane chooses which global chunk it fetches) so that fragment reads are spread over
// the banks.  The accumulators hold the transposed 32x32 tile (B fragment first), which gives
// each lane 4 consecutive output columns; the epilogue rounds to bf16 once, stages the wave's
// sub-tile through LDS and writes full 128-byte row segments.
#pragma once
#include "axo_common.hpp"

namespace axo {

constexpr int TILE_BK = 64;
constexpr int TILE_THREADS = 512;
constexpr int NUM_XCD = 8;

typedef __attribute__((address_space(3))) void* lds_void_ptr;

#ifndef AXO_SWZ_KC_SHIFT
#define AXO_SWZ_KC_SHIFT 1
#endif

// KC tile in LDS: row r (128 bytes = 8 chunks of 16 bytes), chunk c stored at c ^ f(r).
__device__ __forceinline__ int swz_kc(int r) { return (r >> AXO_SWZ_KC_SHIFT) & 7; }
// MC tile in LDS: reduction row k (ROWLEN*2 bytes), chunk c stored at c ^ 4*(k & 3).
__device__ __forceinline__ int swz_mc(int k) { return (k & 3) << 2; }

// Workgroup -> output tile.  Consecutive workgroup ids go round-robin to the 8 XCDs, each with
// its own L2, so the ids that land on one XCD are given one contiguous run of tiles, and tiles
// are ordered in bands of GROUP_M tile-rows so that the tiles in flight on an XCD share operand
// panels.
__device__ __forceinline__ void tile_of_block(int bid, int nblk, int tiles_m, int tiles_n, int group_m, int& tm, int& tn) {
    int t = bid;
    if (nblk % NUM_XCD == 0) {
        const int per = nblk / NUM_XCD;
        t = (bid % NUM_XCD) * per + bid / NUM_XCD;
    }
    const int band = group_m * tiles_n;
    const int b = t / band;
    const int first_m = b * group_m;
    const int gm = min(group_m, tiles_m - first_m);
    const int in_band = t - b * band;
    tm = first_m + in_band % gm;
    tn = in_band / gm;
}

template <int BM, int BN, int WGM, int WGN, int LA, int LB>
struct TileCfg {
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile
    static constexpr int TM = WTM / 32, TN = WTN / 32;    // MFMA tiles per wave
    static constexpr int A_BYTES = BM * TILE_BK * 2, B_BYTES = BN * TILE_BK * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int A_ROUNDS = BM * 8 / TILE_THREADS, B_ROUNDS = BN * 8 / TILE_THREADS;
    static constexpr int EPI_STRIDE = WTN * 2 + 16;       // bytes per staged row (padded)
    static constexpr int EPI_BYTES = 8 * WTM * EPI_STRIDE;
    static constexpr int LDS_BYTES = (2 * STAGE_BYTES > EPI_BYTES) ? 2 * STAGE_BYTES : EPI_BYTES;
    static_assert(WGM * WGN == 8, "8 waves");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of 32x32 MFMA tiles");
    static_assert((BM * 8) % TILE_THREADS == 0 && (BN * 8) % TILE_THREADS == 0, "whole load rounds");
    static_assert(WTN * 2 % 16 == 0, "staged rows are read in 16-byte chunks");
};

// Per-thread addressing of one operand tile's global -> LDS copy: for each round the element
// offset of the 16-byte chunk this lane fetches (relative to the tile origin at reduction step 0).
template <int ROWS, int LAYOUT, int ROUNDS>
__device__ __forceinline__ void load_offsets(int tid, int64_t ld, int64_t (&off)[ROUNDS]) {
#pragma unroll
    for (int j = 0; j < ROUNDS; ++j) {
        const int q = j * TILE_THREADS + tid;
        if (LAYOUT == KC) {
            const int r = q >> 3, cs = q & 7;
            off[j] = (int64_t)r * ld + ((cs ^ swz_kc(r)) << 3);
        } else {
            constexpr int CPR = ROWS / 8;  // chunks per reduction row
            const int k = q / CPR, cs = q % CPR;
            off[j] = (int64_t)k * ld + ((cs ^ swz_mc(k)) << 3);
        }
    }
}

template <int ROUNDS>
__device__ __forceinline__ void issue_loads(const bf16_t* base, const int64_t* off, char* lds_tile, int wave) {
#pragma unroll
    for (int j = 0; j < ROUNDS; ++j) {
        char* dst = lds_tile + (j * TILE_THREADS + wave * 64) * 16;
        __builtin_amdgcn_global_load_lds(base + off[j], (lds_void_ptr)dst, 16, 0, 0);
    }
}

// Fragment (8 consecutive reduction elements of one output row/column per lane) for the MFMA
// tile whose first row is row0, at reduction sub-step kk (16 elements each).
template <int ROWS, int LAYOUT>
__device__ __forceinline__ bf16x8 read_fragment(const char* lds_tile, int row0, int kk, int lane) {
    if (LAYOUT == KC) {
        const int r = row0 + (lane & 31);
        const int c = kk * 2 + (lane >> 5);
        return *reinterpret_cast<const bf16x8*>(lds_tile + r * 128 + ((c ^ swz_kc(r)) << 4));
    } else {
        // two transposing reads: each hands this lane 4 consecutive reduction elements of column
        // row0 + (lane & 31); lane a of a 16-lane group addresses reduction row a/4, columns 4*(a%4)..+3
        const int i = lane & 15;
        const int krow = kk * 16 + ((lane >> 5) << 3) + (i >> 2);
        const int n = row0 + (((lane >> 4) & 1) << 4) + ((i & 3) << 2);
        const int c = n >> 3, h = (n >> 2) & 1;
        const int sw = (i >> 2) << 2;  // == swz_mc(krow) and == swz_mc(krow + 4)
        const char* p = lds_tile + krow * (ROWS * 2) + ((c ^ sw) << 4) + (h << 3);
        typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * (ROWS * 2)));
        union { struct { s16x4 a, b; } s; bf16x8 v; } u;
        u.s.a = lo;
        u.s.b = hi;
        return u.v;
    }
}

template <int BM, int BN, int WGM, int WGN, int LA, int LB>
__global__ void __launch_bounds__(TILE_THREADS, 1) gemm_tile_kernel(GemmArgs g, int tiles_m, int tiles_n, int group_m) {
    using C = TileCfg<BM, BN, WGM, WGN, LA, LB>;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    int tm, tn;
    tile_of_block(blockIdx.x, gridDim.x, tiles_m, tiles_n, group_m, tm, tn);
    const int i0 = tm * BM, j0 = tn * BN;

    const bf16_t* Ab = (LA == KC) ? g.A + (int64_t)i0 * g.lda : g.A + i0;
    const bf16_t* Bb = (LB == KC) ? g.B + (int64_t)j0 * g.ldb : g.B + j0;
    const int64_t a_step = (LA == KC) ? TILE_BK : (int64_t)TILE_BK * g.lda;
    const int64_t b_step = (LB == KC) ? TILE_BK : (int64_t)TILE_BK * g.ldb;

    int64_t a_off[C::A_ROUNDS], b_off[C::B_ROUNDS];
    load_offsets<BM, LA, C::A_ROUNDS>(tid, g.lda, a_off);
    load_offsets<BN, LB, C::B_ROUNDS>(tid, g.ldb, b_off);

    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int a = 0; a < C::TM; ++a)
#pragma unroll
        for (int b = 0; b < C::TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;

    const int KT = g.R / TILE_BK;
    if (KT > 0) {
        issue_loads<C::A_ROUNDS>(Ab, a_off, smem, wave);
        issue_loads<C::B_ROUNDS>(Bb, b_off, smem + C::A_BYTES, wave);
    }
    for (int kt = 0; kt < KT; ++kt) {
        char* cur = smem + (kt & 1) * C::STAGE_BYTES;
        char* nxt = smem + ((kt + 1) & 1) * C::STAGE_BYTES;
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's copies of step kt have landed
        __syncthreads();                      // ... everyone's have, and everyone left buffer `nxt`
        if (kt + 1 < KT) {
            issue_loads<C::A_ROUNDS>(Ab + (kt + 1) * a_step, a_off, nxt, wave);
            issue_loads<C::B_ROUNDS>(Bb + (kt + 1) * b_step, b_off, nxt + C::A_BYTES, wave);
        }
#pragma unroll
        for (int kk = 0; kk < TILE_BK / 16; ++kk) {
            bf16x8 fa[C::TM], fb[C::TN];
#pragma unroll
            for (int a = 0; a < C::TM; ++a) fa[a] = read_fragment<BM, LA>(cur, wm * C::WTM + a * 32, kk, lane);
#pragma unroll
            for (int b = 0; b < C::TN; ++b) fb[b] = read_fragment<BN, LB>(cur + C::A_BYTES, wn * C::WTN + b * 32, kk, lane);
#pragma unroll
            for (int a = 0; a < C::TM; ++a)
#pragma unroll
                for (int b = 0; b < C::TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[b], fa[a], acc[a][b], 0, 0, 0);
        }
    }

    // ---- epilogue: acc[a][b][e] is C[i0 + wm*WTM + a*32 + (lane&31)][j0 + wn*WTN + b*32 + 8*(e/4) + 4*(lane/32) + e%4]
    __syncthreads();  // all waves are done reading the operand buffers
    char* stage = smem + wave * (C::WTM * C::EPI_STRIDE);
    const int epi = g.epilogue;
#pragma unroll
    for (int b = 0; b < C::TN; ++b) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int ncol = b * 32 + 8 * q + 4 * (lane >> 5);  // within the wave tile
            float bv[4] = {0.f, 0.f, 0.f, 0.f};
            if (epi != EPI_NONE && g.add_bias) {
                const uint2 raw = *reinterpret_cast<const uint2*>(g.bias + j0 + wn * C::WTN + ncol);
                bv[0] = __uint_as_float(raw.x << 16);
                bv[1] = __uint_as_float(raw.x & 0xFFFF0000u);
                bv[2] = __uint_as_float(raw.y << 16);
                bv[3] = __uint_as_float(raw.y & 0xFFFF0000u);
            }
#pragma unroll
            for (int a = 0; a < C::TM; ++a) {
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = acc[a][b][q * 4 + e];
                    if (epi != EPI_NONE) v[e] = apply_epilogue(v[e], bv[e], epi);
                }
                uint2 packed;
                packed.x = (uint32_t)f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
                packed.y = (uint32_t)f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
                const int mrow = a * 32 + (lane & 31);
                *reinterpret_cast<uint2*>(stage + mrow * C::EPI_STRIDE + ncol * 2) = packed;
            }
        }
    }
    // the staging region is private to the wave: only wave-level ordering is needed
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();
    constexpr int LANES_PER_ROW = C::WTN * 2 / 16;
    constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
    bf16_t* Cw = g.C + (int64_t)(i0 + wm * C::WTM) * g.ldc + j0 + wn * C::WTN;
#pragma unroll
    for (int pass = 0; pass < C::WTM / ROWS_PER_PASS; ++pass) {
        const int row = pass * ROWS_PER_PASS + lane / LANES_PER_ROW;
        const int ch = lane % LANES_PER_ROW;
        const u32x4 vdat = *reinterpret_cast<const u32x4*>(stage + row * C::EPI_STRIDE + ch * 16);
        *reinterpret_cast<u32x4*>(Cw + (int64_t)row * g.ldc + ch * 8) = vdat;
    }
}

}  // namespace axo
