// Tuned bf16 MFMA GEMM for gfx950 (MI355X) for shapes that are whole multiples of the tile:
//   C[Mo x No] = sum_r A(i, r) * B(j, r),  Mo % BM == 0, No % BN == 0, R % BK == 0.
// Tile counts that do not fill the last round of CUs are balanced by covering part of the output
// with half-width tiles (TileSched).
//
// One 512-thread workgroup (8 waves, two per SIMD) owns a BM x BN output tile and walks the
// reduction in steps of BK (32 or 64) through a ring of STAGES LDS buffers.  Operand tiles are copied
// global -> LDS by the direct-to-LDS load (16 bytes per lane, no register staging); STAGES-1
// steps are in flight while one is being read, which is what hides the ~1.4 us loaded memory
// latency (a two-deep buffer keeps only one step in flight and is latency bound).  MFMA 32x32x16
// fragments are read from LDS with ds_read_b128 when the reduction index is contiguous in memory
// (KC) and with the transposing ds_read_b64_tr_b16 when the output index is contiguous (MC), so
// no operand is ever transposed in global memory.  16-byte chunks are permuted on their way into
// LDS (the lane chooses which global chunk it fetches) so that fragment reads are spread over
// the banks.  The accumulators hold the transposed 32x32 tile (B fragment first), which gives
// each lane 4 consecutive output columns; the epilogue rounds to bf16 once, stages the wave's
// sub-tile through LDS and writes full 128-byte row segments.
#pragma once
#include <type_traits>

#include "axo_common.hpp"

namespace axo {

constexpr int TILE_THREADS = 512;
constexpr int NUM_XCD = 8;

typedef __attribute__((address_space(3))) void* lds_void_ptr;

#ifndef AXO_SCHED
#define AXO_SCHED 1
#endif

// KC tile in LDS: row r is BK*2 bytes = BK/8 chunks of 16 bytes, chunk c stored at
// c ^ ((r / 2) % 8) for BK = 64 and c ^ ((r / 4) % 4) for BK = 32: 16 consecutive rows read at
// the same c then hit 16 different 16-byte bank groups.
template <int BK>
__device__ __forceinline__ int swz_kc(int r) { return BK == 64 ? ((r >> 1) & 7) : ((r >> 2) & 3); }
// MC tile in LDS: reduction row k is ROWS*2 bytes, chunk c stored at c ^ 4*(k % 4): the four
// reduction rows one transposing read touches land in different bank groups.
__device__ __forceinline__ int swz_mc(int k) { return (k & 3) << 2; }

// How one launch is cut into workgroups.  The output is covered by two column regions: columns
// [0, big_cols * 256) with 256x256 tiles and the rest with 256x128 tiles.  Workgroups
// [0, n_big) take the big tiles, the following n_small the small ones, so that CUs that run out
// of big tiles pick up small ones: a tile count that does not fill the last round of CUs is
// balanced by choosing how many columns each region gets (see the host-side planner).
struct TileSched {
    int tiles_m;     // tile rows (both regions use 256-row tiles)
    int big_cols;    // tile columns of the 256-wide region
    int small_cols;  // tile columns of the 128-wide region
    int n_big;       // = tiles_m * big_cols
    int group_m;     // band height of the tile order
};

// Workgroup -> output tile.  Consecutive workgroup ids go round-robin to the 8 XCDs, each with
// its own L2, so the ids that land on one XCD are given one contiguous run of tiles, and tiles
// are ordered in bands of group_m tile-rows so that the tiles in flight on an XCD share operand
// panels.
__device__ __forceinline__ int xcd_contiguous(int bid, int nblk) {
    if (nblk % NUM_XCD != 0) return bid;
    const int per = nblk / NUM_XCD;
    return (bid % NUM_XCD) * per + bid / NUM_XCD;
}

__device__ __forceinline__ void tile_of_index(int t, int tiles_m, int tiles_n, int group_m, int& tm, int& tn) {
    const int band = group_m * tiles_n;
    const int b = t / band;
    const int first_m = b * group_m;
    const int gm = min(group_m, tiles_m - first_m);
    const int in_band = t - b * band;
    tm = first_m + in_band % gm;
    tn = in_band / gm;
}

template <int BM, int BN, int WGM, int WGN, int BK, int STAGES>
struct TileCfg {
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile
    static constexpr int TM = WTM / 32, TN = WTN / 32;    // MFMA tiles per wave
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int A_ROUNDS = BM * (BK / 8) / TILE_THREADS, B_ROUNDS = BN * (BK / 8) / TILE_THREADS;
    static constexpr int LOADS_PER_STAGE = A_ROUNDS + B_ROUNDS;
    static constexpr int EPI_STRIDE = WTN * 2 + 16;  // bytes per staged row (padded)
    static constexpr int EPI_BYTES = 8 * WTM * EPI_STRIDE;
    static constexpr int RING_BYTES = STAGES * STAGE_BYTES;
    static constexpr int LDS_BYTES = (RING_BYTES > EPI_BYTES) ? RING_BYTES : EPI_BYTES;
    static_assert(WGM * WGN == 8, "8 waves");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of 32x32 MFMA tiles");
    static_assert(BK == 32 || BK == 64, "reduction step");
    static_assert((BM * (BK / 8)) % TILE_THREADS == 0 && (BN * (BK / 8)) % TILE_THREADS == 0, "whole load rounds");
    static_assert(STAGES >= 2, "at least one step in flight");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of one CU");
    static_assert(LOADS_PER_STAGE * (STAGES - 1) < 64, "vmcnt is 6 bits");
};

// Per-thread addressing of one operand tile's global -> LDS copy: for each round the element
// offset of the 16-byte chunk this lane fetches (relative to the tile origin at reduction step 0).
template <int ROWS, int LAYOUT, int BK, int ROUNDS>
__device__ __forceinline__ void load_offsets(int tid, int64_t ld, int64_t* off) {
#pragma unroll
    for (int j = 0; j < ROUNDS; ++j) {
        const int q = j * TILE_THREADS + tid;
        if (LAYOUT == KC) {
            constexpr int CPR = BK / 8;  // chunks per row
            const int r = q / CPR, cs = q % CPR;
            off[j] = (int64_t)r * ld + ((cs ^ swz_kc<BK>(r)) << 3);
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
// tile whose first row is row0, at reduction sub-step kk (16 elements each; BK/16 per stage).
template <int ROWS, int LAYOUT, int BK>
__device__ __forceinline__ bf16x8 read_fragment(const char* lds_tile, int row0, int kk, int lane) {
    if (LAYOUT == KC) {
        const int r = row0 + (lane & 31);
        const int c = kk * 2 + (lane >> 5);
        return *reinterpret_cast<const bf16x8*>(lds_tile + r * (BK * 2) + ((c ^ swz_kc<BK>(r)) << 4));
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

// Tells the scheduler to deal the memory instructions of a half-iteration out between its MFMAs:
// one MFMA occupies the matrix pipe for 32 cycles, the wave can issue loads and LDS reads in
// that shadow, and the other wave of the SIMD fills the pipe meanwhile.
template <int N_MFMA, int N_VMEM, int N_DS, int I>
struct Interleave {
    static __device__ __forceinline__ void run() {
#if AXO_SCHED
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
        constexpr int V = (I + 1) * N_VMEM / N_MFMA - I * N_VMEM / N_MFMA;
        if constexpr (V > 0) __builtin_amdgcn_sched_group_barrier(0x020, V, 0);  // VMEM reads
        constexpr int D = (I + 1) * N_DS / N_MFMA - I * N_DS / N_MFMA;
        if constexpr (D > 0) __builtin_amdgcn_sched_group_barrier(0x100, D, 0);  // LDS reads
        if constexpr (I + 1 < N_MFMA) Interleave<N_MFMA, N_VMEM, N_DS, I + 1>::run();
#endif
    }
};

// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt in bits 3:0 and 15:14).
#define AXO_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

// One BM x BN output tile with its top-left corner at (i0, j0), whole reduction.
template <int BM, int BN, int WGM, int WGN, int LA, int LB, int BK, int STAGES>
__device__ __forceinline__ void gemm_tile_body(const GemmArgs& g, const int i0, const int j0, char* smem) {
    using C = TileCfg<BM, BN, WGM, WGN, BK, STAGES>;
    constexpr int KK = BK / 16;  // MFMA sub-steps per stage
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int KT = g.R / BK;
    const int64_t a_step = (LA == KC) ? BK : (int64_t)BK * g.lda;
    const int64_t b_step = (LB == KC) ? BK : (int64_t)BK * g.ldb;
    const bf16_t* Ab = (LA == KC) ? g.A + (int64_t)i0 * g.lda : g.A + i0;
    const bf16_t* Bb = (LB == KC) ? g.B + (int64_t)j0 * g.ldb : g.B + j0;

    int64_t a_off[C::A_ROUNDS], b_off[C::B_ROUNDS];
    load_offsets<BM, LA, BK, C::A_ROUNDS>(tid, g.lda, a_off);
    load_offsets<BN, LB, BK, C::B_ROUNDS>(tid, g.ldb, b_off);

    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int a = 0; a < C::TM; ++a)
#pragma unroll
        for (int b = 0; b < C::TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;

    bf16x8 fa[2][C::TM], fb[2][C::TN];
    auto read_frags = [&](int buf, const char* stage, int kk) {
#pragma unroll
        for (int a = 0; a < C::TM; ++a) fa[buf][a] = read_fragment<BM, LA, BK>(stage, wm * C::WTM + a * 32, kk, lane);
#pragma unroll
        for (int b = 0; b < C::TN; ++b) fb[buf][b] = read_fragment<BN, LB, BK>(stage + C::A_BYTES, wn * C::WTN + b * 32, kk, lane);
    };
    auto mfma_group = [&](int buf) {
#pragma unroll
        for (int a = 0; a < C::TM; ++a)
#pragma unroll
            for (int b = 0; b < C::TN; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][b], fa[buf][a], acc[a][b], 0, 0, 0);
    };
    constexpr int N_MFMA = C::TM * C::TN;
    constexpr int N_DSREAD = (LA == KC ? 1 : 2) * C::TM + (LB == KC ? 1 : 2) * C::TN;
    auto issue_stage = [&](int step) {
        char* dst = smem + (step % STAGES) * C::STAGE_BYTES;
        issue_loads<C::A_ROUNDS>(Ab + step * a_step, a_off, dst, wave);
        issue_loads<C::B_ROUNDS>(Bb + step * b_step, b_off, dst + C::A_BYTES, wave);
    };
    auto interleave = [&](auto n_vmem, auto n_ds) { Interleave<N_MFMA, decltype(n_vmem)::value, decltype(n_ds)::value, 0>::run(); };
    using IC0 = std::integral_constant<int, 0>;
    using ICD = std::integral_constant<int, N_DSREAD>;
    using ICV = std::integral_constant<int, C::LOADS_PER_STAGE>;

    // Ring schedule.  Step s lives in slot s % STAGES.  Before the loop steps 0..STAGES-1 are
    // issued.  Iteration j: read the second half of step j's fragments while the MFMAs of its
    // first half run; then wait until this wave's copy of step j+1 has landed (all but the
    // youngest STAGES-2 steps), workgroup barrier (everyone's copy landed, everyone is done with
    // slot j), refill slot j with step j+STAGES, read the first fragments of step j+1 while the
    // MFMAs of step j's second half run.  A step is issued STAGES-1 iterations before it is read.
    // The steady-state loop is branch free so that the compiler can interleave across it; the
    // last STAGES iterations (nothing left to issue) run in a second loop.
    if (KT > 0) {
        const int pre = KT < STAGES ? KT : STAGES;
        for (int s = 0; s < pre; ++s) issue_stage(s);
        if (pre == STAGES) AXO_WAIT_VMCNT(C::LOADS_PER_STAGE * (STAGES - 1));
        else AXO_WAIT_VMCNT(0);
        __syncthreads();
        read_frags(0, smem, 0);
    }
    int j = 0;
    for (; j + STAGES < KT; ++j) {
        const char* cur = smem + (j % STAGES) * C::STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk + 1 < KK; ++kk) {
            read_frags((kk + 1) & 1, cur, kk + 1);
            mfma_group(kk & 1);
            interleave(IC0{}, ICD{});
        }
        AXO_WAIT_VMCNT(C::LOADS_PER_STAGE * (STAGES - 2));
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wave's reads of slot j are done
        __syncthreads();
        issue_stage(j + STAGES);
        read_frags(0, smem + ((j + 1) % STAGES) * C::STAGE_BYTES, 0);
        mfma_group((KK - 1) & 1);
        interleave(ICV{}, ICD{});
    }
    for (; j < KT; ++j) {
        const char* cur = smem + (j % STAGES) * C::STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk + 1 < KK; ++kk) {
            read_frags((kk + 1) & 1, cur, kk + 1);
            mfma_group(kk & 1);
            interleave(IC0{}, ICD{});
        }
        AXO_WAIT_VMCNT(0);  // fewer than STAGES-2 steps are outstanding now: wait for all of them
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __syncthreads();
        if (j + 1 < KT) read_frags(0, smem + ((j + 1) % STAGES) * C::STAGE_BYTES, 0);
        mfma_group((KK - 1) & 1);
        interleave(IC0{}, ICD{});
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

constexpr int MIX_BK = 64, MIX_STAGES = 2;
using MixBigCfg = TileCfg<256, 256, 2, 4, MIX_BK, MIX_STAGES>;
using MixSmallCfg = TileCfg<256, 128, 4, 2, MIX_BK, MIX_STAGES>;
constexpr int MIX_LDS_BYTES = MixBigCfg::LDS_BYTES > MixSmallCfg::LDS_BYTES ? MixBigCfg::LDS_BYTES : MixSmallCfg::LDS_BYTES;

// One launch over both regions of a TileSched.
template <int LA, int LB>
__global__ void __launch_bounds__(TILE_THREADS, 1) gemm_mixed_kernel(GemmArgs g, TileSched sc) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int bid = blockIdx.x;
    int tm, tn;
    if (bid < sc.n_big) {
        tile_of_index(xcd_contiguous(bid, sc.n_big), sc.tiles_m, sc.big_cols, sc.group_m, tm, tn);
        gemm_tile_body<256, 256, 2, 4, LA, LB, MIX_BK, MIX_STAGES>(g, tm * 256, tn * 256, smem);
    } else {
        const int n_small = (int)gridDim.x - sc.n_big;
        tile_of_index(xcd_contiguous(bid - sc.n_big, n_small), sc.tiles_m, sc.small_cols, sc.group_m, tm, tn);
        gemm_tile_body<256, 128, 4, 2, LA, LB, MIX_BK, MIX_STAGES>(g, tm * 256, sc.big_cols * 256 + tn * 128, smem);
    }
}

}  // namespace axo
