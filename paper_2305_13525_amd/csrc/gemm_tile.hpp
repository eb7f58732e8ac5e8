// Tuned bf16 MFMA GEMM for gfx950 (MI355X) for outputs that are whole multiples of the tile:
//   C[Mo x No] = sum_r A(i, r) * B(j, r),  Mo % 256 == 0, No % 128 == 0; the reduction length R is
//   any multiple of 8 (any length at all when both operands have it as their row index).
// Tile counts that do not fill the last round of CUs are balanced by covering part of the output
// with half-width tiles (TileSched).
//
// One 512-thread workgroup (8 waves, two per SIMD) owns a BM x BN output tile and walks the
// reduction in steps of 64 through two LDS stages.  Operand tiles are copied global -> LDS by
// direct-to-LDS buffer loads (16 bytes per lane, no register staging).  MFMA 16x16x32 fragments
// are read from LDS with ds_read_b128 when the reduction index is contiguous in memory (KC) and
// with the transposing ds_read_b64_tr_b16 when the output index is contiguous (MC), so no operand
// is ever transposed in global memory.  16-byte chunks are permuted on their way into LDS (the
// lane chooses which global chunk it fetches) so that fragment reads are spread over the banks.
//
// The steady-state loop contains no vector ALU work at all: measurements showed that every VALU
// instruction (64-bit address arithmetic above all) takes issue slots from the MFMAs of the same
// SIMD.  Global addresses are a buffer descriptor per operand tile, a per-lane byte offset computed
// once, and a scalar offset that advances with the reduction step; LDS fragment addresses are
// per-lane registers computed once per stage, with the tile / sub-step part in the instruction's
// immediate offset; the loop is unrolled over the two stages so that nothing depends on the
// stage index at run time.
//
// The 16x16x32 MFMA is used rather than the 32x32x16 one: at the chip's power limit a loop of
// nothing but MFMAs on random operands sustains 2.0 PFLOP/s with the former and 1.75 with the
// latter (two waves per SIMD).  The accumulators hold the transposed 16x16 tile (B fragment
// first), which gives each lane 4 consecutive output columns; the epilogue rounds to bf16 once,
// stages the wave's sub-tile through LDS and writes full 128-byte row segments.
//
// Sustained, the kernel runs at the chip's power limit rather than at a cycle limit: the loop
// takes about 2260 cycles per step where its MFMAs need 2048, at a clock (1.8 GHz) that the power
// controller sets; a probe without the per-step barrier needed 6 % fewer cycles and ran at a 5 %
// lower clock, for the same time.  What is worth changing here is therefore what saves energy per
// flop (operand traffic) or removes idle time of whole CUs, not what hides stalls.
//
// Two kernels share the tile body: gemm_mixed_kernel (one product per launch) and
// gemm_group_kernel (the tiles of up to twelve independent products in one grid).
#pragma once
#include <type_traits>

#include "axo_common.hpp"
#include "bias_grad.hpp"

namespace axo {

constexpr int TILE_THREADS = 512;
constexpr int TILE_BK = 64;
constexpr int NUM_XCD = 8;

typedef __attribute__((address_space(3))) void* lds_void_ptr;

#ifndef AXO_PRIO
#define AXO_PRIO 1
#endif
#if AXO_PRIO
#define AXO_SETPRIO(n) __builtin_amdgcn_s_setprio(n)
#else
#define AXO_SETPRIO(n)
#endif
#ifndef AXO_SCHED
#define AXO_SCHED 1
#endif

// KC tile in LDS: row r is 128 bytes = 8 chunks of 16 bytes, chunk c stored at c ^ ((r / 2) % 8):
// 16 consecutive rows read at the same c then hit 16 different 16-byte bank groups.
__device__ __forceinline__ int swz_kc(int r) { return (r >> 1) & 7; }
// MC tile in LDS: reduction row k is ROWS*2 bytes, chunk c stored at c ^ f(k) with
// f(k) = 4*(k % 4) + 2*((k / 8) % 2): half a wave's transposing read touches 8 reduction rows
// (k % 4 and (k / 8) % 2 vary) times two 16-byte chunks, which then land in 16 different bank
// groups (without the second term the 16-lane groups collide: measured 50 % conflict cycles).
__device__ __forceinline__ int swz_mc(int k) { return ((k & 3) << 2) | (((k >> 3) & 1) << 1); }

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
    int stagger;     // start_stagger() units, 0 = none
};

// Start-up phase shift.  Tiles of equal length that start together end together, and then all
// 256 CUs write their outputs in one burst (33 MB for 256x256 tiles), which the memory side takes
// 5-6 us to absorb while nothing computes; spread out, a CU's epilogue takes half as long.  The
// first workgroup on every CU (ids below 256) therefore sleeps phase * units * 640 cycles before
// it starts, phase = 0..7 dealt round-robin over the CUs of each XCD; later workgroups start
// whenever their CU falls free, so the shift persists through the launch.  Measured on launches
// of one product: +2 to +5 % (dgrad 4096x2048x16384 1296 -> 1344 TFLOP/s, a one-round launch of
// 256 half-width tiles 1243 -> 1301).  The grouped launch does without: its tiles differ in
// length, which spreads the bursts already, and the idle start then only costs (-1 %).
constexpr int STAGGER_PHASES = 8;
__device__ __forceinline__ void start_stagger(int bid, int units) {
    if (units > 0 && bid < 256) {
        const int n = ((bid >> 3) % STAGGER_PHASES) * units;
        for (int i = 0; i < n; ++i) __builtin_amdgcn_s_sleep(10);
    }
}

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

template <int BM, int BN, int WGM, int WGN>
struct TileCfg {
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile
    static constexpr int TM = WTM / 16, TN = WTN / 16;    // 16x16 MFMA tiles per wave
    static constexpr int AH = TM / 2;                     // A tiles per MFMA group (half the wave tile's rows)
    static constexpr int A_BYTES = BM * TILE_BK * 2, B_BYTES = BN * TILE_BK * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int A_ROUNDS = BM * (TILE_BK / 8) / TILE_THREADS, B_ROUNDS = BN * (TILE_BK / 8) / TILE_THREADS;
    static constexpr int LOADS_PER_STAGE = A_ROUNDS + B_ROUNDS;
    static constexpr int EPI_STRIDE = WTN * 2 + 16;  // bytes per staged row (padded)
    static constexpr int EPI_BYTES = 8 * WTM * EPI_STRIDE;
    static constexpr int RING_BYTES = 2 * STAGE_BYTES;
    static constexpr int LDS_BYTES = (RING_BYTES > EPI_BYTES) ? RING_BYTES : EPI_BYTES;
    static_assert(WGM * WGN == 8, "8 waves");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of pairs of 16x16 MFMA tiles");
    static_assert((BM * (TILE_BK / 8)) % TILE_THREADS == 0 && (BN * (TILE_BK / 8)) % TILE_THREADS == 0, "whole load rounds");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of one CU");
};

// Per-lane byte offset (from the operand tile's origin at reduction step 0) of the 16-byte chunk
// this lane fetches in each load round.  Must stay below 2^32 (checked on the host).
template <int ROWS, int LAYOUT, int ROUNDS>
__device__ __forceinline__ void load_offsets(int tid, int64_t ld, uint32_t* off) {
#pragma unroll
    for (int j = 0; j < ROUNDS; ++j) {
        const int q = j * TILE_THREADS + tid;
        if (LAYOUT == KC) {
            constexpr int CPR = TILE_BK / 8;  // chunks per row
            const int r = q / CPR, cs = q % CPR;
            off[j] = (uint32_t)(((int64_t)r * ld + ((cs ^ swz_kc(r)) << 3)) * 2);
        } else {
            constexpr int CPR = ROWS / 8;  // chunks per reduction row
            const int k = q / CPR, cs = q % CPR;
            off[j] = (uint32_t)(((int64_t)k * ld + ((cs ^ swz_mc(k)) << 3)) * 2);
        }
    }
}

// LDS byte addresses from which this lane reads its MFMA fragments of one operand in one stage.
// A 16x16x32 fragment is 8 consecutive reduction elements (lane/16 selects which 8 of the 32) of
// row/column lane%16 of the tile.  KC: one address per 32-wide reduction sub-step (the tile
// index adds 16 rows = 2048 bytes, folded into the instruction offset).  MC: one address per
// MFMA tile (the sub-step adds 32 reduction rows, folded into the instruction offset).  The two
// stages of an operand are adjacent in LDS, so the stage is an instruction offset as well and one
// set of addresses serves both.
template <int ROWS, int LAYOUT, int NT>
struct FragAddr {
    static constexpr int N = (LAYOUT == KC) ? 2 : NT;
    static constexpr int STAGE_STRIDE = ROWS * TILE_BK * 2;  // bytes between the operand's two stages
    uint32_t a[N];
    __device__ __forceinline__ void init(int row0, int lane, uint32_t tile_base) {
        if (LAYOUT == KC) {
            const int r = row0 + (lane & 15);
#pragma unroll
            for (int kq = 0; kq < 2; ++kq) {
                const int c = kq * 4 + (lane >> 4);
                a[kq] = tile_base + r * (TILE_BK * 2) + ((c ^ swz_kc(r)) << 4);
            }
        } else {
            const int i = lane & 15;
            const int krow = ((lane >> 4) << 3) + (i >> 2);
            const int sw = swz_mc(krow);  // unchanged by the +4 and +32 row offsets added in read()
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int n = row0 + t * 16 + ((i & 3) << 2);
                const int c = n >> 3, h = (n >> 2) & 1;
                a[t] = tile_base + krow * (ROWS * 2) + ((c ^ sw) << 4) + (h << 3);
            }
        }
    }
    // fragment of MFMA tile t at 32-wide sub-step kq of stage s (all compile-time after unrolling)
    __device__ __forceinline__ bf16x8 read(const char* lds0, int s, int t, int kq) const {
        if (LAYOUT == KC) {
            return *reinterpret_cast<const bf16x8*>(lds0 + a[kq] + s * STAGE_STRIDE + t * (16 * TILE_BK * 2));
        } else {
            // two transposing reads: each hands this lane 4 consecutive reduction elements of its column;
            // lane i of a 16-lane group addresses reduction row i/4, columns 4*(i%4)..+3
            typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
            const char* p = lds0 + a[t] + s * STAGE_STRIDE + kq * (32 * ROWS * 2);
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * (ROWS * 2)));
            union { struct { s16x4 a, b; } s; bf16x8 v; } u;
            u.s.a = lo;
            u.s.b = hi;
            return u.v;
        }
    }
};

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;  // a buffer resource descriptor in four SGPRs
template <int V>
using IC = std::integral_constant<int, V>;

// Tells the scheduler to deal the memory instructions of a group out between its MFMAs: one MFMA
// occupies the matrix pipe for 16 cycles, the wave can issue LDS reads in that shadow, and the
// other wave of the SIMD fills the pipe meanwhile.  (The direct-to-LDS loads are inline assembly
// and stay where the source puts them: at the head of their group.)
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
template <int BM, int BN, int WGM, int WGN, int LA, int LB>
__device__ __forceinline__ void gemm_tile_body(const GemmArgs& g, const int i0, const int j0, char* smem) {
    using C = TileCfg<BM, BN, WGM, WGN>;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    // The loop is unrolled over the two LDS stages, so it walks the reduction rounded up to the
    // next multiple of 128; what lies beyond the true length must contribute nothing, whatever
    // the memory there holds (zeros would do for finite data, but a stray infinity times a zero
    // of the other operand would put a NaN into a row that has none: BOTH operands are made zero).
    //  * MC operand (reduction index = row index): rows at or beyond R lie behind the buffer
    //    descriptor's bound, the byte count from the tile origin to the end of the tile's columns
    //    in row R - 1, and read as zeros.
    //  * KC operand (reduction inside the rows): the overrun of a row lands in the next row,
    //    which no linear bound can mask; the surplus 16-byte chunks of the last two steps are
    //    overwritten with zeros in LDS instead (R is a multiple of 8 here, so a chunk is wholly
    //    inside or wholly outside).  The bound (end of the tile's last row) only keeps the last
    //    row's overrun from touching memory behind the matrix.
    // On this chip the range check covers the sum of the per-lane offset and the scalar offset
    // that carries the reduction step (measured: lowering the bound by the scalar offset at every
    // step zeroed the second half of the reduction), so one constant bound serves the whole walk.
    const int KT = (g.R + 2 * TILE_BK - 1) / (2 * TILE_BK) * 2;
    const bool tail = (g.R % (2 * TILE_BK)) != 0;

    // global side: descriptor at the tile origin, per-lane offsets, scalar step
    const bf16_t* Ab = (LA == KC) ? g.A + (int64_t)i0 * g.lda : g.A + i0;
    const bf16_t* Bb = (LB == KC) ? g.B + (int64_t)j0 * g.ldb : g.B + j0;
    // raw buffer descriptor: base, stride 0, dword format, bound in bytes
    auto make_rsrc = [](const bf16_t* p, uint32_t bound) __attribute__((always_inline)) {
        const uint64_t v = reinterpret_cast<uint64_t>(p);
        u32x4_t r;
        r[0] = __builtin_amdgcn_readfirstlane((uint32_t)v);
        r[1] = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32) & 0xFFFFu);
        r[2] = __builtin_amdgcn_readfirstlane(bound);
        r[3] = 0x00020000u;
        return r;
    };
    const uint32_t a_valid = (LA == KC) ? (uint32_t)(((int64_t)(BM - 1) * g.lda + g.R) * 2)
                                        : (uint32_t)((((int64_t)g.R - 1) * g.lda + BM) * 2);
    const uint32_t b_valid = (LB == KC) ? (uint32_t)(((int64_t)(BN - 1) * g.ldb + g.R) * 2)
                                        : (uint32_t)((((int64_t)g.R - 1) * g.ldb + BN) * 2);
    const u32x4_t a_rsrc = make_rsrc(Ab, a_valid);
    const u32x4_t b_rsrc = make_rsrc(Bb, b_valid);
    const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void_ptr)smem;
    const uint32_t a_step = (uint32_t)((LA == KC) ? TILE_BK * 2 : (int64_t)TILE_BK * g.lda * 2);
    const uint32_t b_step = (uint32_t)((LB == KC) ? TILE_BK * 2 : (int64_t)TILE_BK * g.ldb * 2);
    uint32_t a_off[C::A_ROUNDS], b_off[C::B_ROUNDS];
    load_offsets<BM, LA, C::A_ROUNDS>(tid, g.lda, a_off);
    load_offsets<BN, LB, C::B_ROUNDS>(tid, g.ldb, b_off);

    // LDS side: [A stage 0][A stage 1][B stage 0][B stage 1]; fragment addresses of stage 0
    FragAddr<BM, LA, C::TM> fra;
    FragAddr<BN, LB, C::TN> frb;
    fra.init(wm * C::WTM, lane, 0);
    frb.init(wn * C::WTN, lane, 2 * C::A_BYTES);

    f32x4 acc[C::TM][C::TN];
#pragma unroll
    for (int a = 0; a < C::TM; ++a)
#pragma unroll
        for (int b = 0; b < C::TN; ++b)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[a][b][e] = 0.0f;

    // A reduction step of 64 is four MFMA groups: (sub-step kq, row half ah) for kq, ah in {0, 1};
    // a group multiplies AH A fragments with all TN B fragments of its sub-step.  A fragments are
    // double buffered per group, B fragments per sub-step.
    bf16x8 fa[2][C::AH], fb[2][C::TN];
    auto read_a = [&](int set, int s, int kq, int ah) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < C::AH; ++a) fa[set][a] = fra.read(smem, s, ah * C::AH + a, kq);
    };
    auto read_b = [&](int set, int s, int kq) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < C::TN; ++b) fb[set][b] = frb.read(smem, s, b, kq);
    };
    auto mfma_group = [&](int aset, int bset, int ah) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < C::AH; ++a)
#pragma unroll
            for (int b = 0; b < C::TN; ++b)
                acc[ah * C::AH + a][b] =
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[bset][b], fa[aset][a], acc[ah * C::AH + a][b], 0, 0, 0);
    };
    constexpr int N_MFMA = C::AH * C::TN;
    constexpr int RD_A = (LA == KC ? 1 : 2) * C::AH, RD_B = (LB == KC ? 1 : 2) * C::TN;
    uint32_t a_soff = 0, b_soff = 0;  // scalar byte offsets of the reduction step being loaded
    constexpr int NL = C::LOADS_PER_STAGE;
    // One direct-to-LDS load: 16 bytes per lane from descriptor base + off + soff to LDS address
    // M0 + 16 * lane.  Issued through inline assembly on purpose: for a load the compiler knows
    // to write LDS it puts a full vmcnt(0) wait in front of every later transposing LDS read,
    // which stalls the wave for a whole memory latency in every step.  The kernel keeps the
    // ordering itself: the vmcnt(0) wait and the barrier before the last MFMA group of each step.
    // M0 (the LDS destination of the load) is an input operand bound to the physical register, so
    // the compiler writes it itself and knows what the statement reads.
    auto load_lds = [](uint32_t lds_dst, uint32_t off, u32x4_t rsrc, uint32_t soff) __attribute__((always_inline)) {
        asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds"
                     :
                     : "v"(off), "s"(rsrc), "s"(soff), "{m0}"(lds_dst)
                     : "memory");
    };
    // Loads LO..HI-1 of the NL loads that fill stage s with the step at (a_soff, b_soff): the A
    // rounds first, then the B rounds; round j of wave w lands at tile + (j * 512 + w * 64 + lane) * 16.
    auto issue_range = [&](auto lo_tag, auto hi_tag, int s) __attribute__((always_inline)) {
        constexpr int LO = decltype(lo_tag)::value, HI = decltype(hi_tag)::value;
#pragma unroll
        for (int j = LO; j < HI; ++j) {
            if (j < C::A_ROUNDS) {
                load_lds(smem_base + s * C::A_BYTES + (j * TILE_THREADS + wave * 64) * 16, a_off[j], a_rsrc, a_soff);
            } else {
                const int jb = j - C::A_ROUNDS;
                load_lds(smem_base + 2 * C::A_BYTES + s * C::B_BYTES + (jb * TILE_THREADS + wave * 64) * 16,
                         b_off[jb], b_rsrc, b_soff);
            }
        }
    };
    auto advance = [&]() __attribute__((always_inline)) {
        a_soff += a_step;
        b_soff += b_step;
    };
    // A stage's loads are dealt out over three MFMA groups instead of one burst: half right after
    // the barrier that frees the stage, a quarter in each of the first two groups of the next
    // step.  The texture addresser takes one 1 KB wave-load per ~20 cycles, so eight waves that
    // all issue their loads after the barrier block each other (and their MFMAs) for most of a
    // group; the third group of the next step stays free of loads to cover their latency.
    constexpr int E4 = (NL + 1) / 2, E1 = E4 + (NL - E4 + 1) / 2, E2 = NL;

    // One reduction step held in stage s (compile-time).  On entry the fragments of sub-step 0
    // are in register set 0.  The workgroup barrier sits before the last MFMA group: at that
    // point this wave has read all its fragments of stage s and has seen its own copies of stage
    // s^1 land, so after the barrier stage s can be refilled (step j+2) and stage s^1 read.
    // `head`: the previous step began a refill of stage s^1 that this step has to finish;
    // `load`: begin the refill of stage s; `next`: read the first fragments of the next step.
    // Wave priorities fall through the step and are highest right after the barrier: of the two
    // waves of a SIMD the one that lags is then preferred by the MFMA arbiter, which keeps them
    // from serialising (measured: without this one wave of each SIMD waits at the barrier for
    // about 40 % of the step while the other one is starved of MFMA issue slots).
    // A reduction that ends inside the last two steps: the 16-byte chunks of a KC operand that lie
    // beyond its end are overwritten with zeros in LDS once the stage has landed, by the lane
    // that fetched them (round j of thread tid filled slot q = j * 512 + tid of the tile: row
    // q / 8, LDS chunk q % 8, which holds global chunk (q % 8) ^ swz_kc(row), i.e. reduction
    // elements 8 * that onwards).  `rem` = reduction elements of the stage that are real.
    auto zero_tail = [&](auto s_tag, const int rem) __attribute__((always_inline)) {
        constexpr int s = decltype(s_tag)::value;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        if (LA == KC) {
#pragma unroll
            for (int j = 0; j < C::A_ROUNDS; ++j) {
                const int q = j * TILE_THREADS + tid, r = q >> 3, cs = q & 7;
                if (((cs ^ swz_kc(r)) << 3) >= rem) *reinterpret_cast<u32x4*>(smem + s * C::A_BYTES + q * 16) = zero;
            }
        }
        if (LB == KC) {
#pragma unroll
            for (int j = 0; j < C::B_ROUNDS; ++j) {
                const int q = j * TILE_THREADS + tid, r = q >> 3, cs = q & 7;
                if (((cs ^ swz_kc(r)) << 3) >= rem)
                    *reinterpret_cast<u32x4*>(smem + 2 * C::A_BYTES + s * C::B_BYTES + q * 16) = zero;
            }
        }
    };
    // `fix` (first of the two tail steps only): stage s^1 holds the last step, which has just
    // landed; its chunks beyond the end of the reduction are zeroed before the barrier publishes it.
    auto step = [&](auto s_tag, const bool head, const bool load, const bool next, const bool fix) __attribute__((always_inline)) {
        constexpr int s = decltype(s_tag)::value;
        AXO_SETPRIO(2);
        if (head) issue_range(IC<E4>{}, IC<E1>{}, s ^ 1);
        read_a(1, s, 0, 1);
        mfma_group(0, 0, 0);  // (kq 0, ah 0)
        Interleave<N_MFMA, 0, RD_A, 0>::run();
        AXO_SETPRIO(1);
        if (head) {
            issue_range(IC<E1>{}, IC<E2>{}, s ^ 1);
            advance();
        }
        read_a(0, s, 1, 0);
        read_b(1, s, 1);
        mfma_group(1, 0, 1);  // (kq 0, ah 1)
        Interleave<N_MFMA, 0, RD_A + RD_B, 0>::run();
        AXO_SETPRIO(0);
        read_a(1, s, 1, 1);
        mfma_group(0, 1, 0);  // (kq 1, ah 0)
        Interleave<N_MFMA, 0, RD_A, 0>::run();
        __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
        if (fix) zero_tail(IC<s ^ 1>{}, g.R - (KT - 1) * TILE_BK);
        __syncthreads();
        AXO_SETPRIO(3);
        if (load) issue_range(IC<0>{}, IC<E4>{}, s);
        if (next) {
            read_a(0, s ^ 1, 0, 0);
            read_b(0, s ^ 1, 0);
        }
        mfma_group(1, 1, 1);  // (kq 1, ah 1)
        Interleave<N_MFMA, 0, RD_A + RD_B, 0>::run();
    };
    using T0 = std::integral_constant<int, 0>;
    using T1 = std::integral_constant<int, 1>;

    // KT is even and at least 2
    issue_range(IC<0>{}, IC<NL>{}, 0);
    advance();
    issue_range(IC<0>{}, IC<E4>{}, 1);  // step 0 issues the rest of stage 1
    AXO_WAIT_VMCNT(E4);                 // stage 0 has landed
    __syncthreads();
    read_a(0, 0, 0, 0);
    read_b(0, 0, 0);
    for (int j = 0; j + 2 < KT; j += 2) {  // steady state, branch free: steps j, j+1; refills j+2, j+3
        step(T0{}, true, true, true, false);
        step(T1{}, true, true, true, false);
    }
    // The last two steps: nothing left to load.  Step KT-2 sits in stage 0, landed and published
    // (by the barrier of the step before, or the one above); where the reduction ends inside it
    // its surplus chunks are zeroed now, behind a barrier of their own, and the fragments that
    // were read ahead are read again.
    const bool fix = (LA == KC || LB == KC) && tail;
    if (fix) {
        zero_tail(T0{}, g.R - (KT - 2) * TILE_BK);
        __syncthreads();
        read_a(0, 0, 0, 0);
        read_b(0, 0, 0);
    }
    step(T0{}, true, false, true, fix);
    step(T1{}, false, false, false, false);
    AXO_SETPRIO(0);

    // ---- epilogue: acc[a][b][e] is C[i0 + wm*WTM + a*16 + lane%16][j0 + wn*WTN + b*16 + 4*(lane/16) + e]
    __syncthreads();  // all waves are done reading the operand buffers
    char* stage = smem + wave * (C::WTM * C::EPI_STRIDE);
    // The epilogue kind is decided once, outside the element loops: the plain path is then
    // straight-line code (the activation code is large; branching around it per element made the
    // epilogue several times slower than the stores it feeds).  Every branch of that decision is
    // a complete epilogue, stores included; whatever the branches share (the wave tile's origin,
    // the output pointer) is formed here, ahead of the decision, with the origin pinned in scalar
    // registers, so no branch has a version of its own to merge afterwards.  (An earlier form
    // computed the origin behind a three-way switch; the generated code of one dgrad branch then
    // lacked the upper half of the 64-bit column offset and the stores went astray.  Positional,
    // bit-exact tests of every epilogue kind on both tile sizes guard this.)
    int wrow0 = i0 + wm * C::WTM, wcol0 = j0 + wn * C::WTN;
    asm volatile("" : "+s"(wrow0), "+s"(wcol0));
    bf16_t* const Cw = g.C + (int64_t)wrow0 * g.ldc + wcol0;
    auto convert_and_stage = [&](auto epi_tag) __attribute__((always_inline)) {
        constexpr int EPI = decltype(epi_tag)::value;
        constexpr bool FWD_EPI = EPI >= EPI_BIAS && EPI <= EPI_BIAS_GELU_ERF;
        constexpr bool DACT = EPI == EPI_MUL_DGELU_TANH || EPI == EPI_MUL_DGELU_ERF;
#pragma unroll
        for (int b = 0; b < C::TN; ++b) {
            const int ncol = b * 16 + 4 * (lane >> 4);  // within the wave tile
            float bv[4] = {0.f, 0.f, 0.f, 0.f};
            if (FWD_EPI && g.add_bias) {
                const uint2 raw = *reinterpret_cast<const uint2*>(g.bias + wcol0 + ncol);
                bv[0] = __uint_as_float(raw.x << 16);
                bv[1] = __uint_as_float(raw.x & 0xFFFF0000u);
                bv[2] = __uint_as_float(raw.y << 16);
                bv[3] = __uint_as_float(raw.y & 0xFFFF0000u);
            }
#pragma unroll
            for (int a = 0; a < C::TM; ++a) {
                const int mrow = a * 16 + (lane & 15);
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[a][b][e];
                if (FWD_EPI) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = apply_epilogue(v[e], bv[e], EPI);
                }
                if (DACT) {  // the four pre-activations that belong to this lane's four outputs
                    const uint2 raw = *reinterpret_cast<const uint2*>(
                        g.aux + (int64_t)(wrow0 + mrow) * g.ldaux + wcol0 + ncol);
                    v[0] = apply_dact(v[0], __uint_as_float(raw.x << 16), EPI);
                    v[1] = apply_dact(v[1], __uint_as_float(raw.x & 0xFFFF0000u), EPI);
                    v[2] = apply_dact(v[2], __uint_as_float(raw.y << 16), EPI);
                    v[3] = apply_dact(v[3], __uint_as_float(raw.y & 0xFFFF0000u), EPI);
                }
                uint2 packed;
                packed.x = pack_bf16x2(v[0], v[1]);
                packed.y = pack_bf16x2(v[2], v[3]);
                *reinterpret_cast<uint2*>(stage + mrow * C::EPI_STRIDE + ncol * 2) = packed;
            }
        }
    };
    // The staged sub-tile out to memory as full row segments of 16 bytes per lane.
    auto store_staged = [&]() __attribute__((always_inline)) {
        // the staging region is private to the wave: only wave-level ordering is needed
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
        __builtin_amdgcn_wave_barrier();
        constexpr int LANES_PER_ROW = C::WTN * 2 / 16;
        constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
        // All reads are issued before the first store: interleaved one by one (as the compiler
        // orders them when left alone) every store waits for its own LDS read, and the 16 round
        // trips cost more than the stores themselves (measured 5000 cycles for the slower wave of
        // each SIMD).  The accumulators are dead by now, so the registers are free.
        constexpr int PASSES = C::WTM / ROWS_PER_PASS;
        u32x4 vdat[PASSES];
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = p * ROWS_PER_PASS + lane / LANES_PER_ROW, ch = lane % LANES_PER_ROW;
            vdat[p] = *reinterpret_cast<const u32x4*>(stage + row * C::EPI_STRIDE + ch * 16);
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = p * ROWS_PER_PASS + lane / LANES_PER_ROW, ch = lane % LANES_PER_ROW;
            // non-temporal: the output is not read again by this launch, and a workgroup cannot retire
            // before its stores are acknowledged
            __builtin_nontemporal_store(vdat[p], reinterpret_cast<u32x4*>(Cw + (int64_t)row * g.ldc + ch * 8));
        }
    };
    auto finish = [&](auto epi_tag) __attribute__((always_inline)) {
        convert_and_stage(epi_tag);
        store_staged();
    };
    // Each product has its own epilogue kinds, so each layout pair compiles only those.
    if (LA == KC && LB == MC) {  // forward
        switch (g.epilogue) {
            case EPI_NONE: finish(IC<EPI_NONE>{}); return;
            case EPI_BIAS: finish(IC<EPI_BIAS>{}); return;
            case EPI_BIAS_GELU_TANH: finish(IC<EPI_BIAS_GELU_TANH>{}); return;
            default: finish(IC<EPI_BIAS_GELU_ERF>{}); return;
        }
    } else if (LA == KC && LB == KC) {  // dgrad
        switch (g.epilogue) {
            case EPI_NONE: finish(IC<EPI_NONE>{}); return;
            case EPI_MUL_DGELU_TANH: finish(IC<EPI_MUL_DGELU_TANH>{}); return;
            default: finish(IC<EPI_MUL_DGELU_ERF>{}); return;
        }
    } else {  // wgrad
        if (g.epilogue == EPI_ACC_F32) {
            // fp32 accumulation dW32 += acc, no rounding.  The wave's 64 fp32 columns are 256 bytes
            // per row: the sums are staged through the wave's LDS region (half the wave tile's rows
            // at a time, rows padded to 272 bytes) so that 16 lanes read, add and write back one
            // whole row segment with 16 bytes each; the old values are requested before the staging so
            // that their latency hides behind it.  (Straight from the MFMA register layout a row is
            // four separate 64-byte runs: measured 14-28 % over the bf16-output product.)
            float* Cf = reinterpret_cast<float*>(g.C) + (int64_t)wrow0 * g.ldc + wcol0;
            constexpr int F_STRIDE = C::WTN * 4 + 16;  // bytes per staged fp32 row
            constexpr int RP = C::WTM / 2;             // rows per pass
            constexpr int NI = RP / 4;                 // a wave instruction covers 4 rows
            static_assert(C::WTN == 64, "16 lanes x 16 bytes per fp32 row");
            static_assert(RP * F_STRIDE <= C::WTM * C::EPI_STRIDE, "fits the wave's staging region");
            const int frow = lane >> 4, fcol = (lane & 15) << 2;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f32x4 old[NI];
#pragma unroll
                for (int i = 0; i < NI; ++i)
                    old[i] = *reinterpret_cast<const f32x4*>(Cf + (int64_t)(h * RP + i * 4 + frow) * g.ldc + fcol);
#pragma unroll
                for (int a = 0; a < C::TM / 2; ++a)
#pragma unroll
                    for (int b = 0; b < C::TN; ++b)
                        *reinterpret_cast<f32x4*>(stage + (a * 16 + (lane & 15)) * F_STRIDE + (b * 16 + 4 * (lane >> 4)) * 4) =
                            acc[h * (C::TM / 2) + a][b];
                __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the region is private to the wave
                __builtin_amdgcn_wave_barrier();
                f32x4 sum[NI];
#pragma unroll
                for (int i = 0; i < NI; ++i)
                    sum[i] = *reinterpret_cast<const f32x4*>(stage + (i * 4 + frow) * F_STRIDE + fcol * 4);
#pragma unroll
                for (int i = 0; i < NI; ++i)
                    *reinterpret_cast<f32x4*>(Cf + (int64_t)(h * RP + i * 4 + frow) * g.ldc + fcol) = old[i] + sum[i];
                __builtin_amdgcn_wave_barrier();  // LDS operations of a wave complete in order: the next pass may overwrite
            }
            return;
        }
        finish(IC<EPI_NONE>{});
    }
}

using MixBigCfg = TileCfg<256, 256, 2, 4>;
using MixSmallCfg = TileCfg<256, 128, 4, 2>;
constexpr int MIX_LDS_BYTES = MixBigCfg::LDS_BYTES > MixSmallCfg::LDS_BYTES ? MixBigCfg::LDS_BYTES : MixSmallCfg::LDS_BYTES;

// One launch over both regions of a TileSched.
template <int LA, int LB>
__global__ void __launch_bounds__(TILE_THREADS, 1) gemm_mixed_kernel(GemmArgs g, TileSched sc) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int bid = blockIdx.x;
    start_stagger(bid, sc.stagger);
    int tm, tn;
    if (bid < sc.n_big) {
        tile_of_index(xcd_contiguous(bid, sc.n_big), sc.tiles_m, sc.big_cols, sc.group_m, tm, tn);
        gemm_tile_body<256, 256, 2, 4, LA, LB>(g, tm * 256, tn * 256, smem);
    } else {
        const int n_small = (int)gridDim.x - sc.n_big;
        tile_of_index(xcd_contiguous(bid - sc.n_big, n_small), sc.tiles_m, sc.small_cols, sc.group_m, tm, tn);
        gemm_tile_body<256, 128, 4, 2, LA, LB>(g, tm * 256, sc.big_cols * 256 + tn * 128, smem);
    }
}

// ---- grouped launch: the tiles of several independent products in one grid ----------------
// A product on its own often cannot fill the 256 CUs (a 1536x1536 output is 36 big tiles), and a
// chain of such launches pays a ramp-up and a tail each.  A group launch strings the tile lists of
// up to GROUP_MAX_PRODUCTS products together: the grid is cut into segments, a segment is all the
// tiles of one size of one product, and segments are ordered by decreasing tile cost so that the
// in-order workgroup dispatch approximates longest-processing-time-first scheduling.  One of the
// slots may instead hold a bias gradient, whose 64-column strips form one more (cheap, hence
// late) segment of memory-bound workgroups.
constexpr int GROUP_MAX_PRODUCTS = 12;
constexpr int GROUP_MAX_SEGMENTS = 2 * GROUP_MAX_PRODUCTS;

struct GroupSeg {
    int first_block;  // first workgroup id of the segment
    int n_blocks;
    int product;      // index into GroupArgs::g
    int kind;         // 2 * layout pair (0: KC/MC, 1: KC/KC, 2: MC/MC) + (1 if 256x128 tiles);
                      // GROUP_KIND_BIAS_GRAD: 64-column strips of a bias gradient
    int tiles_m;      // tile rows
    int cols;         // tile columns of this segment
    int col0;         // first output column of this segment
    int group_m;      // band height of the tile order
};

constexpr int GROUP_KIND_BIAS_GRAD = 6;
constexpr int GROUP_BIAS_COLS = 64;

struct GroupArgs {
    int n_seg;
    GroupSeg seg[GROUP_MAX_SEGMENTS];
    GemmArgs g[GROUP_MAX_PRODUCTS];
};

__global__ void __launch_bounds__(TILE_THREADS, 1) gemm_group_kernel(GroupArgs ga) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int bid = blockIdx.x;
    int si = 0;
    for (int i = 1; i < ga.n_seg; ++i)
        if (bid >= ga.seg[i].first_block) si = i;
    const GroupSeg sg = ga.seg[si];
    const GemmArgs g = ga.g[sg.product];
    if (sg.kind == GROUP_KIND_BIAS_GRAD) {
        // A bias gradient rides along: memory-bound strips that fill CUs the products leave idle
        // towards the end of the launch.  Its arguments travel in a GemmArgs: A = dY, C = db (fp32),
        // Mo = rows, No = columns, epilogue = accumulate flag.
        BiasGradArgs bg;
        bg.dY = g.A;
        bg.lddy = g.lda;
        bg.db = reinterpret_cast<float*>(g.C);
        bg.M = g.Mo;
        bg.Nl = g.No;
        bg.accumulate = g.epilogue;
        bias_grad_strip<GROUP_BIAS_COLS, TILE_THREADS>(bg, bid - sg.first_block, reinterpret_cast<float*>(smem));
        return;
    }
    int tm, tn;
    // workgroup ids with equal id % 8 share an XCD whatever the segment's first id is
    tile_of_index(xcd_contiguous(bid - sg.first_block, sg.n_blocks), sg.tiles_m, sg.cols, sg.group_m, tm, tn);
    switch (sg.kind) {
        case 0: gemm_tile_body<256, 256, 2, 4, KC, MC>(g, tm * 256, sg.col0 + tn * 256, smem); break;
        case 1: gemm_tile_body<256, 128, 4, 2, KC, MC>(g, tm * 256, sg.col0 + tn * 128, smem); break;
        case 2: gemm_tile_body<256, 256, 2, 4, KC, KC>(g, tm * 256, sg.col0 + tn * 256, smem); break;
        case 3: gemm_tile_body<256, 128, 4, 2, KC, KC>(g, tm * 256, sg.col0 + tn * 128, smem); break;
        case 4: gemm_tile_body<256, 256, 2, 4, MC, MC>(g, tm * 256, sg.col0 + tn * 256, smem); break;
        default: gemm_tile_body<256, 128, 4, 2, MC, MC>(g, tm * 256, sg.col0 + tn * 128, smem); break;
    }
}

}  // namespace axo
