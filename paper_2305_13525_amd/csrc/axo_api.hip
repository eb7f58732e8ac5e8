// C ABI of the shard-GEMM library: host-side validation, shard derivation, kernel selection and
// launch.  Every check runs before the first HIP call, so all statuses except AXO_ERR_HIP can be
// exercised on a machine without a GPU.
#include "../../include/axo.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <deque>
#include <functional>
#include <map>
#include <mutex>
#include <new>
#include <queue>
#include <utility>
#include <vector>

#include "axo_common.hpp"
#include "bias_grad.hpp"
#include "gemm_generic.hpp"
#include "gemm_tile.hpp"

// Scratch memory of the allocation-free entry point (axo_bias_grad_static): arrival counters and
// slice sums of the split bias gradient, laid out as BiasSplit says.  One copy per GPU, held from
// the moment the library is loaded on it until the process ends; zero-initialised by the loader,
// and every call leaves the counters at zero.  In host code this name only stands for the symbol:
// the device address comes from hipGetSymbolAddress (static_scratch() below), per device.
constexpr size_t STATIC_SCRATCH_BYTES = 256 * 1024;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

using axo::GemmArgs;

struct Shard {
    int64_t M, Kl, Nl, row0, k0, n0;
    int k_coord;  // coordinate along the axis that splits K
};

int derive_shard(const axo_problem_t* p, Shard* s) {
    if (!p) return AXO_ERR_NULL_PTR;
    if (p->reserved != 0 || (p->transposed != 0 && p->transposed != 1)) return AXO_ERR_BAD_ARG;
    if (p->Gx < 1 || p->Gy < 1 || p->Gz < 1) return AXO_ERR_BAD_GRID;
    if (p->ix < 0 || p->ix >= p->Gx || p->iy < 0 || p->iy >= p->Gy || p->iz < 0 || p->iz >= p->Gz)
        return AXO_ERR_BAD_COORD;
    if (p->T < 0 || p->K < 0 || p->N < 0) return AXO_ERR_BAD_SIZE;
    // Section 3.2: I is cut over the token axis (Z) and the reduction axis, W over the reduction
    // axis and the output axis.  transposed swaps which of X / Y plays which role.
    const int gk = p->transposed ? p->Gy : p->Gx, ik = p->transposed ? p->iy : p->ix;
    const int gn = p->transposed ? p->Gx : p->Gy, in = p->transposed ? p->ix : p->iy;
    if (p->T % p->Gz != 0 || p->K % gk != 0 || p->N % gn != 0) return AXO_ERR_INDIVISIBLE;
    s->M = p->T / p->Gz;
    s->Kl = p->K / gk;
    s->Nl = p->N / gn;
    if (s->M > INT32_MAX || s->Kl > INT32_MAX || s->Nl > INT32_MAX) return AXO_ERR_BAD_SIZE;
    s->row0 = s->M * p->iz;
    s->k0 = s->Kl * ik;
    s->n0 = s->Nl * in;
    s->k_coord = ik;
    return AXO_OK;
}

bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

// One matrix argument: pointer, leading dimension, row length.  A matrix without elements is
// never dereferenced, so nothing about it is checked.
int check_matrix(const void* ptr, int64_t ld, int64_t rows, int64_t row_len) {
    if (rows == 0 || row_len == 0) return AXO_OK;
    if (!ptr) return AXO_ERR_NULL_PTR;
    if (ld < row_len) return AXO_ERR_BAD_LD;
    if (!aligned16(ptr) || (ld % 8) != 0) return AXO_ERR_MISALIGNED;
    return AXO_OK;
}

int launch_generic(const GemmArgs& g, int la, int lb, hipStream_t st) {
    dim3 grid((g.No + axo::GEN_BN - 1) / axo::GEN_BN, (g.Mo + axo::GEN_BM - 1) / axo::GEN_BM, 1);
    dim3 block(256, 1, 1);
    if (grid.y > 65535u) return AXO_ERR_BAD_SIZE;
    if (la == axo::KC && lb == axo::MC)
        hipLaunchKernelGGL((axo::gemm_generic_kernel<axo::KC, axo::MC>), grid, block, 0, st, g);
    else if (la == axo::KC && lb == axo::KC)
        hipLaunchKernelGGL((axo::gemm_generic_kernel<axo::KC, axo::KC>), grid, block, 0, st, g);
    else
        hipLaunchKernelGGL((axo::gemm_generic_kernel<axo::MC, axo::MC>), grid, block, 0, st, g);
    return hipGetLastError() == hipSuccess ? AXO_OK : AXO_ERR_HIP;
}

// The tuned kernel covers the output with 256x256 tiles and, to balance tile counts that do not
// fill the last round of CUs, a region of 256x128 tiles.  The CU count is a design constant
// (MI355X: 256 CUs) so that planning needs no device.
constexpr int NUM_CU = 256;
// relative cost of a half-width tile (half the flops at lower efficiency: more operand traffic
// per flop), in units of one big tile; measured on MI355X
constexpr double SMALL_TILE_COST = 0.60;

// The tuned kernel addresses an operand tile through a buffer descriptor with 32-bit byte offsets:
// the span a workgroup walks (256 rows of a KC operand, or the whole reduction of an MC operand)
// has to stay below 4 GiB.
bool span_ok(int layout, int64_t ld, int64_t R) {
    const int64_t elems = layout == axo::KC ? 256 * ld + R : R * ld + 256;
    return elems * 2 < (int64_t)0xFFFF0000;
}

// Reductions: any length where both operands have the reduction index as their row index (wgrad:
// rows beyond the end read as zeros through the buffer bound); any multiple of 8 otherwise (an
// operand with the reduction inside its rows has its last fragments masked in registers, which
// needs whole 16-byte fragments).  The kernel walks the length rounded up to 128.
bool tileable(const GemmArgs& g, int la, int lb) {
    const bool any_reduction = la == axo::MC && lb == axo::MC;
    if (!(g.R > 0 && (any_reduction || g.R % 8 == 0) && g.Mo > 0 && g.No > 0 && g.Mo % 256 == 0 &&
          g.No % 128 == 0))
        return false;
    // the span is that of the rows the kernel walks: the reduction rounded up to the unrolled loop's
    // 128 (the surplus rows of wgrad read as zeros, but their offsets are still formed in 32 bits)
    const int64_t walked = ((int64_t)g.R + 2 * axo::TILE_BK - 1) / (2 * axo::TILE_BK) * (2 * axo::TILE_BK);
    return span_ok(la, g.lda, walked) && span_ok(lb, g.ldb, walked);
}

// Time (in big-tile units) a greedy dispatch of n_big big tiles followed by n_small small tiles
// takes on NUM_CU CUs: workgroups are handed out in order to whichever CU is free first.
double makespan(int n_big, int n_small) {
    std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
    for (int i = 0; i < NUM_CU; ++i) free_at.push(0.0);
    double end = 0.0;
    auto run = [&](int n, double cost) {
        for (int i = 0; i < n; ++i) {
            const double t = free_at.top() + cost;
            free_at.pop();
            free_at.push(t);
            if (t > end) end = t;
        }
    };
    run(n_big, 1.0);
    run(n_small, SMALL_TILE_COST);
    return end;
}

// Start-up phase shift of a single-product launch (see start_stagger): 8 phases 1920 cycles
// apart, once the launch has a workgroup for every CU (a smaller one has no chip-wide burst).
int stagger_units(int blocks) { return blocks >= NUM_CU ? 3 : 0; }

// Choose how many 256-wide tile columns to use; the remaining columns become 128-wide tiles.
// Plans are cached per output shape (the search simulates the dispatch).
axo::TileSched plan_tiles(int Mo, int No) {
    static std::mutex mu;
    static std::map<std::pair<int, int>, axo::TileSched> cache;
    std::lock_guard<std::mutex> lock(mu);
    auto it = cache.find({Mo, No});
    if (it != cache.end()) return it->second;
    axo::TileSched sc{};
    sc.tiles_m = Mo / 256;
    const int max_big_cols = No / 256;
    int best_cols = max_big_cols;
    double best = 1e30;
    for (int cb = max_big_cols; cb >= 0; --cb) {
        const int small_cols = (No - cb * 256) / 128;
        const double t = makespan(sc.tiles_m * cb, sc.tiles_m * small_cols);
        if (t < best - 1e-9) {
            best = t;
            best_cols = cb;
        }
    }
    sc.big_cols = best_cols;
    sc.small_cols = (No - best_cols * 256) / 128;
    sc.n_big = sc.tiles_m * sc.big_cols;
    sc.group_m = sc.tiles_m < 4 ? sc.tiles_m : 4;
    sc.stagger = stagger_units(sc.n_big + sc.tiles_m * sc.small_cols);
    if (cache.size() < 4096) cache[{Mo, No}] = sc;
    return sc;
}

// The tuned kernels' dynamic LDS size is above the default limit, so the limit is raised once per
// kernel and device (`raised` holds one bit per device ordinal; a process rarely sees more than
// 8, and beyond 64 the attribute is simply set on every launch).
bool raise_lds_limit(const void* kernel, std::atomic<uint64_t>* raised) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t)1 << dev : 0;
    if (bit && (raised->load(std::memory_order_acquire) & bit)) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, axo::MIX_LDS_BYTES) != hipSuccess)
        return false;
    raised->fetch_or(bit, std::memory_order_release);
    return true;
}

// Launch of one tuned-kernel instantiation.
template <int LA, int LB>
int launch_tile(const GemmArgs& g, hipStream_t st) {
    auto kern = axo::gemm_mixed_kernel<LA, LB>;
    static std::atomic<uint64_t> raised{0};
    if (!raise_lds_limit(reinterpret_cast<const void*>(kern), &raised)) return AXO_ERR_HIP;
    const axo::TileSched sc = plan_tiles(g.Mo, g.No);
    const int blocks = sc.n_big + sc.tiles_m * sc.small_cols;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(axo::TILE_THREADS), axo::MIX_LDS_BYTES, st, g, sc);
    return hipGetLastError() == hipSuccess ? AXO_OK : AXO_ERR_HIP;
}

int launch_tile_layout(const GemmArgs& g, int la, int lb, hipStream_t st) {
    if (la == axo::KC && lb == axo::MC) return launch_tile<axo::KC, axo::MC>(g, st);
    if (la == axo::KC && lb == axo::KC) return launch_tile<axo::KC, axo::KC>(g, st);
    return launch_tile<axo::MC, axo::MC>(g, st);
}

// ---- grouped launch ------------------------------------------------------------------------
// Cost of one tile in reduction steps of a big tile: the steps themselves plus a fixed share for
// the tile's first loads and its epilogue (measured: a two-step tile takes about as long as six
// steps of a long one).
constexpr double TILE_OVERHEAD_STEPS = 4.0;
double tile_cost(int R, bool small) {
    return (R / (double)axo::TILE_BK + TILE_OVERHEAD_STEPS) * (small ? SMALL_TILE_COST : 1.0);
}

int layout_pair(int la, int lb) { return (la == axo::KC && lb == axo::MC) ? 0 : (la == axo::KC ? 1 : 2); }

struct GroupItem {
    int Mo, No, R, pair;
    bool operator<(const GroupItem& o) const {
        if (Mo != o.Mo) return Mo < o.Mo;
        if (No != o.No) return No < o.No;
        if (R != o.R) return R < o.R;
        return pair < o.pair;
    }
};

struct SegCost {
    double cost;
    int count, item, small;
};

// A bias gradient inside a grouped launch (GroupItem::pair == PAIR_BIAS_GRAD, Mo = rows, No =
// columns): strips of 64 columns, each a workgroup that streams Mo rows of 128 bytes.  A strip
// is bound by memory latency, not bandwidth: measured 19 us for 4096 rows, which is what 15
// reduction steps of a big tile take.
constexpr int PAIR_BIAS_GRAD = 3;
double bias_strip_cost(int rows) { return 1.0 + 15.0 * rows / 4096.0; }
int bias_strips(int cols) { return (cols + axo::GROUP_BIAS_COLS - 1) / axo::GROUP_BIAS_COLS; }
// The standalone launch picks its strip width by shape; only shapes for which it picks the
// grouped launch's 64 columns may ride along, so that both give the same bits.
bool bias_grad_groupable(const axo::BiasGradArgs& g) { return g.Nl > 0 && bias_strips(g.Nl) >= NUM_CU / 4; }

// segments of a group for a choice of big_cols per item, most expensive tiles first
std::vector<SegCost> group_segments(const std::vector<GroupItem>& items, const std::vector<int>& big_cols) {
    std::vector<SegCost> segs;
    for (size_t i = 0; i < items.size(); ++i) {
        if (items[i].pair == PAIR_BIAS_GRAD) {
            segs.push_back({bias_strip_cost(items[i].Mo), bias_strips(items[i].No), (int)i, 0});
            continue;
        }
        const int tiles_m = items[i].Mo / 256, cb = big_cols[i], cs = (items[i].No - cb * 256) / 128;
        if (cb > 0) segs.push_back({tile_cost(items[i].R, false), tiles_m * cb, (int)i, 0});
        if (cs > 0) segs.push_back({tile_cost(items[i].R, true), tiles_m * cs, (int)i, 1});
    }
    std::stable_sort(segs.begin(), segs.end(), [](const SegCost& a, const SegCost& b) { return a.cost > b.cost; });
    return segs;
}

double group_makespan(const std::vector<SegCost>& segs) {
    std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
    for (int i = 0; i < NUM_CU; ++i) free_at.push(0.0);
    double end = 0.0;
    for (const SegCost& sg : segs)
        for (int i = 0; i < sg.count; ++i) {
            const double t = free_at.top() + sg.cost;
            free_at.pop();
            free_at.push(t);
            if (t > end) end = t;
        }
    return end;
}

// big_cols per item that minimise the simulated makespan of the whole group: coordinate descent
// from "all big tiles", two sweeps.  Cached per list of shapes.
std::vector<int> plan_group(const std::vector<GroupItem>& items) {
    static std::mutex mu;
    static std::map<std::vector<GroupItem>, std::vector<int>> cache;
    std::lock_guard<std::mutex> lock(mu);
    auto it = cache.find(items);
    if (it != cache.end()) return it->second;
    std::vector<int> cols(items.size());
    for (size_t i = 0; i < items.size(); ++i) cols[i] = items[i].pair == PAIR_BIAS_GRAD ? 0 : items[i].No / 256;
    double best = group_makespan(group_segments(items, cols));
    for (int sweep = 0; sweep < 2; ++sweep)
        for (size_t i = 0; i < items.size(); ++i) {
            if (items[i].pair == PAIR_BIAS_GRAD) continue;
            const int max_cols = items[i].No / 256;
            const int stride = max_cols > 16 ? (max_cols + 15) / 16 : 1;
            int best_c = cols[i];
            for (int c = max_cols; c >= 0; c -= stride) {
                cols[i] = c;
                const double t = group_makespan(group_segments(items, cols));
                if (t < best - 1e-9) {
                    best = t;
                    best_c = c;
                }
            }
            cols[i] = best_c;
        }
    if (cache.size() < 1024) cache[items] = cols;
    return cols;
}

int check_workspace(const axo_problem_t* p, int op, const void* ws, size_t ws_bytes) {
    const size_t need = axo_workspace_bytes(p, op);
    if (need == 0) return AXO_OK;
    if (!ws || ws_bytes < need) return AXO_ERR_WORKSPACE;
    if (!aligned16(ws)) return AXO_ERR_MISALIGNED;
    return AXO_OK;
}

// Validated, launch-ready description of one unit of work of a chain: a product (the usual
// case) or a bias gradient.
struct Plan {
    GemmArgs g{};
    int la = 0, lb = 0;
    bool bias_grad = false;   // bg is valid instead of g
    axo::BiasGradArgs bg{};
    bool nothing_to_do() const { return bias_grad ? bg.Nl == 0 : (g.Mo == 0 || g.No == 0); }
};

// One launch over the tiles of all given products (each tileable and non-empty, at most
// GROUP_MAX_PRODUCTS of them).
int launch_group(const Plan* const* plans, int n, hipStream_t st) {
    static std::atomic<uint64_t> raised{0};
    if (!raise_lds_limit(reinterpret_cast<const void*>(axo::gemm_group_kernel), &raised)) return AXO_ERR_HIP;
    std::vector<GroupItem> items(n);
    for (int i = 0; i < n; ++i)
        items[i] = plans[i]->bias_grad ? GroupItem{plans[i]->bg.M, plans[i]->bg.Nl, 0, PAIR_BIAS_GRAD}
                                       : GroupItem{plans[i]->g.Mo, plans[i]->g.No, plans[i]->g.R,
                                                   layout_pair(plans[i]->la, plans[i]->lb)};
    const std::vector<int> cols = plan_group(items);
    const std::vector<SegCost> segs = group_segments(items, cols);
    axo::GroupArgs ga{};
    ga.n_seg = (int)segs.size();
    int blocks = 0;
    for (int k = 0; k < ga.n_seg; ++k) {
        const SegCost& sc = segs[k];
        axo::GroupSeg& sg = ga.seg[k];
        sg.first_block = blocks;
        sg.n_blocks = sc.count;
        sg.product = sc.item;
        if (items[sc.item].pair == PAIR_BIAS_GRAD) {
            sg.kind = axo::GROUP_KIND_BIAS_GRAD;
            sg.tiles_m = 1;
            sg.cols = sc.count;
            sg.col0 = 0;
            sg.group_m = 1;
        } else {
            sg.kind = 2 * items[sc.item].pair + sc.small;
            sg.tiles_m = items[sc.item].Mo / 256;
            sg.cols = sc.count / sg.tiles_m;
            sg.col0 = sc.small ? cols[sc.item] * 256 : 0;
            sg.group_m = sg.tiles_m < 4 ? sg.tiles_m : 4;
        }
        blocks += sc.count;
    }
    for (int i = 0; i < n; ++i) {
        if (!plans[i]->bias_grad) {
            ga.g[i] = plans[i]->g;
            continue;
        }
        GemmArgs b{};  // the bias gradient's arguments in a GemmArgs, as gemm_group_kernel reads them
        b.A = plans[i]->bg.dY;
        b.lda = plans[i]->bg.lddy;
        b.C = reinterpret_cast<axo::bf16_t*>(plans[i]->bg.db);
        b.Mo = plans[i]->bg.M;
        b.No = plans[i]->bg.Nl;
        b.epilogue = plans[i]->bg.accumulate;
        ga.g[i] = b;
    }
    hipLaunchKernelGGL(axo::gemm_group_kernel, dim3(blocks), dim3(axo::TILE_THREADS), axo::MIX_LDS_BYTES, st, ga);
    return hipGetLastError() == hipSuccess ? AXO_OK : AXO_ERR_HIP;
}

// The product restricted to output rows [r0, r0 + rows) and columns [c0, c0 + cols): the same
// operands and output addressed through offset pointers, same leading dimensions.
GemmArgs sub_product(const GemmArgs& g, int la, int lb, int r0, int rows, int c0, int cols) {
    GemmArgs s = g;
    s.A = la == axo::KC ? g.A + (int64_t)r0 * g.lda : g.A + r0;   // KC: row i of A; MC: column i of A
    s.B = lb == axo::KC ? g.B + (int64_t)c0 * g.ldb : g.B + c0;
    if (g.epilogue == axo::EPI_ACC_F32)                           // C counts fp32 elements
        s.C = reinterpret_cast<axo::bf16_t*>(reinterpret_cast<float*>(g.C) + (int64_t)r0 * g.ldc + c0);
    else
        s.C = g.C + (int64_t)r0 * g.ldc + c0;
    if (g.bias) s.bias = g.bias + c0;
    if (g.aux) s.aux = g.aux + (int64_t)r0 * g.ldaux + c0;
    s.Mo = rows;
    s.No = cols;
    return s;
}

// A product whose reduction fits the tuned kernel but whose output misses its granularity (256
// rows, 128 columns) can still be covered with whole tiles: the interior, plus a band of the last
// 256 rows and a band of the last 128 columns that reach back over the interior.  Where bands and
// interior overlap an element is computed twice, by the same instructions in the same order (its
// value does not depend on the tile it falls in), so the second store rewrites the same bits.
// Conditions: the shifted origins must keep the 16-byte alignment of the loads and stores, i.e.
// No % 8 == 0 and, where the output row index is the contiguous one of operand A (wgrad),
// Mo % 8 == 0; and the epilogue must be a pure function of the sum (not the fp32 accumulation,
// which would add twice).  On success `out` receives 2 to 4 tileable pieces.
bool cover_with_tiles(const Plan& pl, std::vector<Plan>* out) {
    const GemmArgs& g = pl.g;
    if (g.epilogue == axo::EPI_ACC_F32 || g.Mo < 256 || g.No < 128 || g.No % 8 != 0) return false;
    if (pl.la == axo::MC && g.Mo % 8 != 0) return false;
    const int Mi = g.Mo / 256 * 256, Ni = g.No / 128 * 128;
    int rows[2][2] = {{0, Mi}, {g.Mo - 256, 256}}, cols[2][2] = {{0, Ni}, {g.No - 128, 128}};
    const int nr = g.Mo > Mi ? 2 : 1, nc = g.No > Ni ? 2 : 1;
    out->clear();
    for (int a = 0; a < nr; ++a)
        for (int b = 0; b < nc; ++b) {
            Plan piece = pl;
            piece.g = sub_product(g, pl.la, pl.lb, rows[a][0], rows[a][1], cols[b][0], cols[b][1]);
            if (!tileable(piece.g, pl.la, pl.lb)) return false;
            out->push_back(piece);
        }
    return out->size() > 1;
}

// One product: the tuned kernel when it takes the shape; a cover of whole tiles in one grouped
// launch when only the output's granularity is in the way (measured on 4096 x 2048 x 6152, eight
// columns over: 198 TFLOP/s through the general kernel alone); failing that, the interior on the
// tuned kernel and the leftover strips on the general one; the general kernel for the rest.
int route_of(const GemmArgs& g, int la, int lb, std::vector<Plan>* pieces) {
    if (g.Mo == 0 || g.No == 0) return AXO_ROUTE_NONE;
    if (tileable(g, la, lb)) return AXO_ROUTE_TILED;
    Plan whole;
    whole.g = g;
    whole.la = la;
    whole.lb = lb;
    if (cover_with_tiles(whole, pieces)) return AXO_ROUTE_COVERED;
    const int Mi = g.Mo / 256 * 256, Ni = g.No / 128 * 128;
    // block offsets that are multiples of 256 rows and 128 columns keep every alignment
    if (Mi > 0 && Ni > 0 && tileable(sub_product(g, la, lb, 0, Mi, 0, Ni), la, lb)) return AXO_ROUTE_INTERIOR_STRIPS;
    return AXO_ROUTE_GENERAL;
}

int launch(const GemmArgs& g, int la, int lb, hipStream_t st) {
    std::vector<Plan> pieces;
    switch (route_of(g, la, lb, &pieces)) {
        case AXO_ROUTE_NONE: return AXO_OK;
        case AXO_ROUTE_TILED: return launch_tile_layout(g, la, lb, st);
        case AXO_ROUTE_COVERED: {
            const Plan* ptr[4];
            for (size_t i = 0; i < pieces.size(); ++i) ptr[i] = &pieces[i];
            return launch_group(ptr, (int)pieces.size(), st);
        }
        case AXO_ROUTE_INTERIOR_STRIPS: {
            const int Mi = g.Mo / 256 * 256, Ni = g.No / 128 * 128;
            int rc = launch_tile_layout(sub_product(g, la, lb, 0, Mi, 0, Ni), la, lb, st);
            if (rc == AXO_OK && g.No > Ni) rc = launch_generic(sub_product(g, la, lb, 0, g.Mo, Ni, g.No - Ni), la, lb, st);
            if (rc == AXO_OK && g.Mo > Mi) rc = launch_generic(sub_product(g, la, lb, Mi, g.Mo - Mi, 0, Ni), la, lb, st);
            return rc;
        }
        default: return launch_generic(g, la, lb, st);
    }
}

int check_no_alias(const Plan& pl);  // defined with the byte-range code below

int plan_fwd(const axo_problem_t* p, const void* X, int64_t ldx, const void* W, int64_t ldw, const void* bias,
             int epilogue, void* Y, int64_t ldy, void* ws, size_t ws_bytes, Plan* out) {
    Shard s;
    int rc = derive_shard(p, &s);
    if (rc) return rc;
    if (epilogue < AXO_EPI_NONE || epilogue > AXO_EPI_BIAS_GELU_ERF) return AXO_ERR_BAD_EPILOGUE;
    if (epilogue != AXO_EPI_NONE && !bias) return AXO_ERR_BAD_EPILOGUE;
    if ((rc = check_matrix(X, ldx, s.M, s.Kl))) return rc;
    if ((rc = check_matrix(W, ldw, s.Kl, s.Nl))) return rc;
    if ((rc = check_matrix(Y, ldy, s.M, s.Nl))) return rc;
    if (epilogue != AXO_EPI_NONE && !aligned16(bias)) return AXO_ERR_MISALIGNED;
    if ((rc = check_workspace(p, AXO_OP_FWD, ws, ws_bytes))) return rc;
    GemmArgs& g = out->g;
    g.A = static_cast<const axo::bf16_t*>(X); g.lda = ldx;
    g.B = static_cast<const axo::bf16_t*>(W); g.ldb = ldw;
    g.C = static_cast<axo::bf16_t*>(Y); g.ldc = ldy;
    g.bias = static_cast<const axo::bf16_t*>(bias);
    g.aux = nullptr; g.ldaux = 0;
    g.Mo = (int)s.M; g.No = (int)s.Nl; g.R = (int)s.Kl;
    g.epilogue = epilogue;
    g.add_bias = (epilogue != AXO_EPI_NONE && s.k_coord == 0) ? 1 : 0;
    out->la = axo::KC; out->lb = axo::MC;
    return check_no_alias(*out);
}

int plan_dgrad(const axo_problem_t* p, const void* dY, int64_t lddy, const void* W, int64_t ldw, void* dX,
               int64_t lddx, void* ws, size_t ws_bytes, Plan* out) {
    Shard s;
    int rc = derive_shard(p, &s);
    if (rc) return rc;
    if ((rc = check_matrix(dY, lddy, s.M, s.Nl))) return rc;
    if ((rc = check_matrix(W, ldw, s.Kl, s.Nl))) return rc;
    if ((rc = check_matrix(dX, lddx, s.M, s.Kl))) return rc;
    if ((rc = check_workspace(p, AXO_OP_DGRAD, ws, ws_bytes))) return rc;
    GemmArgs& g = out->g;
    g.A = static_cast<const axo::bf16_t*>(dY); g.lda = lddy;
    g.B = static_cast<const axo::bf16_t*>(W); g.ldb = ldw;
    g.C = static_cast<axo::bf16_t*>(dX); g.ldc = lddx;
    g.bias = nullptr;
    g.aux = nullptr; g.ldaux = 0;
    g.Mo = (int)s.M; g.No = (int)s.Kl; g.R = (int)s.Nl;
    g.epilogue = AXO_EPI_NONE; g.add_bias = 0;
    out->la = axo::KC; out->lb = axo::KC;
    return check_no_alias(*out);
}

int plan_wgrad(const axo_problem_t* p, const void* X, int64_t ldx, const void* dY, int64_t lddy, void* dW,
               int64_t lddw, void* ws, size_t ws_bytes, Plan* out) {
    Shard s;
    int rc = derive_shard(p, &s);
    if (rc) return rc;
    if ((rc = check_matrix(X, ldx, s.M, s.Kl))) return rc;
    if ((rc = check_matrix(dY, lddy, s.M, s.Nl))) return rc;
    if ((rc = check_matrix(dW, lddw, s.Kl, s.Nl))) return rc;
    if ((rc = check_workspace(p, AXO_OP_WGRAD, ws, ws_bytes))) return rc;
    GemmArgs& g = out->g;
    g.A = static_cast<const axo::bf16_t*>(X); g.lda = ldx;
    g.B = static_cast<const axo::bf16_t*>(dY); g.ldb = lddy;
    g.C = static_cast<axo::bf16_t*>(dW); g.ldc = lddw;
    g.bias = nullptr;
    g.aux = nullptr; g.ldaux = 0;
    g.Mo = (int)s.Kl; g.No = (int)s.Nl; g.R = (int)s.M;
    g.epilogue = AXO_EPI_NONE; g.add_bias = 0;
    out->la = axo::MC; out->lb = axo::MC;
    return check_no_alias(*out);
}

int plan_bias_grad(const axo_problem_t* p, const void* dY, int64_t lddy, float* db, int accumulate, Plan* out) {
    Shard s;
    int rc = derive_shard(p, &s);
    if (rc) return rc;
    if (accumulate != 0 && accumulate != 1) return AXO_ERR_BAD_ARG;
    if ((rc = check_matrix(dY, lddy, s.M, s.Nl))) return rc;
    out->bias_grad = true;
    out->bg.dY = static_cast<const axo::bf16_t*>(dY);
    out->bg.lddy = lddy;
    out->bg.db = db;
    out->bg.M = (int)s.M;
    out->bg.Nl = (int)s.Nl;
    out->bg.accumulate = accumulate;
    if (s.Nl == 0) return AXO_OK;
    if (!db) return AXO_ERR_NULL_PTR;
    if (reinterpret_cast<uintptr_t>(db) & 3u) return AXO_ERR_MISALIGNED;
    return check_no_alias(*out);
}

int launch_bias_grad(const axo::BiasGradArgs& g, hipStream_t st) {
    if (g.Nl == 0) return AXO_OK;
    auto blocks = [&](int cols) { return (unsigned)((g.Nl + cols - 1) / cols); };
    // the widest column block that still gives a quarter (an eighth) of the CUs a workgroup
    if (blocks(64) >= (unsigned)NUM_CU / 4)
        hipLaunchKernelGGL(axo::bias_grad_kernel<64>, dim3(blocks(64)), dim3(axo::BG_THREADS), 0, st, g);
    else if (blocks(32) >= (unsigned)NUM_CU / 8)
        hipLaunchKernelGGL(axo::bias_grad_kernel<32>, dim3(blocks(32)), dim3(axo::BG_THREADS), 0, st, g);
    else
        hipLaunchKernelGGL(axo::bias_grad_kernel<16>, dim3(blocks(16)), dim3(axo::BG_THREADS), 0, st, g);
    return hipGetLastError() == hipSuccess ? AXO_OK : AXO_ERR_HIP;
}

// ---- bias gradient with the rows split over workgroups (needs scratch memory) ----------------
// How a shape is cut: 64-column strips, each cut into S row slices of a multiple of 64 rows so that
// about BIAS_SPLIT_WORKGROUPS workgroups are in flight, no slice below 128 rows.  A function of the
// shape alone, so the summation order (and with it every bit of the result) is too.  Measured on
// 4096 rows (time per call in a loop, launch included; 6144 / 16384 / 1536 columns): 128
// workgroups 14.6 / 25.0 / 9.0 us, 256: 12.6 / 22.0 / 8.4, 384: 11.6 / 22.4 / 10.5, 512: 11.6 / 22.2 /
// 10.6, 1024: 15.2 / 27.4 / 17.1 (every slice costs a publication and a share of the final
// addition); the strips of axo_bias_grad: 15.6 / 24.6 / 14.7.
constexpr int BIAS_SPLIT_WORKGROUPS = 384;
struct BiasSplit {
    int strips, S, rows_per_slice;
    size_t counter_bytes, partial_bytes;  // scratch layout: [counters][partial sums]
    size_t bytes() const { return S > 1 ? counter_bytes + partial_bytes : 0; }
};
BiasSplit plan_bias_split(int64_t M, int64_t Nl) {
    BiasSplit b{};
    b.strips = (int)((Nl + axo::BGS_COLS - 1) / axo::BGS_COLS);
    b.S = 1;
    b.rows_per_slice = (int)((M + axo::BGS_ROW_LANES - 1) / axo::BGS_ROW_LANES * axo::BGS_ROW_LANES);
    if (b.strips > 0 && M > 0) {
        int64_t want = (BIAS_SPLIT_WORKGROUPS + b.strips / 2) / b.strips;
        want = std::min<int64_t>(std::min<int64_t>(want, axo::BGS_MAX_SPLIT), M / 128);
        if (want > 1) {
            const int64_t rows = ((M + want - 1) / want + axo::BGS_ROW_LANES - 1) / axo::BGS_ROW_LANES * axo::BGS_ROW_LANES;
            b.rows_per_slice = (int)rows;
            b.S = (int)((M + rows - 1) / rows);
        }
    }
    b.counter_bytes = ((size_t)b.strips * sizeof(uint32_t) + 255) / 256 * 256;
    b.partial_bytes = (size_t)b.S * (size_t)Nl * sizeof(float);
    return b;
}

// Enqueues the split kernel on scratch memory laid out as BiasSplit says (ignored when S == 1).
int launch_bias_grad_split(const axo::BiasGradArgs& g, const BiasSplit& b, void* scratch, hipStream_t st) {
    if (g.Nl == 0) return AXO_OK;
    axo::BiasGradSplitArgs a{};
    a.dY = g.dY;
    a.lddy = g.lddy;
    a.db = g.db;
    a.M = g.M;
    a.Nl = g.Nl;
    a.accumulate = g.accumulate;
    a.S = b.S;
    a.rows_per_slice = b.rows_per_slice;
    a.counters = static_cast<uint32_t*>(scratch);
    a.partial = reinterpret_cast<float*>(static_cast<char*>(scratch) + b.counter_bytes);
    hipLaunchKernelGGL(axo::bias_grad_split_kernel, dim3((unsigned)b.strips * (unsigned)b.S), dim3(axo::BGS_THREADS), 0, st, a);
    return hipGetLastError() == hipSuccess ? AXO_OK : AXO_ERR_HIP;
}

// Device address of this GPU's copy of `scratch`: asked for once per device, with that device
// current, and kept (each GPU holds its own copy at its own address).  No allocation.
int static_scratch(void** out) {
    static std::atomic<void*> known[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return AXO_ERR_HIP;
    const bool slot = dev >= 0 && dev < 64;
    if (slot) {
        if (void* p = known[dev].load(std::memory_order_acquire)) {
            *out = p;
            return AXO_OK;
        }
    }
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return AXO_ERR_HIP;
    if (slot) known[dev].store(p, std::memory_order_release);
    *out = p;
    return AXO_OK;
}

// one unit of work on its own
int launch_plan(const Plan& pl, hipStream_t st) {
    return pl.bias_grad ? launch_bias_grad(pl.bg, st) : launch(pl.g, pl.la, pl.lb, st);
}

// Validates a chain and lists its products in the order of Section 4.1: forwards of layers
// 0..n-1, then for layers n-1..0 dgrad followed by wgrad.  Nothing is launched here, so a chain
// with a malformed product enqueues nothing.
int plan_chain(const axo_layer_t* layers, int n_layers, void* ws, size_t ws_bytes, std::vector<Plan>* out) {
    if (n_layers < 0) return AXO_ERR_BAD_ARG;
    if (n_layers == 0) return AXO_OK;
    if (!layers) return AXO_ERR_NULL_PTR;
    if (n_layers > 4096) return AXO_ERR_BAD_ARG;
    out->resize(3 * (size_t)n_layers);
    for (int i = 0; i < n_layers; ++i) {
        const axo_layer_t& L = layers[i];
        if (L.reserved != 0) return AXO_ERR_BAD_ARG;
        int rc = plan_fwd(&L.p, L.X, L.ldx, L.W, L.ldw, L.bias, L.epilogue, L.Y, L.ldy, ws, ws_bytes, &(*out)[i]);
        if (rc) return rc;
        const size_t b = (size_t)n_layers + 2 * (size_t)(n_layers - 1 - i);
        rc = plan_dgrad(&L.p, L.dY, L.lddy, L.W, L.ldw, L.dX, L.lddx, ws, ws_bytes, &(*out)[b]);
        if (rc) return rc;
        rc = plan_wgrad(&L.p, L.X, L.ldx, L.dY, L.lddy, L.dW, L.lddw, ws, ws_bytes, &(*out)[b + 1]);
        if (rc) return rc;
    }
    return AXO_OK;
}

// dgrad with the activation's derivative fused in (see axo_fc_dgrad_act)
int plan_dgrad_act(const axo_problem_t* p, const void* dY, int64_t lddy, const void* W, int64_t ldw, const void* pre,
                   int64_t ldpre, int act, void* dX, int64_t lddx, void* ws, size_t ws_bytes, Plan* out) {
    if (act != AXO_EPI_BIAS_GELU_TANH && act != AXO_EPI_BIAS_GELU_ERF) return AXO_ERR_BAD_EPILOGUE;
    int rc = plan_dgrad(p, dY, lddy, W, ldw, dX, lddx, ws, ws_bytes, out);
    if (rc) return rc;
    if ((rc = check_matrix(pre, ldpre, out->g.Mo, out->g.No))) return rc;
    out->g.aux = static_cast<const axo::bf16_t*>(pre);
    out->g.ldaux = ldpre;
    out->g.epilogue = act == AXO_EPI_BIAS_GELU_TANH ? axo::EPI_MUL_DGELU_TANH : axo::EPI_MUL_DGELU_ERF;
    return check_no_alias(*out);
}

// wgrad accumulated into an fp32 matrix (see axo_fc_wgrad_acc)
int plan_wgrad_acc(const axo_problem_t* p, const void* X, int64_t ldx, const void* dY, int64_t lddy, float* dW32,
                   int64_t lddw, void* ws, size_t ws_bytes, Plan* out) {
    Shard s;
    int rc = derive_shard(p, &s);
    if (rc) return rc;
    if (s.Kl > 0 && s.Nl > 0) {  // the fp32 output: 16-byte aligned rows of 4-byte elements
        if (!dW32) return AXO_ERR_NULL_PTR;
        if (lddw < s.Nl) return AXO_ERR_BAD_LD;
        if (!aligned16(dW32) || (lddw % 4) != 0) return AXO_ERR_MISALIGNED;
    }
    // the bf16 checks of the output do not apply; validate the inputs through plan_wgrad with a stand-in
    rc = plan_wgrad(p, X, ldx, dY, lddy, dW32, (lddw + 7) / 8 * 8, ws, ws_bytes, out);
    if (rc) return rc;
    out->g.C = reinterpret_cast<axo::bf16_t*>(dW32);
    out->g.ldc = lddw;
    out->g.epilogue = axo::EPI_ACC_F32;
    return check_no_alias(*out);
}

// The chain of axo_layer_step_ext: 3 or 4 units per layer, in program order.
int plan_chain_ext(const axo_layer_ext_t* layers, int n_layers, void* ws, size_t ws_bytes, std::vector<Plan>* out) {
    if (n_layers < 0) return AXO_ERR_BAD_ARG;
    if (n_layers == 0) return AXO_OK;
    if (!layers) return AXO_ERR_NULL_PTR;
    if (n_layers > 4096) return AXO_ERR_BAD_ARG;
    out->clear();
    out->resize((size_t)n_layers);  // the forwards; the backward units are appended in order
    for (int i = 0; i < n_layers; ++i) {
        const axo_layer_t& L = layers[i].layer;
        if (L.reserved != 0) return AXO_ERR_BAD_ARG;
        const int rc = plan_fwd(&L.p, L.X, L.ldx, L.W, L.ldw, L.bias, L.epilogue, L.Y, L.ldy, ws, ws_bytes, &(*out)[i]);
        if (rc) return rc;
    }
    for (int i = n_layers - 1; i >= 0; --i) {
        const axo_layer_ext_t& E = layers[i];
        const axo_layer_t& L = E.layer;
        if (E.accumulate_db != 0 && E.accumulate_db != 1) return AXO_ERR_BAD_ARG;
        Plan pl;
        int rc;
        if (E.pre) {
            rc = plan_dgrad_act(&L.p, L.dY, L.lddy, L.W, L.ldw, E.pre, E.ldpre, E.act_below, L.dX, L.lddx, ws, ws_bytes, &pl);
        } else {
            if (E.act_below != 0) return AXO_ERR_BAD_EPILOGUE;
            rc = plan_dgrad(&L.p, L.dY, L.lddy, L.W, L.ldw, L.dX, L.lddx, ws, ws_bytes, &pl);
        }
        if (rc) return rc;
        out->push_back(pl);
        pl = Plan();
        rc = E.dW32 ? plan_wgrad_acc(&L.p, L.X, L.ldx, L.dY, L.lddy, E.dW32, E.lddw32, ws, ws_bytes, &pl)
                    : plan_wgrad(&L.p, L.X, L.ldx, L.dY, L.lddy, L.dW, L.lddw, ws, ws_bytes, &pl);
        if (rc) return rc;
        out->push_back(pl);
        if (E.db) {
            pl = Plan();
            rc = plan_bias_grad(&L.p, L.dY, L.lddy, E.db, E.accumulate_db, &pl);
            if (rc) return rc;
            out->push_back(pl);
        }
    }
    return AXO_OK;
}

// ---- dependence analysis of a chain --------------------------------------------------------
// Byte range [lo, hi) that a matrix argument covers (rows x row_len elements of elem bytes, rows
// ld elements apart); empty matrices cover nothing.  The matrix itself is kept beside its range
// for the exact overlap test.
struct Range {
    uintptr_t lo, hi;
    int64_t pitch, rows, width;  // bytes between rows, row count, bytes per row
    bool overlaps(const Range& o) const { return lo < o.hi && o.lo < hi; }
    // Do the two matrices share a byte?  (Ranges that overlap need not: two column blocks of one
    // buffer interleave.)  Row r of this matrix covers [a, a + width) relative to the other's
    // base; row q of the other covers [q * pitch, q * pitch + width_o); they meet iff
    // q * pitch < a + width and q * pitch + width_o > a, an interval of q that is clamped to the
    // other's rows.  Only called when the ranges overlap, which no well-formed call makes them do.
    bool shares_bytes_with(const Range& o) const {
        if (!overlaps(o)) return false;
        auto floor_div = [](int64_t x, int64_t y) { return x / y - ((x % y != 0) && ((x < 0) != (y < 0)) ? 1 : 0); };
        const int64_t op = o.rows > 1 ? o.pitch : (int64_t)(o.hi - o.lo) + 1;  // one row: any positive pitch
        for (int64_t r = 0; r < rows; ++r) {
            const int64_t a = (int64_t)(lo - o.lo) + r * pitch;
            const int64_t q_hi = std::min<int64_t>(floor_div(a + width - 1, op), o.rows - 1);
            const int64_t q_lo = std::max<int64_t>(floor_div(a - o.width, op) + 1, 0);
            if (q_lo <= q_hi) return true;
        }
        return false;
    }
};
bool matrix_range(const void* ptr, int64_t ld, int64_t rows, int64_t row_len, int elem, Range* r) {
    if (!ptr || rows <= 0 || row_len <= 0) return false;
    r->lo = reinterpret_cast<uintptr_t>(ptr);
    r->hi = r->lo + (uintptr_t)(((rows - 1) * ld + row_len) * elem);
    r->pitch = ld * elem;
    r->rows = rows;
    r->width = row_len * elem;
    return true;
}
// What one product reads and writes.  (Ranges, not elements: two column blocks interleaved in one
// buffer count as overlapping, which only costs concurrency.)
struct Footprint {
    Range in[4];
    int n_in = 0;
    Range out{0, 0, 0, 0, 0};
    bool has_out = false;
    bool conflicts_with_later(const Footprint& later) const {
        if (has_out) {
            if (later.has_out && out.overlaps(later.out)) return true;                 // write after write
            for (int k = 0; k < later.n_in; ++k)
                if (out.overlaps(later.in[k])) return true;                            // read after write
        }
        if (later.has_out)
            for (int k = 0; k < n_in; ++k)
                if (in[k].overlaps(later.out)) return true;                            // write after read
        return false;
    }
    // the output shares bytes with one of the product's own inputs
    bool output_aliases_input() const {
        if (!has_out) return false;
        for (int k = 0; k < n_in; ++k)
            if (out.shares_bytes_with(in[k])) return true;
        return false;
    }
};
Footprint footprint(const Plan& pl) {
    const GemmArgs& g = pl.g;
    Footprint f;
    if (pl.nothing_to_do()) return f;  // nothing is launched for it
    Range r;
    if (pl.bias_grad) {  // reads dY, writes (or updates) db
        if (matrix_range(pl.bg.dY, pl.bg.lddy, pl.bg.M, pl.bg.Nl, 2, &r)) f.in[f.n_in++] = r;
        f.has_out = matrix_range(pl.bg.db, pl.bg.Nl, 1, pl.bg.Nl, 4, &f.out);
        return f;
    }
    // A(i, r): KC is Mo rows of R elements, MC is R rows of Mo elements; B likewise with No
    if (pl.la == axo::KC ? matrix_range(g.A, g.lda, g.Mo, g.R, 2, &r) : matrix_range(g.A, g.lda, g.R, g.Mo, 2, &r))
        f.in[f.n_in++] = r;
    if (pl.lb == axo::KC ? matrix_range(g.B, g.ldb, g.No, g.R, 2, &r) : matrix_range(g.B, g.ldb, g.R, g.No, 2, &r))
        f.in[f.n_in++] = r;
    if (g.add_bias && matrix_range(g.bias, g.No, 1, g.No, 2, &r)) f.in[f.n_in++] = r;
    if (matrix_range(g.aux, g.ldaux, g.Mo, g.No, 2, &r)) f.in[f.n_in++] = r;
    f.has_out = matrix_range(g.C, g.ldc, g.Mo, g.No, g.epilogue == axo::EPI_ACC_F32 ? 4 : 2, &f.out);
    return f;
}
// The rule of the header, checked: an output that shares bytes with an input of its own product is
// refused.  The kernels write an output tile while other workgroups still read the operands, and
// a ragged output is covered with overlapping tiles that are computed twice, so an in-place call
// (say dX written over the pre-activation it is multiplied with) would silently go wrong.
int check_no_alias(const Plan& pl) { return footprint(pl).output_aliases_input() ? AXO_ERR_BAD_ARG : AXO_OK; }
// Dependence level of every product of a chain given in program order: 0 when it conflicts with
// no earlier product, otherwise one more than the highest level among the earlier products it
// conflicts with.  Products of one level are independent of each other, and every product a
// given one depends on sits on a lower level, so enqueueing level by level on one stream gives
// the results of the program order.  The pairwise comparison is quadratic; beyond
// MAX_ANALYSED products the chain simply keeps its order (level = position).  Returns the
// number of levels.
constexpr size_t MAX_ANALYSED = 768;  // 256 layers
int dependence_levels(const std::vector<Plan>& plans, std::vector<int>* level) {
    const size_t n = plans.size();
    level->assign(n, 0);
    if (n == 0) return 0;
    if (n > MAX_ANALYSED) {
        for (size_t j = 0; j < n; ++j) (*level)[j] = (int)j;
        return (int)n;
    }
    std::vector<Footprint> fp(n);
    for (size_t j = 0; j < n; ++j) fp[j] = footprint(plans[j]);
    int levels = 1;
    for (size_t j = 1; j < n; ++j) {
        int lv = 0;
        for (size_t i = 0; i < j; ++i)
            if ((*level)[i] >= lv && fp[i].conflicts_with_later(fp[j])) lv = (*level)[i] + 1;
        (*level)[j] = lv;
        if (lv + 1 > levels) levels = lv + 1;
    }
    return levels;
}

// Enqueues the products level by level: those of a level that the tiled kernel takes share
// grouped launches (GROUP_MAX_PRODUCTS per launch), the others get a launch of their own.
int enqueue_by_level(const std::vector<Plan>& plans, const std::vector<int>& level, int levels, hipStream_t st) {
    int rc = AXO_OK;
    std::deque<Plan> covers;          // pieces of covered products (a deque keeps their addresses)
    std::vector<const Plan*> group;   // products of the level the tiled kernel takes
    std::vector<const Plan*> riders;  // bias gradients of the level that may share their launch
    auto flush = [&]() {
        if (group.empty() || rc != AXO_OK) return;
        rc = group.size() == 1 ? launch_tile_layout(group[0]->g, group[0]->la, group[0]->lb, st)
                               : launch_group(group.data(), (int)group.size(), st);
        group.clear();
    };
    // the last launch of a level takes the level's bias gradients along, as many as fit
    auto flush_level = [&]() {
        while (!riders.empty() && !group.empty() && (int)group.size() < axo::GROUP_MAX_PRODUCTS) {
            group.push_back(riders.back());
            riders.pop_back();
        }
        flush();
        for (size_t k = 0; k < riders.size() && rc == AXO_OK; ++k) rc = launch_bias_grad(riders[k]->bg, st);
        riders.clear();
    };
    for (int lv = 0; lv < levels && rc == AXO_OK; ++lv) {
        for (size_t i = 0; i < plans.size() && rc == AXO_OK; ++i) {
            const Plan& pl = plans[i];
            if (level[i] != lv || pl.nothing_to_do()) continue;
            if (pl.bias_grad) {
                if (bias_grad_groupable(pl.bg)) riders.push_back(&pl);
                else rc = launch_bias_grad(pl.bg, st);
                continue;
            }
            if (!tileable(pl.g, pl.la, pl.lb)) {
                std::vector<Plan> pieces;
                if (!cover_with_tiles(pl, &pieces)) {
                    rc = launch(pl.g, pl.la, pl.lb, st);
                    continue;
                }
                if (group.size() + pieces.size() > (size_t)axo::GROUP_MAX_PRODUCTS) flush();
                for (const Plan& piece : pieces) {  // the pieces of a cover share the level's grouped launch
                    covers.push_back(piece);
                    group.push_back(&covers.back());
                }
                if ((int)group.size() >= axo::GROUP_MAX_PRODUCTS) flush();
                continue;
            }
            group.push_back(&pl);
            if ((int)group.size() == axo::GROUP_MAX_PRODUCTS) flush();
        }
        flush_level();
    }
    return rc;
}

// A validated chain, scheduled by dependence level.
int enqueue_scheduled(const std::vector<Plan>& plans, hipStream_t st) {
    if (plans.size() > MAX_ANALYSED) {  // not analysed: program order, one unit per launch
        int rc = AXO_OK;
        for (size_t i = 0; i < plans.size() && rc == AXO_OK; ++i) rc = launch_plan(plans[i], st);
        return rc;
    }
    std::vector<int> level;
    const int levels = dependence_levels(plans, &level);
    return enqueue_by_level(plans, level, levels, st);
}

// No exception leaves the library: the planners keep their lists and caches in standard
// containers, whose allocations can fail.
template <typename F>
int guarded(F&& body) noexcept {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return AXO_ERR_NO_MEMORY;
    } catch (...) {
        return AXO_ERR_BAD_ARG;
    }
}

}  // namespace

extern "C" {

int axo_version(void) { return AXO_VERSION; }

const char* axo_status_string(int status) {
    switch (status) {
        case AXO_OK: return "ok";
        case AXO_ERR_BAD_GRID: return "grid dimension < 1";
        case AXO_ERR_BAD_COORD: return "grid coordinate outside the grid";
        case AXO_ERR_INDIVISIBLE: return "T, K or N not divisible by its grid dimension";
        case AXO_ERR_NULL_PTR: return "required pointer is NULL";
        case AXO_ERR_MISALIGNED: return "pointer not 16-byte aligned or leading dimension not a multiple of 8";
        case AXO_ERR_BAD_LD: return "leading dimension smaller than the row length";
        case AXO_ERR_WORKSPACE: return "workspace too small";
        case AXO_ERR_BAD_EPILOGUE: return "unknown epilogue or epilogue without bias";
        case AXO_ERR_HIP: return "HIP launch failed";
        case AXO_ERR_BAD_SIZE: return "negative size or shard dimension beyond 2^31-1";
        case AXO_ERR_BAD_ARG: return "malformed argument";
        case AXO_ERR_NO_MEMORY: return "host allocation failed";
        case AXO_ERR_TOO_LARGE: return "problem needs more scratch memory than the allocation-free entry point holds";
        default: return "unknown status";
    }
}

int axo_shard_dims(const axo_problem_t* p, int64_t* M, int64_t* Kl, int64_t* Nl, int64_t* row0, int64_t* k0,
                   int64_t* n0) {
    Shard s;
    int rc = derive_shard(p, &s);
    if (rc) return rc;
    if (M) *M = s.M;
    if (Kl) *Kl = s.Kl;
    if (Nl) *Nl = s.Nl;
    if (row0) *row0 = s.row0;
    if (k0) *k0 = s.k0;
    if (n0) *n0 = s.n0;
    return AXO_OK;
}

size_t axo_workspace_bytes(const axo_problem_t* p, int op) {
    Shard s;
    if (derive_shard(p, &s) != AXO_OK) return 0;
    if (op < AXO_OP_FWD || op > AXO_OP_WGRAD) return 0;
    return 0;  // no product needs workspace at present; the argument is kept for split reductions
}

int axo_fc_route(const axo_problem_t* p, int op, int64_t ld_a, int64_t ld_b, int64_t ld_out, int* route) {
    return guarded([&]() -> int {
        if (!route) return AXO_ERR_NULL_PTR;
        if (op < AXO_OP_FWD || op > AXO_OP_WGRAD) return AXO_ERR_BAD_ARG;
        // made-up, well-separated and aligned addresses: the planners compare pointers, never follow them
        const void* a = reinterpret_cast<const void*>((uintptr_t)1 << 40);
        const void* b = reinterpret_cast<const void*>((uintptr_t)2 << 40);
        void* c = reinterpret_cast<void*>((uintptr_t)3 << 40);
        Plan pl;
        const int rc = op == AXO_OP_FWD     ? plan_fwd(p, a, ld_a, b, ld_b, nullptr, AXO_EPI_NONE, c, ld_out, nullptr, 0, &pl)
                       : op == AXO_OP_DGRAD ? plan_dgrad(p, a, ld_a, b, ld_b, c, ld_out, nullptr, 0, &pl)
                                            : plan_wgrad(p, a, ld_a, b, ld_b, c, ld_out, nullptr, 0, &pl);
        if (rc) return rc;
        std::vector<Plan> pieces;
        *route = route_of(pl.g, pl.la, pl.lb, &pieces);
        return AXO_OK;
    });
}

int axo_fc_fwd(const axo_problem_t* p, const void* X, int64_t ldx, const void* W, int64_t ldw, const void* bias,
               int epilogue, void* Y, int64_t ldy, void* ws, size_t ws_bytes, void* hip_stream) {
    return guarded([&]() -> int {
        Plan pl;
        int rc = plan_fwd(p, X, ldx, W, ldw, bias, epilogue, Y, ldy, ws, ws_bytes, &pl);
        if (rc) return rc;
        return launch(pl.g, pl.la, pl.lb, static_cast<hipStream_t>(hip_stream));
    });
}

int axo_fc_dgrad(const axo_problem_t* p, const void* dY, int64_t lddy, const void* W, int64_t ldw, void* dX,
                 int64_t lddx, void* ws, size_t ws_bytes, void* hip_stream) {
    return guarded([&]() -> int {
        Plan pl;
        int rc = plan_dgrad(p, dY, lddy, W, ldw, dX, lddx, ws, ws_bytes, &pl);
        if (rc) return rc;
        return launch(pl.g, pl.la, pl.lb, static_cast<hipStream_t>(hip_stream));
    });
}

int axo_fc_wgrad(const axo_problem_t* p, const void* X, int64_t ldx, const void* dY, int64_t lddy, void* dW,
                 int64_t lddw, void* ws, size_t ws_bytes, void* hip_stream) {
    return guarded([&]() -> int {
        Plan pl;
        int rc = plan_wgrad(p, X, ldx, dY, lddy, dW, lddw, ws, ws_bytes, &pl);
        if (rc) return rc;
        return launch(pl.g, pl.la, pl.lb, static_cast<hipStream_t>(hip_stream));
    });
}

int axo_fc_dgrad_act(const axo_problem_t* p, const void* dY, int64_t lddy, const void* W, int64_t ldw, const void* pre,
                     int64_t ldpre, int act, void* dX, int64_t lddx, void* ws, size_t ws_bytes, void* hip_stream) {
    return guarded([&]() -> int {
        Plan pl;
        int rc = plan_dgrad_act(p, dY, lddy, W, ldw, pre, ldpre, act, dX, lddx, ws, ws_bytes, &pl);
        if (rc) return rc;
        return launch(pl.g, pl.la, pl.lb, static_cast<hipStream_t>(hip_stream));
    });
}

int axo_fc_wgrad_acc(const axo_problem_t* p, const void* X, int64_t ldx, const void* dY, int64_t lddy, float* dW,
                     int64_t lddw, void* ws, size_t ws_bytes, void* hip_stream) {
    return guarded([&]() -> int {
        Plan pl;
        int rc = plan_wgrad_acc(p, X, ldx, dY, lddy, dW, lddw, ws, ws_bytes, &pl);
        if (rc) return rc;
        return launch(pl.g, pl.la, pl.lb, static_cast<hipStream_t>(hip_stream));
    });
}

int axo_bias_grad(const axo_problem_t* p, const void* dY, int64_t lddy, float* db, int accumulate, void* hip_stream) {
    Plan pl;
    const int rc = plan_bias_grad(p, dY, lddy, db, accumulate, &pl);
    if (rc) return rc;
    return launch_bias_grad(pl.bg, static_cast<hipStream_t>(hip_stream));
}

size_t axo_bias_grad_workspace_bytes(const axo_problem_t* p) {
    Shard s;
    if (derive_shard(p, &s) != AXO_OK) return 0;
    return plan_bias_split(s.M, s.Nl).bytes();
}

int axo_bias_grad_ws(const axo_problem_t* p, const void* dY, int64_t lddy, float* db, int accumulate, void* ws,
                     size_t ws_bytes, void* hip_stream) {
    Plan pl;
    const int rc = plan_bias_grad(p, dY, lddy, db, accumulate, &pl);
    if (rc) return rc;
    const BiasSplit b = plan_bias_split(pl.bg.M, pl.bg.Nl);
    if (b.bytes() > 0) {
        if (!ws || ws_bytes < b.bytes()) return AXO_ERR_WORKSPACE;
        if (!aligned16(ws)) return AXO_ERR_MISALIGNED;
    }
    return launch_bias_grad_split(pl.bg, b, ws, static_cast<hipStream_t>(hip_stream));
}

int axo_bias_grad_static(const axo_problem_t* p, const void* dY, int64_t lddy, float* db, int accumulate,
                         void* hip_stream) {
    Plan pl;
    const int rc = plan_bias_grad(p, dY, lddy, db, accumulate, &pl);
    if (rc) return rc;
    if (pl.bg.Nl == 0) return AXO_OK;
    const BiasSplit b = plan_bias_split(pl.bg.M, pl.bg.Nl);
    if (b.bytes() > STATIC_SCRATCH_BYTES) return AXO_ERR_TOO_LARGE;
    void* dev_scratch = nullptr;
    if (b.bytes() > 0) {
        const int sc = static_scratch(&dev_scratch);
        if (sc) return sc;
    }
    return launch_bias_grad_split(pl.bg, b, dev_scratch, static_cast<hipStream_t>(hip_stream));
}

size_t axo_bias_grad_static_limit(void) { return STATIC_SCRATCH_BYTES; }

size_t axo_layer_step_workspace_bytes(const axo_layer_t* layers, int n_layers) {
    size_t need = 0;
    if (!layers) return 0;
    for (int i = 0; i < n_layers; ++i)
        for (int op = AXO_OP_FWD; op <= AXO_OP_WGRAD; ++op) {
            size_t b = axo_workspace_bytes(&layers[i].p, op);
            if (b > need) need = b;
        }
    return need;
}

int axo_layer_step(const axo_layer_t* layers, int n_layers, void* ws, size_t ws_bytes, void* hip_stream) {
    return guarded([&]() -> int {
        std::vector<Plan> plans;
        const int rc = plan_chain(layers, n_layers, ws, ws_bytes, &plans);
        if (rc != AXO_OK) return rc;
        return enqueue_scheduled(plans, static_cast<hipStream_t>(hip_stream));
    });
}

int axo_layer_step_ext(const axo_layer_ext_t* layers, int n_layers, void* ws, size_t ws_bytes, void* hip_stream) {
    return guarded([&]() -> int {
        std::vector<Plan> plans;
        const int rc = plan_chain_ext(layers, n_layers, ws, ws_bytes, &plans);
        if (rc != AXO_OK) return rc;
        return enqueue_scheduled(plans, static_cast<hipStream_t>(hip_stream));
    });
}

int axo_layer_step_ordered(const axo_layer_t* layers, int n_layers, void* ws, size_t ws_bytes, void* hip_stream) {
    return guarded([&]() -> int {
        std::vector<Plan> plans;
        int rc = plan_chain(layers, n_layers, ws, ws_bytes, &plans);
        for (size_t i = 0; i < plans.size() && rc == AXO_OK; ++i)
            rc = launch_plan(plans[i], static_cast<hipStream_t>(hip_stream));
        return rc;
    });
}

int axo_layer_step_levels(const axo_layer_t* layers, int n_layers, int* n_levels, int* levels) {
    return guarded([&]() -> int {
        if (!n_levels) return AXO_ERR_NULL_PTR;
        std::vector<Plan> plans;
        const int rc = plan_chain(layers, n_layers, nullptr, 0, &plans);
        if (rc != AXO_OK) return rc;
        std::vector<int> level;
        *n_levels = dependence_levels(plans, &level);
        if (levels)
            for (size_t i = 0; i < level.size(); ++i) levels[i] = level[i];
        return AXO_OK;
    });
}

}  // extern "C"
