// grass_compressed_grad and grass_dense_grad: C[j, i] = scale_j * sum_t dY[t, col_j] * X[t, i].
//
// Both operands are stored with the contraction index t as the ROW index (dY is T x m, X is
// T x n), i.e. this is a "TN" GEMM C = A^T B with A = dY[:, cols] and B = X.
//
// bf16 path (the hot one):
//   1. pack:   the r selected columns of dY are gathered once into a dense T x r_pad bf16
//              panel (zero padded to the tile width).  A per-element gather inside the
//              GEMM main loop would pull m/r times more cache lines through each CU's L1
//              than the tile uses; doing it once in an HBM-bound pass keeps the GEMM's
//              inner loop on full 16-byte loads.  (The dense gradient needs no pack.)
//              Wide matrices stage whole rows of dY through LDS (streaming loads, gather
//              from LDS); narrow sets of a group share one launch.  With dY stored m x T
//              there is no pack: the GEMM's tile loads fetch the selected rows themselves.
//   2. GEMM:   v_mfma_f32_32x32x16_bf16 tiles.  Global tiles [BK x BM] / [BK x BN] are staged
//              through LDS in their memory order (t-major) with 16-byte loads; the MFMA
//              operand layout (8 consecutive t per lane) is produced by the gfx950
//              transposing LDS read ds_read_b64_tr_b16, so no transpose is ever
//              materialised.  Split-K over T fills the 256 CUs; work items are numbered
//              so that the workgroups an XCD receives share one K slice (L2 reuse).
//   3. reduce: sums the split-K partials in a fixed order (deterministic), applies rho and
//              converts to the output dtype; in a regular step this, Adam and the update of
//              the rows of W are one kernel that reads the partial tiles directly.
// fp32 path: a plain LDS-tiled FMA kernel (small reference-precision configurations).
#include <atomic>

#include "common.hpp"

#include "gemm_common.hpp"
#include "pack_kernels.hpp"
#include "gemm_small.hpp"
#include "gemm_large.hpp"
#include "gemm_gather_narrow.hpp"
#include "reduce_kernels.hpp"

namespace grass {
namespace {

// ------------------------------------------------------------------------------ host side
using Cfg128 = TileCfg<128, 128, 64, 2, 2>;
enum TileId { kTile128 = 0, kTile256 = 1 };
struct Shape256 {
    static constexpr int BM = kFastBM, BN = kFastBN, BK = kFastBK, kWgPerCu = 1;
    static constexpr bool kWholeKTilesOnly = true;  // a ragged tail of T is a separate slice
};

struct Plan {
    int64_t Mp, Np, rp;  // padded rows / cols of the partial buffer; packed panel width
    int tiles_m, tiles_n, splits, ktiles_per_split;
    size_t pack_bytes, partial_bytes;
};

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// A slice of partial tiles up to this size is re-read from the caches by the reduction.
constexpr int64_t kCachedSliceBytes = int64_t{16} << 20;
constexpr int kManySlices = 8;  // above this the reduction spreads the slices over wavefronts

template <typename Cfg>
Plan make_plan(int64_t T, int64_t rows, int64_t n, bool needs_pack) {
    Plan p;
    p.tiles_m = static_cast<int>((rows + Cfg::BM - 1) / Cfg::BM);
    p.tiles_n = static_cast<int>((n + Cfg::BN - 1) / Cfg::BN);
    p.Mp = static_cast<int64_t>(p.tiles_m) * Cfg::BM;
    p.Np = static_cast<int64_t>(p.tiles_n) * Cfg::BN;
    p.rp = p.Mp;
    const int64_t ktiles = Cfg::kWholeKTilesOnly ? T / Cfg::BK : (T + Cfg::BK - 1) / Cfg::BK;
    const int64_t tiles = static_cast<int64_t>(p.tiles_m) * p.tiles_n;
    // Split K so that the workgroups fill whole rounds of the machine (256 CUs x workgroups
    // per CU) without paying too much for the partial tiles every slice adds.  In units of
    // the GEMM's time at full occupancy, c slices cost about 1 / fill(c) + c * k / T.  For
    // outputs of more than 16 MB per slice (the 7B / 13B layers) k = 1400: a slice writes and
    // re-reads 8 bytes per output element at ~4 TB/s while the GEMM spends 2 T flops per output
    // element at ~1.4 PFLOP/s.  The short, wide products of the small models are bound by
    // memory, not by the matrix cores, so an unfilled round costs them less and a slice
    // relatively more; k is then fitted to sweeps of the slice count on their layer shapes
    // (T = 65536): 2400 for the large tile (1024 x 1024 at r = 256: 42 slices, 81 us per step,
    // against 64 slices, 92 us) and 800 for the small one (512 x 512 at r = 128: 94 slices).
    // Each slice keeps at least 8 K tiles.
    const int64_t slots = 256 * Cfg::kWgPerCu;
    int64_t smax = ktiles / 8 > 0 ? (ktiles / 8 < 128 ? ktiles / 8 : 128) : 1;
    if (const int cap = test_option(GRASS_TEST_MAX_K_SLICES)) smax = cap > 0 && cap < smax ? cap : smax;
    const bool cached = p.Mp * p.Np * 4 <= kCachedSliceBytes;
    const double k = cached ? (Cfg::BM == 256 ? 2400.0 : 800.0) : 1400.0;
    const double per_slice = k / static_cast<double>(T > 0 ? T : 1);
    int64_t s = 1;
    double best = 1e300;
    for (int64_t c = 1; c <= smax && tiles > 0; ++c) {
        const int64_t wgs = tiles * c, rounds = (wgs + slots - 1) / slots;
        const double cost = static_cast<double>(rounds * slots) / static_cast<double>(wgs) + per_slice * c;
        if (cost < best - 1e-12) { best = cost; s = c; }
    }
    p.ktiles_per_split = static_cast<int>((ktiles + s - 1) / s);
    if (p.ktiles_per_split < 1) p.ktiles_per_split = 1;
    p.splits = static_cast<int>((ktiles + p.ktiles_per_split - 1) / p.ktiles_per_split);
    if (p.splits < 1) p.splits = 1;
    p.pack_bytes = needs_pack ? round_up(static_cast<size_t>(T) * p.rp * 2, 256) : 0;
    // one spare slice: the large-tile path gives the ragged tail of T to the small-tile kernel
    p.partial_bytes = static_cast<size_t>(p.splits + 1) * p.Mp * p.Np * 4;
    return p;
}

// The GEMM kernels read the left operand as T x rows with 16-byte chunks along the rows: a
// gather, the m x T storage, or a row count that breaks the chunks needs the packing pass.
bool needs_pack(grass_dy_layout layout, bool gathered, int64_t rows) {
    return gathered || layout == GRASS_DY_MxT || rows % 8 != 0;
}

// X with n not a multiple of 8 is first copied to rows of round_up(n, 8) elements.
size_t aligned_x_bytes(int64_t T, int64_t n) {
    return n % 8 != 0 ? round_up(static_cast<size_t>(T) * ((n + 7) / 8 * 8) * 2, 256) : 0;
}

// The 256 x 256 tile halves the LDS traffic per flop and is the faster kernel whenever it
// does not waste much of itself on padding; narrow problems (r = 128, say) keep 128 x 128.
TileId choose_tile(int64_t T, int64_t rows, int64_t n) {
    if (const int forced = test_option(GRASS_TEST_GEMM_TILE)) return forced == 256 ? kTile256 : kTile128;
    (void)T;
    if (rows < 1 || n < 1) return kTile128;
    const double padded = static_cast<double>((rows + 255) / 256 * 256) * ((n + 255) / 256 * 256);
    return padded <= 1.35 * static_cast<double>(rows) * static_cast<double>(n) ? kTile256 : kTile128;
}

Plan plan_for(TileId id, int64_t T, int64_t rows, int64_t n, bool pack) {
    return id == kTile256 ? make_plan<Shape256>(T, rows, n, pack) : make_plan<Cfg128>(T, rows, n, pack);
}

// ---- narrow layers: the gather inside the GEMM (gemm_gather_narrow.hpp)
// Shapes the kernel takes, apart from what is asked of every set and of the addresses: at most two
// column tiles (beyond that each tile re-reads and re-gathers the rows of dY once more and the
// packed route wins: the step of a 512 x 1376 layer at r = 128, T = 65536 takes 83 us this way
// against 74), whole K tiles.
bool narrow_shape_ok(int64_t T, int64_t n, grass_dtype dt, grass_dy_layout layout) {
    return test_option(GRASS_TEST_NO_NARROW_GATHER) == 0 && test_option(GRASS_TEST_GEMM_TILE) == 0 &&
           dt == GRASS_BF16 && layout == GRASS_DY_TxM && T >= kNarrowBK && T % kNarrowBK == 0 &&
           n >= 8 && n % 8 == 0 && n <= 2 * kNarrowBN;
}
// one set: a single row tile, rows of dY that fit a stage
bool narrow_set_ok(int64_t rows, int64_t m_src) {
    return rows > 0 && rows <= kNarrowBM && m_src >= 8 && m_src % 8 == 0 && m_src <= kNarrowMaxM;
}
struct NarrowPlan {
    int64_t Mp, Np;
    int tiles_n, splits, ktiles_per_split;
};
// `tiles_m` row tiles in all, `panel_rows` rows of partial tiles per slice, `in_cols` = the row
// lengths of all inputs together (sum of m over the sets, plus n).  Slices: about two workgroups
// per compute unit (what the kernel's LDS use allows), as long as the partial tiles stay under a
// quarter of the input bytes (measured at the 60M shapes, T = 65536: 512 x 512 at r = 128 takes
// 26 us with 128 slices, 30 - 33 with 96, 170 or 256; the q/k/v group 66 us with 85 slices, 82
// with 42), every slice keeps at least four K tiles, and the workspace holds them.
NarrowPlan narrow_plan(int64_t T, int64_t n, int tiles_m, int64_t panel_rows, int64_t in_cols,
                       size_t cap_bytes) {
    NarrowPlan p;
    p.tiles_n = static_cast<int>((n + kNarrowBN - 1) / kNarrowBN);
    p.Np = static_cast<int64_t>(p.tiles_n) * kNarrowBN;
    p.Mp = (panel_rows + 7) / 8 * 8;
    const int64_t ktiles = T / kNarrowBK, tiles = static_cast<int64_t>(tiles_m) * p.tiles_n;
    const int64_t slice_bytes = p.Mp * p.Np * 4;
    int64_t s = tiles > 0 ? (512 + tiles - 1) / tiles : 1;
    const int64_t by_traffic = T * in_cols * 2 / 4 / (slice_bytes > 0 ? slice_bytes : 1);
    const int64_t by_space = static_cast<int64_t>(cap_bytes) / (slice_bytes > 0 ? slice_bytes : 1);
    s = s < by_traffic ? s : by_traffic;
    s = s < by_space ? s : by_space;
    s = s < ktiles / 4 ? s : ktiles / 4;
    s = s < 128 ? s : 128;
    if (const int cap = test_option(GRASS_TEST_MAX_K_SLICES)) s = cap > 0 && cap < s ? cap : s;
    s = s < 1 ? 1 : s;
    p.ktiles_per_split = static_cast<int>((ktiles + s - 1) / s);
    p.splits = static_cast<int>((ktiles + p.ktiles_per_split - 1) / p.ktiles_per_split);
    return p;
}

template <typename Cfg, bool kDense>
hipError_t launch_gemm_kernel(const GemmArgs& g, unsigned grid, hipStream_t s) {
    auto kernel = tn_gemm_bf16_kernel<Cfg, kDense>;
    if (Cfg::kLdsBytes > 64 * 1024) {
        // per instantiation and device; the attribute sticks for the life of the process, so it
        // is set once (the only state the library keeps: a flag per device, set with release
        // order after the attribute call has returned; two first callers both make the call)
        static std::atomic<bool> raised[64];
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
        if (dev < 0 || dev >= 64 || !raised[dev].load(std::memory_order_acquire)) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     static_cast<int>(Cfg::kLdsBytes));
            if (e != hipSuccess) return e;
            if (dev >= 0 && dev < 64) raised[dev].store(true, std::memory_order_release);
        }
    }
    kernel<<<grid, Cfg::kThreads, Cfg::kLdsBytes, s>>>(g);
    return hipSuccess;
}

bool fused_stats_shape_ok(int64_t T, int64_t m, int64_t n, grass_dtype dt, grass_dy_layout layout,
                          int64_t ldy, int64_t ldx) {
    // the squares need complete sums, so the fused form cannot split K: it only pays when the
    // output tiles alone fill most of the 256 compute units
    const int64_t tiles = ((m + kFastBM - 1) / kFastBM) * ((n + kFastBN - 1) / kFastBN);
    const bool force = test_option(GRASS_TEST_FUSED_STATS) == 1;  // whenever the shape allows
    return (tiles >= 192 || force) && dt == GRASS_BF16 && layout == GRASS_DY_TxM && T >= kFastBK &&
           T % kFastBK == 0 &&
           m >= 8 && n >= 8 && m % 8 == 0 && n % 8 == 0 && ldy % 8 == 0 && ldx % 8 == 0 &&
           (kFastBK + 1) * ldy * 2 < (int64_t{1} << 32) && (kFastBK + 1) * ldx * 2 < (int64_t{1} << 32);
}

size_t fused_stats_bytes(int64_t m, int64_t n) {
    const int64_t tiles_m = (m + kFastBM - 1) / kFastBM, tiles_n = (n + kFastBN - 1) / kFastBN;
    return static_cast<size_t>(2 * tiles_n) * tiles_m * kFastBM * 4 + 256;
}

}  // namespace

size_t grad_row_stats_workspace_bytes(int64_t T, int64_t m, int64_t n, grass_dtype dt,
                                      grass_dy_layout layout, int64_t ldy, int64_t ldx) {
    if (fused_stats_shape_ok(T, m, n, dt, layout, ldy, ldx)) return fused_stats_bytes(m, n);
    // otherwise G is formed in fp32 inside the workspace and reduced from there
    return static_cast<size_t>(m) * n * 4 + 256 + gemm_workspace_bytes(T, m, n, dt, layout, false);
}

grass_status launch_grad_row_stats(const void* dY, grass_dy_layout layout, int64_t ldy,
                                   const void* X, int64_t ldx, grass_dtype dt, int64_t T, int64_t m,
                                   int64_t n, float* sumsq, void* ws, size_t ws_bytes,
                                   hipStream_t s) {
    if (m == 0) return GRASS_OK;
    char* base = static_cast<char*>(ws);
    base += (256 - reinterpret_cast<uintptr_t>(base) % 256) % 256;
    const bool fused = fused_stats_shape_ok(T, m, n, dt, layout, ldy, ldx) && aligned_to(dY, 16) &&
                       aligned_to(X, 16);
    if (fused) {
        if (ws_bytes < fused_stats_bytes(m, n)) return GRASS_ERR_WORKSPACE;
        GemmArgs g;
        g.A = static_cast<const uint16_t*>(dY);
        g.B = static_cast<const uint16_t*>(X);
        g.P = reinterpret_cast<float*>(base);
        g.lda = ldy; g.ldb = ldx; g.K = T; g.Mcols = m; g.Ncols = n;
        g.tiles_m = static_cast<int>((m + kFastBM - 1) / kFastBM);
        g.tiles_n = static_cast<int>((n + kFastBN - 1) / kFastBN);
        g.Mp = static_cast<int64_t>(g.tiles_m) * kFastBM;
        g.Np = static_cast<int64_t>(g.tiles_n) * kFastBN;
        g.splits = 1;
        g.ktiles_per_split = static_cast<int>(T / kFastBK);
        g.a_fast = g.b_fast = 1;
        g.a_rows = nullptr;
        const int64_t items = static_cast<int64_t>(g.tiles_m) * g.tiles_n;
        const int64_t chunk = (items + kNumXcd - 1) / kNumXcd;
        if (chunk * kNumXcd > 0x7FFFFFFF) return GRASS_ERR_SHAPE;
        tn_gemm_bf16_direct_kernel<true, true><<<static_cast<unsigned>(chunk * kNumXcd), 256, 0, s>>>(g);
        rowpart_reduce_kernel<<<static_cast<unsigned>((m + 255) / 256), 256, 0, s>>>(
            g.P, 2 * g.tiles_n, g.Mp, m, sumsq);
        return launch_status();
    }
    const size_t g_bytes = static_cast<size_t>(m) * n * 4 + 256;
    const size_t need = g_bytes + gemm_workspace_bytes(T, m, n, dt, layout, false);
    if (ws_bytes < need) return GRASS_ERR_WORKSPACE;
    if (m > 65535) return GRASS_ERR_SHAPE;
    float* G = reinterpret_cast<float*>(base);
    const grass_status st = launch_tn_gemm(dY, layout, ldy, X, ldx, dt, T, m, n, nullptr, nullptr, G,
                                           GRASS_F32, n, base + g_bytes, s, m);
    if (st != GRASS_OK) return st;
    return launch_row_stats(G, GRASS_F32, m, n, n, sumsq, s);
}

size_t gemm_workspace_bytes(int64_t T, int64_t mrows, int64_t n, grass_dtype dt,
                            grass_dy_layout layout, bool gathered) {
    if (dt == GRASS_F32) return 0;
    // the launcher may fall back to the small tile when alignment rules out the large one
    const bool pack = needs_pack(layout, gathered, mrows);
    const Plan a = plan_for(kTile128, T, mrows, n, pack), b = plan_for(kTile256, T, mrows, n, pack);
    const size_t wa = a.pack_bytes + a.partial_bytes, wb = b.pack_bytes + b.partial_bytes;
    return (wa > wb ? wa : wb) + aligned_x_bytes(T, n) + 256;
}

void gemm_plan_summary(int64_t T, int64_t m, int64_t rows, int count, int64_t n, grass_dtype dt,
                       grass_dy_layout layout, int* tile, int* k_slices) {
    if (dt == GRASS_F32) {  // the fp32 kernel: 64 x 64 tiles, K not split
        *tile = 64;
        *k_slices = 1;
        return;
    }
    if (m > 0 && count >= 1 && narrow_shape_ok(T, n, dt, layout) &&
        narrow_set_ok((rows / count + 7) / 8 * 8, m)) {  // the sets taken to be of equal size
        const size_t cap = gemm_workspace_bytes(T, rows, n, dt, layout, true) - 256;
        const NarrowPlan p = narrow_plan(T, n, count, rows, m * count + n, cap);
        *tile = 0;
        *k_slices = p.splits;
        return;
    }
    const TileId id = T >= kFastBK && rows >= 8 && n >= 8 ? choose_tile(T, rows, n) : kTile128;
    Plan p = plan_for(id, T, rows, n, needs_pack(layout, true, rows));
    if (id == kTile256 && layout == GRASS_DY_MxT && T % (2 * kFastBK) == 0 &&
        test_option(GRASS_TEST_PACK_MXT) == 0 && test_option(GRASS_TEST_NO_PAIRS) == 0 &&
        p.ktiles_per_split % 2 != 0) {  // the row-gathering kernel takes K tiles in pairs
        ++p.ktiles_per_split;
        p.splits = static_cast<int>((T / kFastBK + p.ktiles_per_split - 1) / p.ktiles_per_split);
    }
    *tile = id == kTile256 ? 256 : 128;
    // the large tile takes whole K tiles; a ragged tail of T is one more slice
    *k_slices = p.splits + (id == kTile256 && T % kFastBK != 0 ? 1 : 0);
}

size_t gemm_group_workspace_bytes(int64_t T, const int64_t* rows, int count, int64_t n,
                                  grass_dtype dt, grass_dy_layout layout) {
    int64_t total = 0;
    size_t need = 0;  // the sets may also be run one at a time
    for (int i = 0; i < count; ++i) {
        total += (rows[i] + 7) / 8 * 8;
        const size_t one = gemm_workspace_bytes(T, rows[i], n, dt, layout, true);
        need = one > need ? one : need;
    }
    const size_t joint = gemm_workspace_bytes(T, total, n, dt, layout, true);
    return joint > need ? joint : need;
}

// Adam and the row update from a G_C that has been written to seg.C (two-kernel route).
grass_status run_tail_unfused(const GemmSegment& q, int64_t n, hipStream_t s) {
    if (!q.tail || q.rows == 0) return GRASS_OK;
    const StepTail& t = *q.tail;
    if (t.U) {  // column form: Adam into U, then the update of the columns of W
        const grass_status st = launch_adam_rows(static_cast<const float*>(q.C), q.ldc, t.M, t.V, t.sdt,
                                                 q.rows, n, t.lr, t.beta1, t.beta2, t.eps, t.t, t.U, s);
        if (st != GRASS_OK) return st;
        return launch_scatter_cols(t.W, t.wdt, t.w_rows, t.ldw, q.idx, q.rho, t.alpha, t.U, q.rows, s);
    }
    return launch_adam_scatter(static_cast<const float*>(q.C), q.ldc, t.M, t.V, t.sdt, q.rows, n,
                               t.lr, t.beta1, t.beta2, t.eps, t.t, t.W, t.wdt, t.ldw, q.idx, q.rho,
                               t.alpha, s, t.step_scalars);
}

// What follows the matrix product for every set: the split-K reduction into the set's output,
// or, for a regular step, the fused reduction + Adam + update straight from the partial tiles
// [slices][Mp][Np] (the sets lie one after the other along the rows, each starting at a
// multiple of 8).
grass_status finish_segments(const GemmSegment* seg, int count, const float* partial, int slices,
                             int64_t Mp, int64_t Np, int64_t n, grass_dtype odt, hipStream_t s,
                             hipEvent_t ev_tail_start, hipEvent_t ev_tail_stop) {
    int64_t off = 0;
    TailSets tails;  // sets whose reduction, Adam and row update run as one kernel (one launch)
    int ntails = 0;
    const StepTail* tail_common = nullptr;
    for (int i = 0; i < count; ++i) {
        const GemmSegment& q = seg[i];
        if (q.rows > 0 && q.tail && odt == GRASS_F32 &&
            reduce_adam_scatter_ok(*q.tail, n, q.c_wanted ? static_cast<float*>(q.C) : nullptr, q.ldc)) {
            // straight from the partial tiles; launched after the loop, together
            const TailSet one{partial + off * Np, q.rows, q.tail->M, q.tail->V, q.tail->W,
                              q.tail->ldw, q.idx, q.rho,
                              q.c_wanted ? static_cast<float*>(q.C) : nullptr, q.ldc, q.tail->U};
            if (q.tail->U) {  // column form: its own launch, followed by the column update
                TailSets single;
                single.set[0] = one;
                grass_status st = launch_reduce_adam_scatter(single, 1, slices, Mp, Np, n, *q.tail, s,
                                                             ev_tail_start, ev_tail_stop);
                if (st != GRASS_OK) return st;
                st = launch_scatter_cols(q.tail->W, q.tail->wdt, q.tail->w_rows, q.tail->ldw, q.idx,
                                         q.rho, q.tail->alpha, q.tail->U, q.rows, s);
                if (st != GRASS_OK) return st;
            } else {
                tails.set[ntails++] = one;
                tail_common = q.tail;
            }
        } else if (q.rows > 0) {
            const dim3 rgrid(static_cast<unsigned>((n + 255) / 256), static_cast<unsigned>(q.rows));
            const float* part = partial + off * Np;
            if (slices > kManySlices && Np % 128 == 0) {
                if (odt == GRASS_F32)
                    splitk_reduce_many_kernel<float><<<rgrid, 256, 0, s>>>(
                        part, slices, Mp, Np, q.rows, n, q.rho, static_cast<float*>(q.C), q.ldc);
                else
                    splitk_reduce_many_kernel<uint16_t><<<rgrid, 256, 0, s>>>(
                        part, slices, Mp, Np, q.rows, n, q.rho, static_cast<uint16_t*>(q.C), q.ldc);
            } else if (odt == GRASS_F32)
                splitk_reduce_kernel<float><<<rgrid, 256, 0, s>>>(
                    part, slices, Mp, Np, q.rows, n, q.rho, static_cast<float*>(q.C), q.ldc);
            else
                splitk_reduce_kernel<uint16_t><<<rgrid, 256, 0, s>>>(
                    part, slices, Mp, Np, q.rows, n, q.rho, static_cast<uint16_t*>(q.C), q.ldc);
            if (q.tail && ev_tail_start) (void)hipEventRecord(ev_tail_start, s);
            const grass_status st = run_tail_unfused(q, n, s);
            if (st != GRASS_OK) return st;
            if (q.tail && ev_tail_stop) (void)hipEventRecord(ev_tail_stop, s);
        }
        off += (q.rows + 7) / 8 * 8;
    }
    if (ntails > 0) {
        const grass_status st = launch_reduce_adam_scatter(tails, ntails, slices, Mp, Np, n,
                                                           *tail_common, s, ev_tail_start, ev_tail_stop);
        if (st != GRASS_OK) return st;
    }
    return launch_status();
}

// C_i = scale_i * (A_i^T X) for `count` row sets that share X.  The sets are packed side by
// side into one panel (each starts at a multiple of 8 columns), one GEMM covers the panel,
// and the partial tiles are reduced into each set's own output.
grass_status launch_tn_gemm_segments(const GemmSegment* seg, int count, grass_dy_layout layout,
                                     const void* X, int64_t ldx, grass_dtype dt, int64_t T,
                                     int64_t n, grass_dtype odt, void* ws, hipStream_t s,
                                     hipEvent_t ev_start, hipEvent_t ev_stop,
                                     hipEvent_t ev_tail_start, hipEvent_t ev_tail_stop) {
    int64_t total = 0;  // panel columns in use
    for (int i = 0; i < count; ++i) {
        if (seg[i].rows > 65535) return GRASS_ERR_SHAPE;
        total += count > 1 ? (seg[i].rows + 7) / 8 * 8 : seg[i].rows;
    }
    if (total == 0 || n == 0) return GRASS_OK;
    if (dt == GRASS_F32) {
        if (ev_start) (void)hipEventRecord(ev_start, s);
        for (int i = 0; i < count; ++i) {
            const GemmSegment& g = seg[i];
            if (g.rows == 0) continue;
            const dim3 grid(static_cast<unsigned>((n + 63) / 64), static_cast<unsigned>((g.rows + 63) / 64));
            if (odt == GRASS_F32)
                tn_gemm_f32_kernel<float><<<grid, 256, 0, s>>>(
                    static_cast<const float*>(g.dY), layout, g.ldy, static_cast<const float*>(X),
                    ldx, T, g.rows, n, g.idx, g.rho, static_cast<float*>(g.C), g.ldc);
            else
                tn_gemm_f32_kernel<uint16_t><<<grid, 256, 0, s>>>(
                    static_cast<const float*>(g.dY), layout, g.ldy, static_cast<const float*>(X),
                    ldx, T, g.rows, n, g.idx, g.rho, static_cast<uint16_t*>(g.C), g.ldc);
        }
        if (ev_stop) (void)hipEventRecord(ev_stop, s);
        if (ev_tail_start) (void)hipEventRecord(ev_tail_start, s);
        for (int i = 0; i < count; ++i) {
            const grass_status st = run_tail_unfused(seg[i], n, s);
            if (st != GRASS_OK) return st;
        }
        if (ev_tail_stop) (void)hipEventRecord(ev_tail_stop, s);
        return launch_status();
    }

    const bool gathered = count > 1 || seg[0].idx != nullptr;
    bool pack = needs_pack(layout, gathered, total);
    if (count > 1) {
        // One panel pays off while a slice of partial tiles of the joint problem still fits
        // the caches (fewer, fuller launches).  Beyond that every set fills the machine on its
        // own and the joint partial tiles would only spill to HBM: run the sets one by one.
        const Plan joint = plan_for(choose_tile(T, total, n), T, total, n, pack);
        if (joint.Mp * joint.Np * 4 > kCachedSliceBytes) {
            for (int i = 0; i < count; ++i) {
                // (timing hooks: the first set's GEMM and the last set's tail)
                const bool first = i == 0, last = i + 1 == count;
                const grass_status st = launch_tn_gemm_segments(
                    seg + i, 1, layout, X, ldx, dt, T, n, odt, ws, s, first ? ev_start : nullptr,
                    first ? ev_stop : nullptr, last ? ev_tail_start : nullptr,
                    last ? ev_tail_stop : nullptr);
                if (st != GRASS_OK) return st;
            }
            return GRASS_OK;
        }
    }
    // Narrow layers (every set a single row tile of short dY rows): the gather runs inside the
    // GEMM, no panel is written.
    bool narrow = gathered && narrow_shape_ok(T, n, dt, layout) && aligned_to(X, 16) && ldx % 8 == 0 &&
                  ldx >= n && (kNarrowBK + 1) * ldx * 2 < (int64_t{1} << 32);
    for (int i = 0; i < count && narrow; ++i)
        narrow = seg[i].idx && narrow_set_ok(seg[i].rows, seg[i].src_rows) && aligned_to(seg[i].dY, 16) &&
                 seg[i].ldy % 8 == 0 && seg[i].ldy >= seg[i].src_rows &&
                 (kNarrowBK + 1) * seg[i].ldy * 2 < (int64_t{1} << 32);
    if (narrow) {
        char* base = static_cast<char*>(ws);
        base += (256 - reinterpret_cast<uintptr_t>(base) % 256) % 256;
        NarrowArgs a;
        int64_t in_cols = n;
        int off = 0;
        for (int i = 0; i < count; ++i) {
            a.set[i] = NarrowSet{static_cast<const uint16_t*>(seg[i].dY), seg[i].ldy, seg[i].idx,
                                 static_cast<int>(seg[i].rows), static_cast<int>(seg[i].src_rows / 8), off, i};
            off += static_cast<int>((seg[i].rows + 7) / 8 * 8);
            in_cols += seg[i].src_rows;
        }
        // the workspace every caller has been asked for holds at least this much (same formula)
        const size_t cap = gemm_workspace_bytes(T, total, n, dt, layout, true) - 256;
        const NarrowPlan np = narrow_plan(T, n, count, off, in_cols, cap);
        a.count = count;
        a.X = static_cast<const uint16_t*>(X);
        a.ldx = ldx;
        a.n = n;
        a.P = reinterpret_cast<float*>(base);
        a.Mp = np.Mp;
        a.Np = np.Np;
        a.ktiles = T / kNarrowBK;
        a.tiles_m = count;
        a.tiles_n = np.tiles_n;
        a.splits = np.splits;
        a.ktiles_per_split = np.ktiles_per_split;
        const int64_t items = static_cast<int64_t>(count) * np.tiles_n * np.splits;
        const unsigned grid = static_cast<unsigned>((items + kNumXcd - 1) / kNumXcd * kNumXcd);
        {   // more than 64 KB of LDS: the attribute is set once per device (see launch_gemm_kernel)
            static std::atomic<bool> raised[64];
            int dev = 0;
            if (hipGetDevice(&dev) != hipSuccess) return GRASS_ERR_DEVICE;
            if (dev < 0 || dev >= 64 || !raised[dev].load(std::memory_order_acquire)) {
                if (hipFuncSetAttribute(reinterpret_cast<const void*>(tn_gemm_gather_narrow_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize,
                                        kNarrowLdsBytes) != hipSuccess)
                    return GRASS_ERR_DEVICE;
                if (dev >= 0 && dev < 64) raised[dev].store(true, std::memory_order_release);
            }
        }
        launch_stamped(tn_gemm_gather_narrow_kernel, dim3(grid), dim3(256), kNarrowLdsBytes, s, ev_start,
                       ev_stop, a);
        return finish_segments(seg, count, a.P, np.splits, np.Mp, np.Np, n, odt, s, ev_tail_start,
                               ev_tail_stop);
    }
    const void* dY0 = seg[0].dY;  // read directly by the GEMM only when nothing is packed
    const int64_t ldy0 = seg[0].ldy;
    TileId tile = choose_tile(T, total, n);
    // X whose width breaks the 16-byte chunks is copied to padded rows first (T > 0: nothing
    // to copy otherwise); the GEMM then sees a matrix of round_up(n, 8) columns
    const bool copy_x = n % 8 != 0 && aligned_to(X, 4) && T > 0;
    const int64_t nb = copy_x ? (n + 7) / 8 * 8 : n;
    {   // the large-tile kernel moves whole aligned 16-byte chunks only
        const bool a_ok = pack || (aligned_to(dY0, 16) && ldy0 % 8 == 0 && total % 8 == 0);
        const bool b_ok = copy_x || (aligned_to(X, 16) && ldx % 8 == 0 && n % 8 == 0);
        // per-lane byte offsets inside one K tile are kept in 32 bits
        const int64_t lda_eff = pack ? (total + kFastBM - 1) / kFastBM * kFastBM : ldy0;
        const bool off_ok = (kFastBK + 1) * lda_eff * 2 < (int64_t{1} << 32) &&
                            (kFastBK + 1) * (copy_x ? nb : ldx) * 2 < (int64_t{1} << 32);
        if (!(a_ok && b_ok && off_ok && T >= kFastBK && total >= 8 && n >= 8)) tile = kTile128;
    }
    // dY stored m x T: the selected rows are contiguous, so the large-tile kernel gathers them
    // itself (no packing pass) when K is whole tiles and its 32-bit row offsets reach every row
    bool a_rows_form = false;
    if (tile == kTile256 && layout == GRASS_DY_MxT && count == 1 && T % kFastBK == 0 &&
        aligned_to(dY0, 16) && ldy0 % 8 == 0 && test_option(GRASS_TEST_PACK_MXT) == 0) {
        const int64_t src_rows = seg[0].idx ? seg[0].src_rows : total;
        a_rows_form = src_rows > 0 && src_rows * ldy0 * 2 + 128 < (int64_t{1} << 32);
    }
    if (a_rows_form) pack = false;
    // whole cache lines per row (64 values of k per load) when the K tiles pair up
    const bool a_pairs = a_rows_form && T % (2 * kFastBK) == 0 && test_option(GRASS_TEST_NO_PAIRS) == 0;
    // the large-tile kernel takes whole K tiles; a ragged tail goes to the small-tile kernel
    const int64_t T_main = tile == kTile256 ? T / kFastBK * kFastBK : T;
    Plan p = plan_for(tile, T, total, n, pack);  // sized for all T rows; K tiling per tile kind
    if (a_pairs && p.ktiles_per_split % 2 != 0) {  // every workgroup gets whole pairs of K tiles
        ++p.ktiles_per_split;
        const int64_t ktiles = T / kFastBK;
        p.splits = static_cast<int>((ktiles + p.ktiles_per_split - 1) / p.ktiles_per_split);
    }
    char* base = static_cast<char*>(ws);
    base += (256 - reinterpret_cast<uintptr_t>(base) % 256) % 256;
    uint16_t* panel = reinterpret_cast<uint16_t*>(base);
    float* partial = reinterpret_cast<float*>(base + p.pack_bytes);
    // launch sizes are checked before the first launch: a refused call has done nothing
    const int64_t items = static_cast<int64_t>(p.tiles_m) * p.tiles_n * p.splits;
    const int64_t chunk = (items + kNumXcd - 1) / kNumXcd;
    const int x_chunks = static_cast<int>((nb / 8 + 255) / 256);  // workgroups per row of the aligning copy
    if (chunk * kNumXcd > 0x7FFFFFFF || (copy_x && T * x_chunks > 0x7FFFFFFF)) return GRASS_ERR_SHAPE;

    GemmArgs g;
    if (pack) {
        // T x m storage, wide rows: staged through LDS (streaming loads of whole rows)
        // measured on the 60M to 1B layer shapes: from 1024 elements per row on the staged form
        // wins (3 - 15 %), at 512 it loses 20 %; the number of selected rows matters little
        constexpr int64_t min_width = 64, min_m = 1024;
        auto staged = [&](int i, int64_t width) {
            const int64_t m_src = seg[i].src_rows;
            return layout == GRASS_DY_TxM && m_src >= min_m && width >= min_width &&
                   pack_stage_row_elems(m_src) * 2 <= kPackStageMaxBytes;
        };
        auto threads_per_row_log2 = [](int64_t width) {
            int tpr_log2 = 8;  // the power of two covering width / 4
            while (tpr_log2 > 0 && (int64_t{4} << (tpr_log2 - 1)) >= width) --tpr_log2;
            return tpr_log2;
        };
        // several sets, none of them wide: one launch gathers them all
        bool one_launch = count > 1 && layout == GRASS_DY_TxM && T > 0;
        {
            PackSets sets;
            int64_t off = 0, gx = 1, gy = 1;
            for (int i = 0; i < count && one_launch; ++i) {
                const int64_t width = i + 1 == count ? p.rp - off : (seg[i].rows + 7) / 8 * 8;
                if (staged(i, width)) one_launch = false;
                const int tpr_log2 = threads_per_row_log2(width > 0 ? width : 1);
                sets.set[i] = PackSet{static_cast<const uint16_t*>(seg[i].dY), seg[i].ldy, seg[i].idx,
                                      seg[i].rows, width, off, tpr_log2};
                const int64_t rows_per_wg = static_cast<int64_t>(kPackRows) * (256 >> tpr_log2);
                const int64_t bx = (T + rows_per_wg - 1) / rows_per_wg;
                const int64_t by = (width + (int64_t{4} << tpr_log2) - 1) / (int64_t{4} << tpr_log2);
                gx = bx > gx ? bx : gx;
                gy = by > gy ? by : gy;
                off += width;
            }
            if (one_launch) {
                const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(gy),
                                static_cast<unsigned>(count));
                pack_txm_group_kernel<<<grid, 256, 0, s>>>(sets, T, p.rp, panel);
            }
        }
        int64_t off = 0;
        for (int i = 0; i < count && T > 0 && !one_launch; ++i) {
            // the last set also zero-fills the panel's padding columns
            const int64_t width = i + 1 == count ? p.rp - off : (seg[i].rows + 7) / 8 * 8;
            if (width > 0) {
                const int64_t m_src = seg[i].src_rows;  // row length of this set's dY
                if (staged(i, width)) {
                    // wide rows: staged through LDS (streaming loads of whole rows)
                    const auto* src = static_cast<const uint16_t*>(seg[i].dY);
                    const size_t row_bytes = static_cast<size_t>(pack_stage_row_elems(m_src)) * 2;
                    if (m_src < kPackStageDeepMinM)
                        pack_txm_staged_kernel<2, 1><<<static_cast<unsigned>((T + 1) / 2), 256, 2 * row_bytes, s>>>(
                            src, seg[i].ldy, T, m_src, seg[i].idx, seg[i].rows, width, p.rp, panel + off);
                    else if (m_src <= kPackStageTwoRowsMaxM)
                        pack_txm_staged_kernel<2, 4><<<static_cast<unsigned>((T + 1) / 2), 256, 2 * row_bytes, s>>>(
                            src, seg[i].ldy, T, m_src, seg[i].idx, seg[i].rows, width, p.rp, panel + off);
                    else
                        pack_txm_staged_kernel<1, 4><<<static_cast<unsigned>(T), 256, row_bytes, s>>>(
                            src, seg[i].ldy, T, m_src, seg[i].idx, seg[i].rows, width, p.rp, panel + off);
                } else if (layout == GRASS_DY_TxM) {
                    const int tpr_log2 = threads_per_row_log2(width);
                    const int64_t gx = (width + (int64_t{4} << tpr_log2) - 1) / (int64_t{4} << tpr_log2);
                    const int64_t rows_per_wg = static_cast<int64_t>(kPackRows) * (256 >> tpr_log2);
                    const dim3 grid(static_cast<unsigned>((T + rows_per_wg - 1) / rows_per_wg),
                                    static_cast<unsigned>(gx));
                    pack_txm_kernel<<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(seg[i].dY),
                                                         seg[i].ldy, T, seg[i].idx, seg[i].rows,
                                                         width, p.rp, tpr_log2, panel + off);
                } else if (aligned_to(seg[i].dY, 16) && seg[i].ldy % 8 == 0 && p.rp % 8 == 0 &&
                           width % 8 == 0) {
                    const dim3 grid(static_cast<unsigned>((T + kPackWideT - 1) / kPackWideT),
                                    static_cast<unsigned>((width + kPackWideJ - 1) / kPackWideJ));
                    pack_mxt_wide_kernel<<<grid, 256, 0, s>>>(
                        static_cast<const uint16_t*>(seg[i].dY), seg[i].ldy, T, seg[i].idx,
                        seg[i].rows, width, p.rp, panel + off);
                } else {
                    const dim3 grid(static_cast<unsigned>((T + 63) / 64),
                                    static_cast<unsigned>((width + 63) / 64));
                    pack_mxt_kernel<<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(seg[i].dY),
                                                         seg[i].ldy, T, seg[i].idx, seg[i].rows,
                                                         width, p.rp, panel + off);
                }
            }
            off += width;
        }
        g.A = panel;
        g.lda = p.rp;
        g.Mcols = p.rp;
        g.a_fast = 1;
    } else {
        g.A = static_cast<const uint16_t*>(dY0);
        g.lda = ldy0;
        g.Mcols = total;
        g.a_fast = aligned_to(dY0, 16) && ldy0 % 8 == 0;
    }
    g.a_rows = a_rows_form ? seg[0].idx : nullptr;
    if (copy_x) {
        uint16_t* xa = reinterpret_cast<uint16_t*>(base + p.pack_bytes + round_up(p.partial_bytes, 256));
        align_rows_kernel<<<static_cast<unsigned>(T * x_chunks), 256, 0, s>>>(
            static_cast<const uint16_t*>(X), ldx, T, n, nb, x_chunks, xa);
        g.B = xa;
        g.ldb = nb;
        g.Ncols = nb;
        g.b_fast = 1;
    } else {
        g.B = static_cast<const uint16_t*>(X);
        g.ldb = ldx;
        g.Ncols = n;
        g.b_fast = aligned_to(X, 16) && ldx % 8 == 0;
    }
    g.P = partial;
    g.K = T_main;
    g.Mp = p.Mp;
    g.Np = p.Np;
    g.tiles_m = p.tiles_m;
    g.tiles_n = p.tiles_n;
    g.splits = p.splits;
    g.ktiles_per_split = p.ktiles_per_split;

    const unsigned grid = static_cast<unsigned>(chunk * kNumXcd);
    hipError_t le;
    if (tile == kTile256) {  // the events are stamped with this dispatch's own start and end
        if (a_pairs)
            launch_stamped(tn_gemm_bf16_direct_kernel<false, false, true, true>, dim3(grid), dim3(256), 0, s,
                           ev_start, ev_stop, g);
        else if (a_rows_form)
            launch_stamped(tn_gemm_bf16_direct_kernel<false, false, true>, dim3(grid), dim3(256), 0, s,
                           ev_start, ev_stop, g);
        else if (gathered)
            launch_stamped(tn_gemm_bf16_direct_kernel<false>, dim3(grid), dim3(256), 0, s, ev_start, ev_stop, g);
        else
            launch_stamped(tn_gemm_bf16_direct_kernel<true>, dim3(grid), dim3(256), 0, s, ev_start, ev_stop, g);
        le = hipSuccess;
    } else {
        if (ev_start) (void)hipEventRecord(ev_start, s);
        le = gathered ? launch_gemm_kernel<Cfg128, false>(g, grid, s)
                      : launch_gemm_kernel<Cfg128, true>(g, grid, s);
        if (le == hipSuccess && ev_stop) (void)hipEventRecord(ev_stop, s);
    }
    if (le != hipSuccess) return GRASS_ERR_DEVICE;
    int slices = p.splits;
    if (T_main < T) {  // rows [T_main, T) as one more slice, computed with 128 x 128 tiles
        GemmArgs t = g;
        t.A = g.A + T_main * g.lda;
        t.B = g.B + T_main * g.ldb;
        t.K = T - T_main;
        t.P = partial + static_cast<int64_t>(p.splits) * p.Mp * p.Np;
        t.tiles_m = static_cast<int>(p.Mp / Cfg128::BM);
        t.tiles_n = static_cast<int>(p.Np / Cfg128::BN);
        t.splits = 1;
        t.ktiles_per_split = 1;
        t.a_fast = t.b_fast = 1;
        const int64_t titems = static_cast<int64_t>(t.tiles_m) * t.tiles_n;
        const unsigned tgrid = static_cast<unsigned>((titems + kNumXcd - 1) / kNumXcd * kNumXcd);
        le = gathered ? launch_gemm_kernel<Cfg128, false>(t, tgrid, s)
                      : launch_gemm_kernel<Cfg128, true>(t, tgrid, s);
        if (le != hipSuccess) return GRASS_ERR_DEVICE;
        ++slices;
    }

    return finish_segments(seg, count, partial, slices, p.Mp, p.Np, n, odt, s, ev_tail_start, ev_tail_stop);
}

grass_status launch_tn_gemm(const void* dY, grass_dy_layout layout, int64_t ldy, const void* X,
                            int64_t ldx, grass_dtype dt, int64_t T, int64_t mrows, int64_t n,
                            const int32_t* idx, const float* rho, void* C, grass_dtype odt,
                            int64_t ldc, void* ws, hipStream_t s, int64_t src_rows,
                            hipEvent_t ev_start, hipEvent_t ev_stop) {
    const GemmSegment one{dY, ldy, idx, rho, C, ldc, mrows, src_rows};
    return launch_tn_gemm_segments(&one, 1, layout, X, ldx, dt, T, n, odt, ws, s, ev_start, ev_stop);
}

}  // namespace grass
