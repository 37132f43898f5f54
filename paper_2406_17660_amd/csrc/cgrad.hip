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
//   2. GEMM:   v_mfma_f32_32x32x16_bf16 tiles.  Global tiles [BK x BM] / [BK x BN] are staged
//              through LDS in their memory order (t-major) with 16-byte loads; the MFMA
//              operand layout (8 consecutive t per lane) is produced by the gfx950
//              transposing LDS read ds_read_b64_tr_b16, so no transpose is ever
//              materialised.  Split-K over T fills the 256 CUs; work items are numbered
//              so that the workgroups an XCD receives share one K slice (L2 reuse).
//   3. reduce: sums the split-K partials in a fixed order (deterministic), applies rho and
//              converts to the output dtype.
// fp32 path: a plain LDS-tiled FMA kernel (small reference-precision configurations).
#include "common.hpp"

namespace grass {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;

constexpr int kNumXcd = 8;

// Tile numbering inside one K slice: panels of four tile rows, column-major inside a panel,
// so that a run of consecutive tile numbers (what one XCD receives) forms a compact block
// and re-reads as little of A and B as possible through that XCD's L2.
__device__ __forceinline__ void tile_coords(int tile, int tiles_m, int tiles_n, int& tm, int& tn) {
    constexpr int kPanel = 4;
    const int per_panel = kPanel * tiles_n;
    const int panel = tile / per_panel;
    const int rows_here = tiles_m - panel * kPanel < kPanel ? tiles_m - panel * kPanel : kPanel;
    const int in_panel = tile - panel * per_panel;
    tm = panel * kPanel + in_panel % rows_here;
    tn = in_panel / rows_here;
}

// ------------------------------------------------------------------------------ pack
// out[t, j] = dY[t, idx[j]] (j < r; idx == nullptr: column j itself), 0 for r <= j < rp; rows
// of `out` are ldo apart (several matrices may fill adjacent column ranges of one panel).
// Thread = 4 adjacent j; 2^tpr_log2 threads cover the columns of one row of t (a narrow panel,
// r = 128 say, puts several rows of t side by side in a workgroup instead of idling most of
// it), and every thread loops over rows_per_thread (4 .. kPackRows) values of t: fewer when
// the matrix is small, so that the launch still has a few thousand workgroups to hide the
// latency of the gather.  Wave stores are contiguous.
constexpr int kPackRows = 16;
__global__ __launch_bounds__(256) void pack_txm_kernel(const uint16_t* __restrict__ dY, int64_t ldy,
                                                       int64_t T, const int32_t* __restrict__ idx,
                                                       int64_t r, int64_t rp, int64_t ldo,
                                                       int tpr_log2, int rows_per_thread,
                                                       uint16_t* __restrict__ out) {
    const int tpr = 1 << tpr_log2, rows_per_pass = 256 >> tpr_log2;
    const int64_t j0 = (static_cast<int64_t>(blockIdx.x) * tpr + (threadIdx.x & (tpr - 1))) * 4;
    if (j0 >= rp) return;
    int64_t col[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) col[e] = j0 + e < r ? (idx ? idx[j0 + e] : j0 + e) : -1;
    const int64_t t0 = static_cast<int64_t>(blockIdx.y) * rows_per_thread * rows_per_pass +
                       (threadIdx.x >> tpr_log2);
#pragma unroll 4
    for (int tt = 0; tt < rows_per_thread; ++tt) {
        const int64_t t = t0 + static_cast<int64_t>(tt) * rows_per_pass;
        if (t >= T) break;
        const uint16_t* row = dY + t * ldy;
        uint16_t v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = col[e] >= 0 ? row[col[e]] : static_cast<uint16_t>(0);
        uint2 w;
        w.x = v[0] | (static_cast<uint32_t>(v[1]) << 16);
        w.y = v[2] | (static_cast<uint32_t>(v[3]) << 16);
        *reinterpret_cast<uint2*>(out + t * ldo + j0) = w;
    }
}

// out[t, j] = dYt[idx[j] (or j), t]: gather of rows of the m x T matrix, transposed through
// a 64 x 64 LDS tile so that both the reads (along t) and the writes (along j) coalesce.
__global__ __launch_bounds__(256) void pack_mxt_kernel(const uint16_t* __restrict__ dYt, int64_t ldy,
                                                       int64_t T, const int32_t* __restrict__ idx,
                                                       int64_t r, int64_t rp, int64_t ldo,
                                                       uint16_t* __restrict__ out) {
    __shared__ uint16_t tile[64][66];
    const int64_t j0 = static_cast<int64_t>(blockIdx.x) * 64;
    const int64_t t0 = static_cast<int64_t>(blockIdx.y) * 64;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (int jj = w; jj < 64; jj += 4) {
        const int64_t j = j0 + jj, t = t0 + lane;
        uint16_t v = 0;
        if (j < r && t < T) v = dYt[static_cast<int64_t>(idx ? idx[j] : j) * ldy + t];
        tile[jj][lane] = v;
    }
    __syncthreads();
    for (int tt = w; tt < 64; tt += 4) {
        const int64_t t = t0 + tt, j = j0 + lane;
        if (t < T && j < rp) out[t * ldo + j] = tile[lane][tt];
    }
}

// The same gather-and-transpose with 16-byte accesses on both sides, for rows that allow them
// (dYt 16-byte aligned, ldy and ldo multiples of 8).  A workgroup turns 64 (j) x 256 (t): each
// lane loads 8 consecutive t of one selected row (a wavefront reads 2 x 512 contiguous bytes),
// the block goes to LDS as [j][t], and the transposing 8-byte LDS read hands every lane four
// consecutive j of one t, so a lane stores 8 values of j (16 bytes) of its own panel row per
// step.  LDS rows are padded by 16 elements: the four rows one 16-lane read touches then fall
// into different banks.
constexpr int kPackWideJ = 64, kPackWideT = 256, kPackWideLd = kPackWideT + 16;
__global__ __launch_bounds__(256) void pack_mxt_wide_kernel(const uint16_t* __restrict__ dYt,
                                                            int64_t ldy, int64_t T,
                                                            const int32_t* __restrict__ idx,
                                                            int64_t r, int64_t rp, int64_t ldo,
                                                            uint16_t* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[kPackWideJ * kPackWideLd];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t j0 = static_cast<int64_t>(blockIdx.x) * kPackWideJ;
    const int64_t t0 = static_cast<int64_t>(blockIdx.y) * kPackWideT;
    const int chunk = threadIdx.x & 31;  // 8 values of t each
#pragma unroll
    for (int pass = 0; pass < kPackWideJ / 8; ++pass) {
        const int jj = pass * 8 + (threadIdx.x >> 5);
        const int64_t j = j0 + jj, t = t0 + chunk * 8;
        s16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (j < r && t < T) {
            const uint16_t* src = dYt + static_cast<int64_t>(idx ? idx[j] : j) * ldy + t;
            if (t + 8 <= T) {
                v = *reinterpret_cast<const s16x8*>(src);
            } else {
                for (int e = 0; e < 8; ++e)
                    if (t + e < T) v[e] = static_cast<short>(src[e]);
            }
        }
        *reinterpret_cast<s16x8*>(tile + jj * kPackWideLd + chunk * 8) = v;
    }
    __syncthreads();
    // wavefront w owns t = 64w .. 64w+63 of the block; lane L ends up with t = 64w + L
    const int grp = lane >> 4, i = lane & 15;
    const uint16_t* src = tile + (i >> 2) * kPackWideLd + w * 64 + grp * 16 + 4 * (i & 3);
    const int64_t t = t0 + w * 64 + lane;
    uint16_t* dst = out + (t < T ? t : 0) * ldo + j0;
#pragma unroll
    for (int j8 = 0; j8 < kPackWideJ; j8 += 8) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(src + j8 * kPackWideLd));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(src + (j8 + 4) * kPackWideLd));
        if (t < T && j0 + j8 < rp)  // rp is a multiple of 8: whole vectors only
            *reinterpret_cast<s16x8*>(dst + j8) = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
}

// out[t, c] = in[t, c] for c < n and 0 for n <= c < np (np even, rows of `out` np apart): a copy
// of a matrix whose rows start at odd element offsets (n not a multiple of 8, as in the
// 5461-wide MLP of the 1B model) into rows the 16-byte loads of the GEMM can take.  `in` itself
// is 4-byte aligned.  A thread moves one 32-bit pair at a time; a row that starts in the upper
// half of an aligned word is read as two words and shifted.
__global__ __launch_bounds__(256) void align_rows_kernel(const uint16_t* __restrict__ in, int64_t ld,
                                                         int64_t n, int64_t np, int chunks,
                                                         uint16_t* __restrict__ out) {
    const int64_t t = blockIdx.x / chunks;
    const int chunk = blockIdx.x % chunks;
    const uint16_t* row = in + t * ld;
    const uintptr_t a = reinterpret_cast<uintptr_t>(row);
    const bool upper = (a & 2) != 0;
    const uint32_t* w = reinterpret_cast<const uint32_t*>(a - (upper ? 2 : 0));
    uint32_t* o = reinterpret_cast<uint32_t*>(out + t * np);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t d = static_cast<int64_t>(chunk) * 1024 + i * 256 + threadIdx.x;
        const int64_t c = 2 * d;
        if (c >= np) break;
        uint32_t v;
        if (upper ? c + 2 < n : c + 1 < n) {  // every word touched lies inside the row
            v = upper ? (w[d] >> 16) | (w[d + 1] << 16) : w[d];
        } else {
            const uint32_t lo = c < n ? row[c] : 0u, hi = c + 1 < n ? row[c + 1] : 0u;
            v = lo | (hi << 16);
        }
        o[d] = v;
    }
}

// ------------------------------------------------------------------------------ bf16 MFMA GEMM
// One 16-byte chunk (8 bf16) of row `krow` starting at column `col` of a [K x ncols] matrix,
// zero outside the matrix.
__device__ __forceinline__ uint4 load_chunk(const uint16_t* __restrict__ base, int64_t ld,
                                            int64_t krow, int64_t col, int64_t K, int64_t ncols,
                                            bool fast) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (krow >= K || col >= ncols) return v;
    const uint16_t* p = base + krow * ld + col;
    if (fast && col + 8 <= ncols) return *reinterpret_cast<const uint4*>(p);
    uint16_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = col + i < ncols ? p[i] : static_cast<uint16_t>(0);
    v.x = e[0] | (static_cast<uint32_t>(e[1]) << 16);
    v.y = e[2] | (static_cast<uint32_t>(e[3]) << 16);
    v.z = e[4] | (static_cast<uint32_t>(e[5]) << 16);
    v.w = e[6] | (static_cast<uint32_t>(e[7]) << 16);
    return v;
}

template <int BM_, int BN_, int BK_, int WR_, int WC_>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WR = WR_, WC = WC_;
    static constexpr int kThreads = 64 * WR * WC;
    static constexpr int WM = BM / WR, WN = BN / WC;  // wave tile
    static constexpr int FM = WM / 32, FN = WN / 32;  // 32x32 MFMA fragments per wave
    static constexpr int PAD = 16;                    // elements; keeps rows 32 B apart mod 128 B
    static constexpr int LDA = BM + PAD, LDB = BN + PAD;
    static constexpr int A_CHUNKS = BK * BM / 8 / kThreads;  // 16-byte chunks per thread
    static constexpr int B_CHUNKS = BK * BN / 8 / kThreads;
    static constexpr size_t kLdsBytes = static_cast<size_t>(BK) * (LDA + LDB) * 2;
    static constexpr int kWgPerCu = 2;
    static constexpr bool kWholeKTilesOnly = false;
    static_assert(BK % 16 == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    static_assert((BK * BM / 8) % kThreads == 0 && (BK * BN / 8) % kThreads == 0, "chunking");
};

// Operand fragment for v_mfma_f32_32x32x16_bf16 from a t-major LDS tile: lane l needs the 8
// values tile[k16 + 8*(l/32) + 0..7][c0 + l%32].  ds_read_b64_tr_b16 hands lane L of each
// 16-lane group the four values found at column (L%16) of the four rows addressed by lanes
// 4e + L/4... concretely: lane i of the group supplies the address of row (i/4), columns
// 4*(i%4)..+3, and receives column i of rows 0..3.  Two such reads give the 8 values.
__device__ __forceinline__ bf16x8 read_frag(const uint16_t* tile, int ld, int k16, int c0) {
    const int l = threadIdx.x & 63;
    const int L = l & 15;
    const int row = k16 + 8 * (l >> 5) + (L >> 2);
    const int col = c0 + 16 * ((l >> 4) & 1) + 4 * (L & 3);
    const uint16_t* p = tile + row * ld + col;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * ld));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

struct GemmArgs {
    const uint16_t* A;  // [K x Mcols], leading dimension lda
    const uint16_t* B;  // [K x Ncols], leading dimension ldb
    float* P;           // partials [S][Mp][Np]
    int64_t lda, ldb, K, Mcols, Ncols, Mp, Np;
    int tiles_m, tiles_n, splits, ktiles_per_split;
    int a_fast, b_fast;
    // row form of the left operand (large-tile kernel only): A is [rows of length K], row j of
    // the product is A + a_rows[j] * lda (a_rows == nullptr: row j itself)
    const int32_t* a_rows;
};

// kDense only tags the instantiation (dense full gradient vs compressed gradient) so that a
// profiler lists the two uses separately; the code is identical.
template <typename Cfg, bool kDense>
__global__ __launch_bounds__(Cfg::kThreads) void tn_gemm_bf16_kernel(GemmArgs g) {
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* As = lds;
    uint16_t* Bs = lds + Cfg::BK * Cfg::LDA;

    // Work numbering: consecutive items share a K slice and neighbouring tiles.  Workgroup
    // b lands on XCD b % 8, so XCD x is handed the contiguous item range [x*chunk, (x+1)*chunk).
    const int64_t items = static_cast<int64_t>(g.tiles_m) * g.tiles_n * g.splits;
    const int64_t chunk = (items + kNumXcd - 1) / kNumXcd;
    const int64_t item = static_cast<int64_t>(blockIdx.x % kNumXcd) * chunk + blockIdx.x / kNumXcd;
    if (item >= items) return;
    const int tiles = g.tiles_m * g.tiles_n;
    const int split = static_cast<int>(item / tiles);
    const int tile = static_cast<int>(item % tiles);
    int tm, tn;
    tile_coords(tile, g.tiles_m, g.tiles_n, tm, tn);
    const int64_t m0 = static_cast<int64_t>(tm) * Cfg::BM, n0 = static_cast<int64_t>(tn) * Cfg::BN;
    const int64_t kt_begin = static_cast<int64_t>(split) * g.ktiles_per_split;
    const int64_t ktiles_all = (g.K + Cfg::BK - 1) / Cfg::BK;
    int64_t kt_end = kt_begin + g.ktiles_per_split;
    if (kt_end > ktiles_all) kt_end = ktiles_all;

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int wr = wave % Cfg::WR, wc = wave / Cfg::WR;

    f32x16 acc[Cfg::FM][Cfg::FN];
#pragma unroll
    for (int i = 0; i < Cfg::FM; ++i)
#pragma unroll
        for (int j = 0; j < Cfg::FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 ra[Cfg::A_CHUNKS], rb[Cfg::B_CHUNKS];
    constexpr int ACPR = Cfg::BM / 8, BCPR = Cfg::BN / 8;  // chunks per tile row

    auto fetch = [&](int64_t kt) {
        const int64_t k0 = kt * Cfg::BK;
#pragma unroll
        for (int c = 0; c < Cfg::A_CHUNKS; ++c) {
            const int id = tid + c * Cfg::kThreads;
            ra[c] = load_chunk(g.A, g.lda, k0 + id / ACPR, m0 + (id % ACPR) * 8, g.K, g.Mcols,
                               g.a_fast);
        }
#pragma unroll
        for (int c = 0; c < Cfg::B_CHUNKS; ++c) {
            const int id = tid + c * Cfg::kThreads;
            rb[c] = load_chunk(g.B, g.ldb, k0 + id / BCPR, n0 + (id % BCPR) * 8, g.K, g.Ncols,
                               g.b_fast);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int c = 0; c < Cfg::A_CHUNKS; ++c) {
            const int id = tid + c * Cfg::kThreads;
            *reinterpret_cast<uint4*>(As + (id / ACPR) * Cfg::LDA + (id % ACPR) * 8) = ra[c];
        }
#pragma unroll
        for (int c = 0; c < Cfg::B_CHUNKS; ++c) {
            const int id = tid + c * Cfg::kThreads;
            *reinterpret_cast<uint4*>(Bs + (id / BCPR) * Cfg::LDB + (id % BCPR) * 8) = rb[c];
        }
    };

    if (kt_begin < kt_end) {
        fetch(kt_begin);
        stash();
        __syncthreads();
        for (int64_t kt = kt_begin; kt < kt_end; ++kt) {
            const bool more = kt + 1 < kt_end;
            if (more) fetch(kt + 1);  // global loads in flight while the MFMAs run
#pragma unroll
            for (int k16 = 0; k16 < Cfg::BK; k16 += 16) {
                bf16x8 af[Cfg::FM], bfr[Cfg::FN];
#pragma unroll
                for (int i = 0; i < Cfg::FM; ++i)
                    af[i] = read_frag(As, Cfg::LDA, k16, wr * Cfg::WM + i * 32);
#pragma unroll
                for (int j = 0; j < Cfg::FN; ++j)
                    bfr[j] = read_frag(Bs, Cfg::LDB, k16, wc * Cfg::WN + j * 32);
#pragma unroll
                for (int i = 0; i < Cfg::FM; ++i)
#pragma unroll
                    for (int j = 0; j < Cfg::FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j],
                                                                            acc[i][j], 0, 0, 0);
            }
            __syncthreads();
            if (more) {
                stash();
                __syncthreads();
            }
        }
    }

    // Partial tile -> P[split].  Accumulator element v of lane l is C[8*(v/4) + 4*(l/32) +
    // v%4][l%32] of its 32x32 fragment.  The partial buffer is padded to whole tiles.
    const int l = tid & 63;
    float* P = g.P + (static_cast<int64_t>(split) * g.Mp + m0 + wr * Cfg::WM) * g.Np + n0 +
               wc * Cfg::WN;
#pragma unroll
    for (int i = 0; i < Cfg::FM; ++i)
#pragma unroll
        for (int j = 0; j < Cfg::FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = i * 32 + 8 * (v / 4) + 4 * (l >> 5) + (v % 4);
                P[static_cast<int64_t>(row) * g.Np + j * 32 + (l & 31)] = acc[i][j][v];
            }
}

// ------------------------------------------------------------------------------ bf16 MFMA GEMM, large tiles
// 256 x 256 output tile, four wavefronts in a 2 x 2 arrangement, each owning a 128 x 128
// block (16 accumulator fragments = 256 registers per lane, one wavefront per SIMD).
//
// Global -> LDS copies use the gfx950 16-byte load-to-LDS instruction, which needs no
// staging registers: a wavefront load writes 1 KiB of consecutive LDS (two 512-byte tile
// rows), each lane choosing its own global address.  K advances in tiles of 32 rows held
// in a ring of four LDS stages (4 x 32 KiB): while tile kt is multiplied the loads of tiles
// kt+1 .. kt+3 are in flight, which covers the L2/HBM latency with a single wavefront per
// SIMD.  One barrier per K tile; the wait before it is s_waitcnt vmcnt(N) with N = the
// loads issued for the younger tiles (the counter retires in order).
//
// LDS rows are not padded (the load-to-LDS destination is contiguous); instead the
// 16-byte slots of row k are permuted by XOR with 4*(k mod 4).  The lane that fills
// physical slot p of row k therefore fetches logical slot p ^ 4*(k%4) from global memory,
// and the transposing LDS reads apply the same XOR.  One ds_read_b64_tr_b16 of a
// wavefront touches 8 rows x 64 B; with the permutation every half-wavefront covers all 64
// banks exactly once.
//
// Edges.  Columns past the matrix edge are redirected to column 0 of the same row: they
// only feed output rows / columns that are never read back.  Only whole K tiles are
// processed (g.K is a multiple of kFastBK here; the launcher hands a ragged tail of T to
// the small-tile kernel as one more split-K slice).
// Requirements (checked by the launcher): bases 16-byte aligned, leading dimensions and
// column counts multiples of 8.
constexpr int kFastBM = 256, kFastBN = 256, kFastBK = 32, kFastStages = 4;
constexpr int kFastOperandElems = kFastBK * 256;          // one operand of one stage
constexpr int kFastStageElems = 2 * kFastOperandElems;    // A then B
constexpr int kFastLoadsPerTile = 2 * (kFastBK / 8);      // load-to-LDS instructions per wavefront

typedef __attribute__((address_space(3))) void lds_void_t;

// 16 bytes per lane from global memory straight into LDS: lane i of the wavefront writes
// LDS bytes [lds_base + 16*i, +16).  Written as inline assembly so that the compiler's
// automatic wait-count insertion does not see the transfer: it cannot tell the ring stages
// apart and would wait for ALL outstanding loads before the first LDS read of every
// stage, which serialises the pipeline.  The waits are placed by hand (wait_vmcnt below).
// The global address is a wavefront-uniform 64-bit base (scalar registers) plus a 32-bit
// per-lane byte offset, so advancing to the next K tile costs two scalar adds and no
// vector arithmetic.
__device__ __forceinline__ void load16_to_lds(const void* base, uint32_t lane_offset,
                                              uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_offset), "s"(base), "s"(lds_base)
                 : "memory", "m0");
}

__device__ __forceinline__ bf16x8 read_frag_swz(const uint16_t* p) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * 256));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in bits
// 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// kRowStats: instead of storing its output tile, the workgroup squares it and sums it along
// each row (columns past the matrix edge excluded) and stores 256 partial row sums per
// half-tile of columns: the row statistic of G without G ever being written.  Only valid
// with a single K slice.
//
// kARows: the left operand is given as rows of length K (dY stored m x T) and the selected rows
// are gathered by the tile loads themselves: row j of the tile is the 64 contiguous bytes
// A[a_rows[j]][k0 .. k0+32).  Its LDS block is [256 rows][32 k] (64 bytes per row, 16-byte
// slot c of row j stored at slot c ^ ((j / 4) % 4), so that the 16 lanes of a quarter
// wavefront, which read one slot of 16 consecutive rows, cover all 64 banks once) and an MFMA
// operand is a single 16-byte read per lane: no transposition is needed, the 8 consecutive k
// a lane feeds to the matrix core are contiguous in the row.
template <bool kDense, bool kRowStats = false, bool kARows = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void tn_gemm_bf16_direct_kernel(GemmArgs g) {
    __shared__ __attribute__((aligned(1024))) uint16_t ring[kFastStages * kFastStageElems];

    const int64_t items = static_cast<int64_t>(g.tiles_m) * g.tiles_n * g.splits;
    const int64_t chunk_items = (items + kNumXcd - 1) / kNumXcd;
    const int64_t item =
        static_cast<int64_t>(blockIdx.x % kNumXcd) * chunk_items + blockIdx.x / kNumXcd;
    if (item >= items) return;
    const int tiles = g.tiles_m * g.tiles_n;
    const int split = static_cast<int>(item / tiles);
    const int tile = static_cast<int>(item % tiles);
    int tm, tn;
    tile_coords(tile, g.tiles_m, g.tiles_n, tm, tn);
    const int64_t m0 = static_cast<int64_t>(tm) * kFastBM, n0 = static_cast<int64_t>(tn) * kFastBN;
    const int64_t kt_begin = static_cast<int64_t>(split) * g.ktiles_per_split;
    const int64_t ktiles_all = g.K / kFastBK;
    int64_t kt_end = kt_begin + g.ktiles_per_split;
    if (kt_end > ktiles_all) kt_end = ktiles_all;
    const int ntiles = kt_end > kt_begin ? static_cast<int>(kt_end - kt_begin) : 0;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave & 1, wc = wave >> 1;

    // ---- global -> LDS addressing: this lane fills physical slot `slot` of row lrow (+8 per pass)
    const int lrow = wave * 2 + (lane >> 5);
    const int slot = lane & 31;
    const int lchunk_g = slot ^ (4 * (lrow & 3));
    int64_t colA = m0 + lchunk_g * 8, colB = n0 + lchunk_g * 8;
    if (colA >= g.Mcols) colA = 0;
    if (colB >= g.Ncols) colB = 0;
    // uniform tile base (advances by one K tile per issue) + constant per-lane byte offsets
    const uint16_t* gA = g.A + (kARows ? kt_begin * kFastBK : kt_begin * kFastBK * g.lda);
    const uint16_t* gB = g.B + kt_begin * kFastBK * g.ldb;
    uint32_t laneA[kFastBK / 8], laneB[kFastBK / 8];
#pragma unroll
    for (int p = 0; p < kFastBK / 8; ++p) {
        if (kARows) {
            // pass p: this wavefront fills tile rows 64p + 16*wave .. +16, four lanes per row
            const int trow = 64 * p + 16 * wave + (lane >> 2);
            int64_t j = m0 + trow;
            if (j >= g.Mcols) j = 0;  // rows past the edge only feed outputs nobody reads
            const int64_t src = g.a_rows ? g.a_rows[j] : j;
            const int lslot = (lane & 3) ^ ((trow >> 2) & 3);
            laneA[p] = static_cast<uint32_t>((src * g.lda + lslot * 8) * 2);
        } else {
            laneA[p] = static_cast<uint32_t>(((p * 8 + lrow) * g.lda + colA) * 2);
        }
        laneB[p] = static_cast<uint32_t>(((p * 8 + lrow) * g.ldb + colB) * 2);
    }
    const int64_t tileA = kARows ? kFastBK : kFastBK * g.lda, tileB = kFastBK * g.ldb;
    const int ldsrow = wave * 2;  // first LDS row this wavefront writes in a pass

    // Loads of K tile number `i` (counted from this workgroup's first tile) into its ring
    // stage, split into kFastLoadsPerTile single instructions (part = 0..7: A rows 8p.., then
    // B rows) so that the main loop can space them out between MFMA groups: the four
    // wavefronts of a workgroup share one address unit, and eight back-to-back 1 KiB loads
    // from each of them right after a barrier stall the last wavefront's MFMAs.
    const uint32_t ring_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void_t*)ring));
    auto issue_part = [&](int i, int part) {
        const uint32_t d = ring_base + ((i % kFastStages) * kFastStageElems + ldsrow * 256) * 2;
        if (part < kFastBK / 8)  // both forms: pass `part` of this wavefront starts 4 KiB further
            load16_to_lds(gA, laneA[part], d + part * 8 * 256 * 2);
        else
            load16_to_lds(gB, laneB[part - kFastBK / 8],
                          d + kFastOperandElems * 2 + (part - kFastBK / 8) * 8 * 256 * 2);
    };
    auto advance_tile = [&]() { gA += tileA; gB += tileB; };
    auto issue = [&](int i) {
#pragma unroll
        for (int part = 0; part < kFastLoadsPerTile; ++part) issue_part(i, part);
        advance_tile();
    };

    // ---- LDS -> MFMA operand addressing (element offsets inside an operand block)
    const int L = lane & 15, g2 = (lane >> 4) & 1, h = lane >> 5;
    const int rrow = 8 * h + (L >> 2);
    const int swz = 4 * (L >> 2);
    const int lchunk = 2 * g2 + ((L & 3) >> 1);
    const int half = (L & 1) * 4;
    int offA[4], offB[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (kARows)  // row wr*128 + 32i + lane%32, slot (k16/8 + lane/32) ^ ((row/4)%4); k16 added later
            offA[i] = (wr * 128 + i * 32 + (lane & 31)) * kFastBK + ((h ^ (((lane & 31) >> 2) & 3)) * 8);
        else
            offA[i] = rrow * 256 + ((((wr * 128 + i * 32) >> 3) ^ swz) + lchunk) * 8 + half;
        offB[i] = kFastOperandElems + rrow * 256 +
                  ((((wc * 128 + i * 32) >> 3) ^ swz) + lchunk) * 8 + half;
    }

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Operand fragments of one k16 slice of a tile: A rows 4 x 32, B columns 4 x 32.
    struct Frags { bf16x8 a[4], b[4]; };
    // Quarter `part` of the fragment reads of a slice, in the order the MFMAs consume them
    // (a0 b0 | b1 b2 | b3 a1 | a2 a3): two fragments = four transposing LDS reads.
    auto read_a = [&](int i, int k16, int a) -> bf16x8 {
        if (kARows) {  // slots 2, 3 hold k16 = 16: flipping bit 1 of the slot = element offset ^ 16
            const uint16_t* sa = ring + (i % kFastStages) * kFastStageElems + (offA[a] ^ k16);
            return *reinterpret_cast<const lds_bf16x8*>((lds_void_t*)sa);
        }
        return read_frag_swz(ring + (i % kFastStages) * kFastStageElems + k16 * 256 + offA[a]);
    };
    auto read_quarter = [&](Frags& f, int i, int k16, int part) {
        const uint16_t* st = ring + (i % kFastStages) * kFastStageElems + k16 * 256;
        if (part == 0) { f.a[0] = read_a(i, k16, 0); f.b[0] = read_frag_swz(st + offB[0]); }
        else if (part == 1) { f.b[1] = read_frag_swz(st + offB[1]); f.b[2] = read_frag_swz(st + offB[2]); }
        else if (part == 2) { f.b[3] = read_frag_swz(st + offB[3]); f.a[1] = read_a(i, k16, 1); }
        else { f.a[2] = read_a(i, k16, 2); f.a[3] = read_a(i, k16, 3); }
    };
    auto read_frags = [&](Frags& f, int i, int k16) {
#pragma unroll
        for (int part = 0; part < 4; ++part) read_quarter(f, i, k16, part);
    };
    // Row `a` of the 4 x 4 fragment products of a slice.
    auto mfma_row = [&](const Frags& f, int a) {
#pragma unroll
        for (int b = 0; b < 4; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[a], f.b[b], acc[a][b], 0, 0, 0);
    };
    auto mfma16 = [&](const Frags& f) {
#pragma unroll
        for (int a = 0; a < 4; ++a) mfma_row(f, a);
    };
    // "one MFMA, one LDS read" four times: the reads issue in the shadow of the MFMAs
    auto interleave_hint4 = [&]() {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
        }
    };
    // One slice of work: the 16 MFMAs of `cur` in four groups of four, each group overlapped
    // with a quarter of the LDS reads of the following slice (`next`) and followed by one
    // global->LDS load of tile `load_tile` (if any).
    auto slice = [&](const Frags& cur, Frags& next, int next_tile, int next_k16, int load_tile,
                     int load_part0, bool do_load) {
#pragma unroll
        for (int part = 0; part < 4; ++part) {
            read_quarter(next, next_tile, next_k16, part);
            mfma_row(cur, part);
            interleave_hint4();
            __builtin_amdgcn_sched_barrier(0);
            if (do_load) issue_part(load_tile, load_part0 + part);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Software pipeline.  Each K tile has two k16 slices.  While the MFMAs of one slice run,
    // the fragments of the next slice are read from LDS into the other fragment set, so the
    // matrix pipe only idles at the barrier.  Loads run kAhead tiles ahead of the MFMAs.
    //
    //   iteration i:  wait(tile i landed) ; barrier
    //                 MFMA on G = slice (i-1,1)  ||  F <- slice (i,0)  ||  A loads of tile i+kAhead
    //                 MFMA on F                  ||  G <- slice (i,1)  ||  B loads of tile i+kAhead
    //   The loads overwrite the stage of tile i-1, whose last LDS reads were issued (and
    //   waited for) before the barrier.
    constexpr int kAhead = kFastStages - 1;
    static_assert(kFastBK == 32 && kFastLoadsPerTile == 8, "two k16 slices, eight loads per tile");
    Frags F, G;
    if (ntiles > 0) {
        const int pre = ntiles < kAhead ? ntiles : kAhead;
        for (int i = 0; i < pre; ++i) issue(i);
        // tile 0: nothing to overlap with yet
        if (ntiles > kAhead - 1) wait_vmcnt<(kAhead - 1) * kFastLoadsPerTile>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        read_frags(F, 0, 0);
        if (kAhead < ntiles) issue(kAhead);
        read_frags(G, 0, 16);
        __builtin_amdgcn_sched_barrier(0);
        mfma16(F);
        __builtin_amdgcn_sched_barrier(0);
        // steady state: tiles i+1, i+2 are in flight behind tile i; tile i+kAhead is issued here
        int i = 1;
        for (; i + kAhead < ntiles; ++i) {
            wait_vmcnt<(kAhead - 1) * kFastLoadsPerTile>();
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): own LDS reads of tile i-1 done
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            slice(G, F, i, 0, i + kAhead, 0, true);
            slice(F, G, i, 16, i + kAhead, 4, true);
            advance_tile();
        }
        // drain: nothing left to issue; wait for everything that is still in flight
        for (; i < ntiles; ++i) {
            wait_vmcnt<0>();
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            slice(G, F, i, 0, 0, 0, false);
            slice(F, G, i, 16, 0, 0, false);
        }
        mfma16(G);
    }

    if (kRowStats) {
        // P is used as float rowpart[2 * tiles_n][Mp]: slot 2*tn + wc holds, for every row of
        // this tile row-block, the sum of squares over this wavefront's 128 columns.
        float* part = g.P + static_cast<int64_t>(2 * tn + wc) * g.Mp + m0 + wr * 128;
        const int64_t col0 = n0 + wc * 128 + (lane & 31);
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float sq = 0.f;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const float x = col0 + b * 32 < g.Ncols ? acc[a][b][v] : 0.f;
                    sq += x * x;
                }
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) sq += __shfl_xor(sq, o, kWave);  // 32 lanes = 32 columns
                if ((lane & 31) == 0) part[a * 32 + 8 * (v / 4) + 4 * h + (v % 4)] = sq;
            }
        return;
    }
    float* P = g.P + (static_cast<int64_t>(split) * g.Mp + m0 + wr * 128) * g.Np + n0 + wc * 128;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = a * 32 + 8 * (v / 4) + 4 * h + (v % 4);
                P[static_cast<int64_t>(row) * g.Np + b * 32 + (lane & 31)] = acc[a][b][v];
            }
}

// sumsq[k] = sum over the column slots of rowpart[slot][k], in slot order (deterministic)
__global__ __launch_bounds__(256) void rowpart_reduce_kernel(const float* __restrict__ part, int slots,
                                                             int64_t Mp, int64_t m,
                                                             float* __restrict__ sumsq) {
    const int64_t k = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (k >= m) return;
    float s = 0.f;
    for (int i = 0; i < slots; ++i) s += part[static_cast<int64_t>(i) * Mp + k];
    sumsq[k] = s;
}

// out[j, i] = scale_j * sum_s P[s][j][i]   (fixed summation order: deterministic)
template <typename OT>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ P, int splits,
                                                            int64_t Mp, int64_t Np, int64_t rows,
                                                            int64_t cols,
                                                            const float* __restrict__ scale,
                                                            OT* __restrict__ out, int64_t ldo) {
    const int64_t j = blockIdx.y;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= cols) return;
    float s = 0.f;
    for (int k = 0; k < splits; ++k) s += P[(static_cast<int64_t>(k) * Mp + j) * Np + i];
    if (scale) s *= scale[j];
    store_from_f32(out + j * ldo + i, s);
}

// The same sum for many slices (short, wide problems split K dozens of times): one workgroup
// per output row and 256 columns; each of its four wavefronts adds a contiguous quarter of the
// slices, four columns per lane, and the four partial sums are added in wavefront order.  The
// order is fixed, so the result does not change from run to run.
template <typename OT>
__global__ __launch_bounds__(256) void splitk_reduce_many_kernel(
    const float* __restrict__ P, int splits, int64_t Mp, int64_t Np, int64_t rows, int64_t cols,
    const float* __restrict__ scale, OT* __restrict__ out, int64_t ldo) {
    __shared__ float4 part[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t j = blockIdx.y;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + lane * 4;  // < Np: Np % 128 == 0
    const int per = (splits + 3) / 4;
    const int k0 = w * per, k1 = k0 + per < splits ? k0 + per : splits;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < Np) {
        const float* p = P + (static_cast<int64_t>(k0) * Mp + j) * Np + i;
        const int64_t step = Mp * Np;
#pragma unroll 4
        for (int k = k0; k < k1; ++k, p += step) {
            const float4 v = *reinterpret_cast<const float4*>(p);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    }
    part[w][lane] = s;
    __syncthreads();
    if (w != 0 || i >= cols) return;
    float r[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float4 v = part[q][lane];
        r[0] += v.x; r[1] += v.y; r[2] += v.z; r[3] += v.w;
    }
    const float sc = scale ? scale[j] : 1.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (i + e < cols) store_from_f32(out + j * ldo + i + e, r[e] * sc);
}

// ------------------------------------------------------------------------------ fp32 path
// 64 x 64 output tile, 256 threads, each a 4 x 4 block; BK = 16.
template <typename OT>
__global__ __launch_bounds__(256) void tn_gemm_f32_kernel(
    const float* __restrict__ dY, int layout, int64_t ldy, const float* __restrict__ X, int64_t ldx,
    int64_t T, int64_t rows, int64_t n, const int32_t* __restrict__ idx,
    const float* __restrict__ scale, OT* __restrict__ C, int64_t ldc) {
    __shared__ float As[16][64 + 1];
    __shared__ float Bs[16][64 + 1];
    const int tid = threadIdx.x;
    const int64_t j0 = static_cast<int64_t>(blockIdx.y) * 64, i0 = static_cast<int64_t>(blockIdx.x) * 64;
    const int ty = tid / 16, tx = tid % 16;
    float acc[4][4] = {};
    for (int64_t k0 = 0; k0 < T; k0 += 16) {
        for (int e = tid; e < 16 * 64; e += 256) {
            const int kk = e / 64, c = e % 64;
            const int64_t t = k0 + kk;
            float a = 0.f, b = 0.f;
            if (t < T) {
                if (j0 + c < rows) {
                    const int64_t col = idx ? idx[j0 + c] : j0 + c;
                    a = layout == GRASS_DY_TxM ? dY[t * ldy + col] : dY[col * ldy + t];
                }
                if (i0 + c < n) b = X[t * ldx + i0 + c];
            }
            As[kk][c] = a;
            Bs[kk][c] = b;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = As[kk][ty * 4 + u]; b[u] = Bs[kk][tx * 4 + u]; }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] += a[u] * b[v];
        }
        __syncthreads();
    }
    for (int u = 0; u < 4; ++u) {
        const int64_t j = j0 + ty * 4 + u;
        if (j >= rows) continue;
        const float s = scale ? scale[j] : 1.0f;
        for (int v = 0; v < 4; ++v) {
            const int64_t i = i0 + tx * 4 + v;
            if (i < n) store_from_f32(C + j * ldc + i, s * acc[u][v]);
        }
    }
}

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
    // the GEMM's time at full occupancy, c slices cost about 1 / fill(c) + c * 1400 / T: a
    // slice writes and re-reads 8 bytes per output element at ~4 TB/s while the GEMM spends
    // 2 T flops per output element at ~1.4 PFLOP/s (a slice of at most 16 MB stays in the
    // caches and costs about a third of that).  Each slice keeps at least 8 K tiles.
    const int64_t slots = 256 * Cfg::kWgPerCu;
    const int64_t smax = ktiles / 8 > 0 ? (ktiles / 8 < 128 ? ktiles / 8 : 128) : 1;
    const bool cached = p.Mp * p.Np * 4 <= kCachedSliceBytes;
    const double per_slice = (cached ? 400.0 : 1400.0) / static_cast<double>(T > 0 ? T : 1);
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
    if (const char* e = getenv("GRASS_GEMM_TILE")) return atoi(e) == 256 ? kTile256 : kTile128;
    (void)T;
    if (rows < 1 || n < 1) return kTile128;
    const double padded = static_cast<double>((rows + 255) / 256 * 256) * ((n + 255) / 256 * 256);
    return padded <= 1.35 * static_cast<double>(rows) * static_cast<double>(n) ? kTile256 : kTile128;
}

Plan plan_for(TileId id, int64_t T, int64_t rows, int64_t n, bool pack) {
    return id == kTile256 ? make_plan<Shape256>(T, rows, n, pack) : make_plan<Cfg128>(T, rows, n, pack);
}

template <typename Cfg, bool kDense>
hipError_t launch_gemm_kernel(const GemmArgs& g, unsigned grid, hipStream_t s) {
    auto kernel = tn_gemm_bf16_kernel<Cfg, kDense>;
    if (Cfg::kLdsBytes > 64 * 1024) {
        static bool raised = false;  // per instantiation; the attribute is sticky per process
        if (!raised) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     static_cast<int>(Cfg::kLdsBytes));
            if (e != hipSuccess) return e;
            raised = true;
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
    const char* force = getenv("GRASS_FUSED_STATS");  // "1": whenever the shape allows (tests)
    return (tiles >= 192 || (force && force[0] == '1')) && dt == GRASS_BF16 && layout == GRASS_DY_TxM && T >= kFastBK &&
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

// C_i = scale_i * (A_i^T X) for `count` row sets that share X.  The sets are packed side by
// side into one panel (each starts at a multiple of 8 columns), one GEMM covers the panel,
// and the partial tiles are reduced into each set's own output.
grass_status launch_tn_gemm_segments(const GemmSegment* seg, int count, grass_dy_layout layout,
                                     const void* X, int64_t ldx, grass_dtype dt, int64_t T,
                                     int64_t n, grass_dtype odt, void* ws, hipStream_t s,
                                     hipEvent_t ev_start, hipEvent_t ev_stop) {
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
                const grass_status st = launch_tn_gemm_segments(
                    seg + i, 1, layout, X, ldx, dt, T, n, odt, ws, s, i == 0 ? ev_start : nullptr,
                    i + 1 == count ? ev_stop : nullptr);
                if (st != GRASS_OK) return st;
            }
            return GRASS_OK;
        }
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
        aligned_to(dY0, 16) && ldy0 % 8 == 0 && getenv("GRASS_GEMM_PACK_MXT") == nullptr) {
        const int64_t src_rows = seg[0].idx ? seg[0].src_rows : total;
        a_rows_form = src_rows > 0 && src_rows * ldy0 * 2 + 64 < (int64_t{1} << 32);
    }
    if (a_rows_form) pack = false;
    // the large-tile kernel takes whole K tiles; a ragged tail goes to the small-tile kernel
    const int64_t T_main = tile == kTile256 ? T / kFastBK * kFastBK : T;
    const Plan p = plan_for(tile, T, total, n, pack);  // sized for all T rows; K tiling per tile kind
    char* base = static_cast<char*>(ws);
    base += (256 - reinterpret_cast<uintptr_t>(base) % 256) % 256;
    uint16_t* panel = reinterpret_cast<uint16_t*>(base);
    float* partial = reinterpret_cast<float*>(base + p.pack_bytes);

    GemmArgs g;
    if (pack) {
        int64_t off = 0;
        for (int i = 0; i < count && T > 0; ++i) {
            // the last set also zero-fills the panel's padding columns
            const int64_t width = i + 1 == count ? p.rp - off : (seg[i].rows + 7) / 8 * 8;
            if (width > 0) {
                if (layout == GRASS_DY_TxM) {
                    int tpr_log2 = 8;  // threads per row of t: the power of two covering width / 4
                    while (tpr_log2 > 0 && (int64_t{4} << (tpr_log2 - 1)) >= width) --tpr_log2;
                    const int64_t gx = (width + (int64_t{4} << tpr_log2) - 1) / (int64_t{4} << tpr_log2);
                    const int64_t passes = (T + (256 >> tpr_log2) - 1) / (256 >> tpr_log2);
                    int64_t rpt = passes * gx / 2048;  // aim at >= 2048 workgroups
                    rpt = rpt < 4 ? 4 : (rpt > kPackRows ? kPackRows : rpt);
                    const int64_t rows_per_wg = rpt * (256 >> tpr_log2);
                    const dim3 grid(static_cast<unsigned>(gx),
                                    static_cast<unsigned>((T + rows_per_wg - 1) / rows_per_wg));
                    pack_txm_kernel<<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(seg[i].dY),
                                                         seg[i].ldy, T, seg[i].idx, seg[i].rows,
                                                         width, p.rp, tpr_log2,
                                                         static_cast<int>(rpt), panel + off);
                } else if (aligned_to(seg[i].dY, 16) && seg[i].ldy % 8 == 0 && p.rp % 8 == 0 &&
                           width % 8 == 0) {
                    const dim3 grid(static_cast<unsigned>((width + kPackWideJ - 1) / kPackWideJ),
                                    static_cast<unsigned>((T + kPackWideT - 1) / kPackWideT));
                    pack_mxt_wide_kernel<<<grid, 256, 0, s>>>(
                        static_cast<const uint16_t*>(seg[i].dY), seg[i].ldy, T, seg[i].idx,
                        seg[i].rows, width, p.rp, panel + off);
                } else {
                    const dim3 grid(static_cast<unsigned>((width + 63) / 64),
                                    static_cast<unsigned>((T + 63) / 64));
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
        const int chunks = static_cast<int>((nb / 2 + 1023) / 1024);
        if (T * chunks > 0x7FFFFFFF) return GRASS_ERR_SHAPE;
        align_rows_kernel<<<static_cast<unsigned>(T * chunks), 256, 0, s>>>(
            static_cast<const uint16_t*>(X), ldx, n, nb, chunks, xa);
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

    const int64_t items = static_cast<int64_t>(p.tiles_m) * p.tiles_n * p.splits;
    const int64_t chunk = (items + kNumXcd - 1) / kNumXcd;
    if (chunk * kNumXcd > 0x7FFFFFFF) return GRASS_ERR_SHAPE;
    if (ev_start) (void)hipEventRecord(ev_start, s);
    const unsigned grid = static_cast<unsigned>(chunk * kNumXcd);
    hipError_t le;
    if (tile == kTile256) {
        if (a_rows_form)
            tn_gemm_bf16_direct_kernel<false, false, true><<<grid, 256, 0, s>>>(g);
        else if (gathered)
            tn_gemm_bf16_direct_kernel<false><<<grid, 256, 0, s>>>(g);
        else
            tn_gemm_bf16_direct_kernel<true><<<grid, 256, 0, s>>>(g);
        le = hipSuccess;
    } else
        le = gathered ? launch_gemm_kernel<Cfg128, false>(g, grid, s)
                      : launch_gemm_kernel<Cfg128, true>(g, grid, s);
    if (le != hipSuccess) return GRASS_ERR_DEVICE;
    if (ev_stop) (void)hipEventRecord(ev_stop, s);
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

    int64_t off = 0;
    for (int i = 0; i < count; ++i) {
        const GemmSegment& q = seg[i];
        if (q.rows > 0) {
            const dim3 rgrid(static_cast<unsigned>((n + 255) / 256), static_cast<unsigned>(q.rows));
            const float* part = partial + off * p.Np;
            if (slices > kManySlices && p.Np % 128 == 0) {
                if (odt == GRASS_F32)
                    splitk_reduce_many_kernel<float><<<rgrid, 256, 0, s>>>(
                        part, slices, p.Mp, p.Np, q.rows, n, q.rho, static_cast<float*>(q.C), q.ldc);
                else
                    splitk_reduce_many_kernel<uint16_t><<<rgrid, 256, 0, s>>>(
                        part, slices, p.Mp, p.Np, q.rows, n, q.rho, static_cast<uint16_t*>(q.C), q.ldc);
            } else if (odt == GRASS_F32)
                splitk_reduce_kernel<float><<<rgrid, 256, 0, s>>>(
                    part, slices, p.Mp, p.Np, q.rows, n, q.rho, static_cast<float*>(q.C), q.ldc);
            else
                splitk_reduce_kernel<uint16_t><<<rgrid, 256, 0, s>>>(
                    part, slices, p.Mp, p.Np, q.rows, n, q.rho, static_cast<uint16_t*>(q.C), q.ldc);
        }
        off += (q.rows + 7) / 8 * 8;
    }
    return launch_status();
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
