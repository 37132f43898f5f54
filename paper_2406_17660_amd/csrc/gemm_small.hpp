// bf16 MFMA GEMM with 128 x 128 tiles, register-staged: small and unaligned problems, K tails.
// Included by cgrad.hip only (device code shares one translation unit with its launchers).
#pragma once
#include "common.hpp"
#include "gemm_common.hpp"

namespace grass {
namespace {

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


}  // namespace
}  // namespace grass
