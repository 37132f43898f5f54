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

constexpr int kNumXcd = 8;

// ------------------------------------------------------------------------------ pack
// out[t, j] = dY[t, idx[j]] (j < r), 0 for r <= j < rp.  Thread = 4 adjacent j, loops over
// kPackRows values of t; wave stores are contiguous 512 B.
constexpr int kPackRows = 16;
__global__ __launch_bounds__(256) void pack_txm_kernel(const uint16_t* __restrict__ dY, int64_t ldy,
                                                       int64_t T, const int32_t* __restrict__ idx,
                                                       int64_t r, int64_t rp,
                                                       uint16_t* __restrict__ out) {
    const int64_t j0 = (static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x) * 4;
    if (j0 >= rp) return;
    int64_t col[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) col[e] = j0 + e < r ? idx[j0 + e] : -1;
    const int64_t t0 = static_cast<int64_t>(blockIdx.y) * kPackRows;
#pragma unroll 4
    for (int tt = 0; tt < kPackRows; ++tt) {
        const int64_t t = t0 + tt;
        if (t >= T) break;
        const uint16_t* row = dY + t * ldy;
        uint16_t v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = col[e] >= 0 ? row[col[e]] : static_cast<uint16_t>(0);
        uint2 w;
        w.x = v[0] | (static_cast<uint32_t>(v[1]) << 16);
        w.y = v[2] | (static_cast<uint32_t>(v[3]) << 16);
        *reinterpret_cast<uint2*>(out + t * rp + j0) = w;
    }
}

// out[t, j] = dYt[idx[j] (or j), t]: gather of rows of the m x T matrix, transposed through
// a 64 x 64 LDS tile so that both the reads (along t) and the writes (along j) coalesce.
__global__ __launch_bounds__(256) void pack_mxt_kernel(const uint16_t* __restrict__ dYt, int64_t ldy,
                                                       int64_t T, const int32_t* __restrict__ idx,
                                                       int64_t r, int64_t rp,
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
        if (t < T && j < rp) out[t * rp + j] = tile[lane][tt];
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
};

template <typename Cfg>
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
    const int tm = tile % g.tiles_m, tn = tile / g.tiles_m;
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

struct Plan {
    int64_t Mp, Np, rp;  // padded rows / cols of the partial buffer; packed panel width
    int tiles_m, tiles_n, splits, ktiles_per_split;
    size_t pack_bytes, partial_bytes;
};

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

template <typename Cfg>
Plan make_plan(int64_t T, int64_t rows, int64_t n, bool needs_pack) {
    Plan p;
    p.tiles_m = static_cast<int>((rows + Cfg::BM - 1) / Cfg::BM);
    p.tiles_n = static_cast<int>((n + Cfg::BN - 1) / Cfg::BN);
    p.Mp = static_cast<int64_t>(p.tiles_m) * Cfg::BM;
    p.Np = static_cast<int64_t>(p.tiles_n) * Cfg::BN;
    p.rp = p.Mp;
    const int64_t ktiles = (T + Cfg::BK - 1) / Cfg::BK;
    const int64_t tiles = static_cast<int64_t>(p.tiles_m) * p.tiles_n;
    // enough workgroups for two per CU, but keep at least 8 K tiles per split
    int64_t s = tiles > 0 ? (2 * 256 + tiles - 1) / tiles : 1;
    const int64_t smax = ktiles / 8 > 0 ? ktiles / 8 : 1;
    if (s > smax) s = smax;
    if (s < 1) s = 1;
    p.ktiles_per_split = static_cast<int>((ktiles + s - 1) / s);
    if (p.ktiles_per_split < 1) p.ktiles_per_split = 1;
    p.splits = static_cast<int>((ktiles + p.ktiles_per_split - 1) / p.ktiles_per_split);
    if (p.splits < 1) p.splits = 1;
    p.pack_bytes = needs_pack ? round_up(static_cast<size_t>(T) * p.rp * 2, 256) : 0;
    p.partial_bytes = static_cast<size_t>(p.splits) * p.Mp * p.Np * 4;
    return p;
}

bool needs_pack(grass_dy_layout layout, bool gathered) {
    return gathered || layout == GRASS_DY_MxT;
}

}  // namespace

size_t gemm_workspace_bytes(int64_t T, int64_t mrows, int64_t n, grass_dtype dt,
                            grass_dy_layout layout, bool gathered) {
    if (dt == GRASS_F32) return 0;
    const Plan p = make_plan<Cfg128>(T, mrows, n, needs_pack(layout, gathered));
    return p.pack_bytes + p.partial_bytes + 256;
}

grass_status launch_tn_gemm(const void* dY, grass_dy_layout layout, int64_t ldy, const void* X,
                            int64_t ldx, grass_dtype dt, int64_t T, int64_t mrows, int64_t n,
                            const int32_t* idx, const float* rho, void* C, grass_dtype odt,
                            int64_t ldc, void* ws, hipStream_t s, hipEvent_t ev_start,
                            hipEvent_t ev_stop) {
    if (mrows == 0 || n == 0) return GRASS_OK;
    if (mrows > 65535) return GRASS_ERR_SHAPE;
    if (dt == GRASS_F32) {
        const dim3 grid(static_cast<unsigned>((n + 63) / 64), static_cast<unsigned>((mrows + 63) / 64));
        if (ev_start) (void)hipEventRecord(ev_start, s);
        if (odt == GRASS_F32)
            tn_gemm_f32_kernel<float><<<grid, 256, 0, s>>>(
                static_cast<const float*>(dY), layout, ldy, static_cast<const float*>(X), ldx, T,
                mrows, n, idx, rho, static_cast<float*>(C), ldc);
        else
            tn_gemm_f32_kernel<uint16_t><<<grid, 256, 0, s>>>(
                static_cast<const float*>(dY), layout, ldy, static_cast<const float*>(X), ldx, T,
                mrows, n, idx, rho, static_cast<uint16_t*>(C), ldc);
        if (ev_stop) (void)hipEventRecord(ev_stop, s);
        return launch_status();
    }

    using Cfg = Cfg128;
    const bool gathered = idx != nullptr;
    const bool pack = needs_pack(layout, gathered);
    const Plan p = make_plan<Cfg>(T, mrows, n, pack);
    char* base = static_cast<char*>(ws);
    base += (256 - reinterpret_cast<uintptr_t>(base) % 256) % 256;
    uint16_t* panel = reinterpret_cast<uint16_t*>(base);
    float* partial = reinterpret_cast<float*>(base + p.pack_bytes);

    GemmArgs g;
    if (pack) {
        if (T > 0) {
            if (layout == GRASS_DY_TxM) {
                const dim3 grid(static_cast<unsigned>((p.rp + 1023) / 1024),
                                static_cast<unsigned>((T + kPackRows - 1) / kPackRows));
                pack_txm_kernel<<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(dY), ldy, T, idx,
                                                     mrows, p.rp, panel);
            } else {
                const dim3 grid(static_cast<unsigned>(p.rp / 64), static_cast<unsigned>((T + 63) / 64));
                pack_mxt_kernel<<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(dY), ldy, T, idx,
                                                     mrows, p.rp, panel);
            }
        }
        g.A = panel;
        g.lda = p.rp;
        g.Mcols = p.rp;
        g.a_fast = 1;
    } else {
        g.A = static_cast<const uint16_t*>(dY);
        g.lda = ldy;
        g.Mcols = mrows;
        g.a_fast = aligned_to(dY, 16) && ldy % 8 == 0;
    }
    g.B = static_cast<const uint16_t*>(X);
    g.ldb = ldx;
    g.Ncols = n;
    g.b_fast = aligned_to(X, 16) && ldx % 8 == 0;
    g.P = partial;
    g.K = T;
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
    tn_gemm_bf16_kernel<Cfg><<<static_cast<unsigned>(chunk * kNumXcd), Cfg::kThreads,
                               Cfg::kLdsBytes, s>>>(g);
    if (ev_stop) (void)hipEventRecord(ev_stop, s);

    const dim3 rgrid(static_cast<unsigned>((n + 255) / 256), static_cast<unsigned>(mrows));
    if (odt == GRASS_F32)
        splitk_reduce_kernel<float><<<rgrid, 256, 0, s>>>(partial, p.splits, p.Mp, p.Np, mrows, n,
                                                          rho, static_cast<float*>(C), ldc);
    else
        splitk_reduce_kernel<uint16_t><<<rgrid, 256, 0, s>>>(partial, p.splits, p.Mp, p.Np, mrows,
                                                             n, rho, static_cast<uint16_t*>(C), ldc);
    return launch_status();
}

}  // namespace grass
