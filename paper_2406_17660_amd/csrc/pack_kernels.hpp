// Gather / transpose / align passes that prepare the GEMM operands (all HBM-bound).
// Included by cgrad.hip only (device code shares one translation unit with its launchers).
#pragma once
#include "common.hpp"
#include "gemm_common.hpp"

namespace grass {
namespace {

// ------------------------------------------------------------------------------ pack
// out[t, j] = dY[t, idx[j]] (j < r; idx == nullptr: column j itself), 0 for r <= j < rp; rows
// of `out` are ldo apart (several matrices may fill adjacent column ranges of one panel).
// Thread = 4 adjacent j; 2^tpr_log2 threads cover the columns of one row of t (a narrow panel,
// r = 128 say, puts several rows of t side by side in a workgroup instead of idling most of
// it), and every thread handles kPackRows values of t, one after the other.  Four measured
// best at the 7B layer: 8 or 16 rows per thread leave fewer workgroups to hide the latency
// of the gather (5 - 8 % slower), 1 or 2 do not amortise the loads of idx, and issuing the
// loads of all rows before the first store is 12 % slower.  Wave stores are contiguous.
constexpr int kPackRows = 4;
__global__ __launch_bounds__(256) void pack_txm_kernel(const uint16_t* __restrict__ dY, int64_t ldy,
                                                       int64_t T, const int32_t* __restrict__ idx,
                                                       int64_t r, int64_t rp, int64_t ldo,
                                                       int tpr_log2, uint16_t* __restrict__ out) {
    const int tpr = 1 << tpr_log2, rows_per_pass = 256 >> tpr_log2;
    // blockIdx.x runs over t (it can be large), blockIdx.y over the blocks of j
    const int64_t j0 = (static_cast<int64_t>(blockIdx.y) * tpr + (threadIdx.x & (tpr - 1))) * 4;
    if (j0 >= rp) return;
    int64_t col[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) col[e] = j0 + e < r ? (idx ? idx[j0 + e] : j0 + e) : -1;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kPackRows * rows_per_pass +
                       (threadIdx.x >> tpr_log2);
#pragma unroll
    for (int tt = 0; tt < kPackRows; ++tt) {
        const int64_t t = t0 + static_cast<int64_t>(tt) * rows_per_pass;
        if (t >= T) break;
        const uint16_t* row = dY + t * ldy;
        uint16_t v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = col[e] >= 0 ? row[col[e]] : static_cast<uint16_t>(0);
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        const u32x2 w = {v[0] | (static_cast<uint32_t>(v[1]) << 16),
                         v[2] | (static_cast<uint32_t>(v[3]) << 16)};
        __builtin_nontemporal_store(w, reinterpret_cast<u32x2*>(out + t * ldo + j0));  // written once, read later
    }
}

// The gather above for several matrices in one launch (layers that share X: their selected
// rows go side by side into one panel): blockIdx.z picks the set.  Short gathers (tens of
// microseconds each) otherwise pay a launch and a ramp-up apiece.
struct PackSet {
    const uint16_t* dY;
    int64_t ldy;
    const int32_t* idx;
    int64_t r, rp;       // selected rows, panel columns of this set (padding included)
    int64_t off;         // first panel column of this set
    int tpr_log2;        // threads per row of t
};
struct PackSets {
    PackSet set[GRASS_MAX_GROUP];
};
__global__ __launch_bounds__(256) void pack_txm_group_kernel(PackSets sets, int64_t T, int64_t ldo,
                                                             uint16_t* __restrict__ panel) {
    const PackSet& q = sets.set[blockIdx.z];
    const int tpr_log2 = q.tpr_log2;
    const int tpr = 1 << tpr_log2, rows_per_pass = 256 >> tpr_log2;
    const int64_t j0 = (static_cast<int64_t>(blockIdx.y) * tpr + (threadIdx.x & (tpr - 1))) * 4;
    if (j0 >= q.rp) return;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kPackRows * rows_per_pass +
                       (threadIdx.x >> tpr_log2);
    if (t0 >= T) return;  // the grid covers the set with the fewest rows of t per workgroup
    int64_t col[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) col[e] = j0 + e < q.r ? (q.idx ? q.idx[j0 + e] : j0 + e) : -1;
    uint16_t* out = panel + q.off;
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int tt = 0; tt < kPackRows; ++tt) {
        const int64_t t = t0 + static_cast<int64_t>(tt) * rows_per_pass;
        if (t >= T) break;
        const uint16_t* row = q.dY + t * q.ldy;
        uint16_t v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = col[e] >= 0 ? row[col[e]] : static_cast<uint16_t>(0);
        const u32x2 w = {v[0] | (static_cast<uint32_t>(v[1]) << 16),
                         v[2] | (static_cast<uint32_t>(v[3]) << 16)};
        __builtin_nontemporal_store(w, reinterpret_cast<u32x2*>(out + t * ldo + j0));
    }
}

// The same gather for wide matrices, with the rows of dY staged through LDS: a workgroup copies
// kRows whole rows of t into LDS with streaming 16-byte loads (every byte of dY is fetched
// exactly once, by a full-width request, and is not kept in the caches), then gathers from LDS
// and stores the panel rows with streaming 8-byte stores.  Measured at the 7B layer against
// the kernel above: 0.21 instead of 0.24 ms (1.34 GB at 6.3 TB/s); one row per workgroup is
// slower than the kernel above at m = 4096, two to eight rows differ little.
// Rows need no alignment: a row that starts e bytes after a 16-byte boundary is copied as the
// aligned vectors that cover it and lands in LDS with the same e, which the gather adds to its
// indices.  Vectors that would reach outside [lo, hi), the bytes of the matrix (the first of the
// first row, the last of the last), are put together element by element.
// LDS: kRows * pack_stage_row_elems(m) * 2 bytes.  Two rows per workgroup while three workgroups
// still fit a compute unit's LDS (m <= 12288), one row beyond (at m = 13824 two rows, 55 KB,
// leave two workgroups per compute unit and lose to the kernel above).
constexpr int64_t kPackStageTwoRowsMaxM = 12288, kPackStageMaxBytes = 65536;
constexpr int64_t kPackStageDeepMinM = 4096;  // from here on four vectors per row in flight
__host__ __device__ constexpr int64_t pack_stage_row_elems(int64_t m) {
    return ((2 * m + 14 + 15) / 16) * 8;  // the most 16-byte vectors a row of m elements can touch
}
template <int kRows, int kDepth>
__global__ __launch_bounds__(256) void pack_txm_staged_kernel(const uint16_t* __restrict__ dY,
                                                              int64_t ldy, int64_t T, int64_t m,
                                                              const int32_t* __restrict__ idx,
                                                              int64_t r, int64_t rp, int64_t ldo,
                                                              uint16_t* __restrict__ out) {
    extern __shared__ __attribute__((aligned(16))) uint16_t stage[];  // kRows x pack_stage_row_elems(m)
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kRows;
    const int64_t stride = pack_stage_row_elems(m);
    const uintptr_t lo = reinterpret_cast<uintptr_t>(dY);
    const uintptr_t hi = lo + static_cast<uintptr_t>(((T - 1) * ldy + m) * 2);
    uintptr_t window[kRows];  // 16-byte aligned start of the vectors covering each row
    int shift[kRows];         // elements between it and the row's first element
    int nvec = 0;
#pragma unroll
    for (int row = 0; row < kRows; ++row) {
        const int64_t t = t0 + row < T ? t0 + row : T - 1;  // a row past the end is not used
        const uintptr_t start = reinterpret_cast<uintptr_t>(dY + t * ldy), e = start & 15;
        window[row] = start - e;
        shift[row] = static_cast<int>(e >> 1);
        const int v = static_cast<int>((e + 2 * static_cast<uintptr_t>(m) + 15) >> 4);
        nvec = v > nvec ? v : nvec;
    }
    // kDepth vectors of every row in flight per thread before the first LDS store (rows of 4096
    // elements and more: 5 % faster at 11008 and 13824 with four than with one; shorter rows are
    // 2 % slower with four)
    for (int c0 = threadIdx.x; c0 < nvec; c0 += 256 * kDepth) {
        s16x8 x[kDepth][kRows];
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int c = c0 + 256 * u;
            if (c >= nvec) break;
#pragma unroll
            for (int row = 0; row < kRows; ++row) {
                const uintptr_t addr = window[row] + 16 * static_cast<uintptr_t>(c);
                if (addr >= lo && addr + 16 <= hi) {
                    x[u][row] = __builtin_nontemporal_load(reinterpret_cast<const s16x8*>(addr));
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const uintptr_t a = addr + 2 * i;
                        x[u][row][i] = a >= lo && a + 2 <= hi ? *reinterpret_cast<const short*>(a) : short{0};
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int c = c0 + 256 * u;
            if (c >= nvec) break;
#pragma unroll
            for (int row = 0; row < kRows; ++row)
                *reinterpret_cast<s16x8*>(stage + row * stride + c * 8) = x[u][row];
        }
    }
    __syncthreads();
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    for (int64_t j0 = static_cast<int64_t>(threadIdx.x) * 4; j0 < rp; j0 += 1024) {
        int32_t col[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            col[e] = j0 + e < r ? (idx ? idx[j0 + e] : static_cast<int32_t>(j0 + e)) : -1;
#pragma unroll
        for (int row = 0; row < kRows; ++row) {
            if (t0 + row >= T) break;
            const uint16_t* src = stage + row * stride + shift[row];
            uint16_t v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = col[e] >= 0 ? src[col[e]] : static_cast<uint16_t>(0);
            const u32x2 w = {v[0] | (static_cast<uint32_t>(v[1]) << 16),
                             v[2] | (static_cast<uint32_t>(v[3]) << 16)};
            __builtin_nontemporal_store(w, reinterpret_cast<u32x2*>(out + (t0 + row) * ldo + j0));
        }
    }
}

// out[t, j] = dYt[idx[j] (or j), t]: gather of rows of the m x T matrix, transposed through
// a 64 x 64 LDS tile so that both the reads (along t) and the writes (along j) coalesce.
__global__ __launch_bounds__(256) void pack_mxt_kernel(const uint16_t* __restrict__ dYt, int64_t ldy,
                                                       int64_t T, const int32_t* __restrict__ idx,
                                                       int64_t r, int64_t rp, int64_t ldo,
                                                       uint16_t* __restrict__ out) {
    __shared__ uint16_t tile[64][66];
    // blockIdx.x runs over t (it can be large), blockIdx.y over the blocks of j
    const int64_t j0 = static_cast<int64_t>(blockIdx.y) * 64;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * 64;
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
    const int64_t j0 = static_cast<int64_t>(blockIdx.y) * kPackWideJ;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kPackWideT;
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

// out[t, c] = in[t, c] for c < n and 0 for n <= c < np (np a multiple of 8, rows of `out` np
// apart and 16-byte aligned): a copy of a matrix whose rows start at odd element offsets (n not a
// multiple of 8, as in the 5461-wide MLP of the 1B model) into rows the 16-byte loads of the GEMM
// can take.  `in` itself is 4-byte aligned, so a row starts e = 0, 2, ..., 14 bytes after a
// 16-byte boundary.  A thread produces 8 output elements (one streaming 16-byte store) from the
// two aligned 16-byte vectors that contain them: with e = 4 k + b, output word i is input word
// k + i of that 32-byte window, or the upper half of it joined to the lower half of the next
// (b = 2).  k and b are the same for a whole row, i.e. for the whole workgroup.  Vectors that
// would reach outside [lo, hi) (the bytes of the matrix: the start of the first row, the end of
// the last) or past column n are put together element by element.
__global__ __launch_bounds__(256) void align_rows_kernel(const uint16_t* __restrict__ in, int64_t ld,
                                                         int64_t T, int64_t n, int64_t np, int chunks,
                                                         uint16_t* __restrict__ out) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int64_t t = blockIdx.x / chunks;
    const int64_t q = static_cast<int64_t>(blockIdx.x % chunks) * 256 + threadIdx.x;  // 8 elements each
    if (8 * q >= np) return;
    const uint16_t* row = in + t * ld;
    const uintptr_t lo = reinterpret_cast<uintptr_t>(in);
    const uintptr_t hi = lo + static_cast<uintptr_t>(((T - 1) * ld + n) * 2);
    const uintptr_t start = reinterpret_cast<uintptr_t>(row), e = start & 15;
    const uintptr_t window = (start - e) + 16 * static_cast<uintptr_t>(q);
    u32x4 v;
    if (8 * q + 8 <= n && window >= lo && window + 32 <= hi) {
        const u32x4* src = reinterpret_cast<const u32x4*>(window);
        const u32x4 a = src[0], b = src[1];
        const uint32_t w[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
        const bool half = (e & 2) != 0;
        auto take = [&](int k) {  // k is a constant at every call site
#pragma unroll
            for (int i = 0; i < 4; ++i)
                v[i] = half ? (w[k + i] >> 16) | (w[k + i + 1] << 16) : w[k + i];
        };
        switch (e >> 2) {  // uniform over the workgroup
            case 0: take(0); break;
            case 1: take(1); break;
            case 2: take(2); break;
            default: take(3); break;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t c = 8 * q + 2 * i;
            const uint32_t l = c < n ? row[c] : 0u, h = c + 1 < n ? row[c + 1] : 0u;
            v[i] = l | (h << 16);
        }
    }
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out + t * np) + q);
}


}  // namespace
}  // namespace grass
