// bf16 MFMA GEMM with the column gather of a T x m left operand done inside the kernel, for
// narrow layers: G_C = (B dY^T) X of Section 3.1 ("Efficient Gradient Projection") without the
// packed panel in between.  Included by cgrad.hip only.
#pragma once
#include "gemm_large.hpp"

namespace grass {
namespace {

// Why only narrow layers.  A tile of selected columns of a T x m matrix touches, per row of t,
// almost every cache line of that row (r/m = 1/4 of the columns, 2 bytes each), so whoever
// gathers has to pull whole rows of dY.  This kernel stages whole rows in LDS: 16 rows of up
// to 512 values are 16 KB, three such stages plus the X stages still leave room for two
// workgroups per compute unit.  At m = 1376 a stage is 44 KB, one workgroup per unit keeps too
// few bytes in flight, and the separate gather pass (many small workgroups) followed by the
// large-tile GEMM is faster (measured at T = 65536, r = 128, gather pass + GEMM against this
// kernel: 97 against 104 us for a pair of 1376-wide sets; 37 against 26 us for a 512 x 512 layer,
// 97 against 66 us for three of them sharing X).
//
// Work: an output tile is 128 selected rows of one set x 256 columns; four wavefronts, each
// 128 x 64 (eight 32 x 32 accumulator fragments).  K advances in tiles of 16 tokens through a
// ring of three LDS stages.  A stage holds the 16 whole rows of the set's dY (a flat copy,
// 4 x 256 chunks of 16 bytes; with m < 512 the tail of the area is padding that the spare
// lanes fill with any valid chunk) and the 16 x 256 block of X (rows of 512 bytes, 16-byte
// slots permuted as in the large-tile kernel, so the same transposing reads apply).  Per K
// tile the workgroup first gathers: thread (j, c) reads the eight values dY[8c .. 8c+8)[idx[j]]
// out of the staged rows and writes them as one 16-byte slot of a compact block [128][16] with
// k contiguous (slot c of row j stored at c ^ ((j / 8) % 2): the 16 lanes of a quarter
// wavefront then cover all banks once).  An MFMA left operand is one 16-byte read of that
// block; no transposition is needed.  Loads run two tiles ahead (load-to-LDS, waits placed by
// hand as in the large-tile kernel).  The result goes to partial tiles [slice][Mp][Np], the
// layout the split-K reductions and the fused tail read.
constexpr int kNarrowBM = 128, kNarrowBN = 256, kNarrowBK = 16, kNarrowStages = 3;
constexpr int kNarrowMaxM = 512;                        // widest dY whose 16 rows fit a stage
constexpr int kNarrowDyLoads = 4;                       // load instructions per wavefront for the dY rows
constexpr int kNarrowDyBytes = kNarrowDyLoads * 256 * 16;
constexpr int kNarrowXBytes = kNarrowBK * 512;
constexpr int kNarrowStageBytes = kNarrowDyBytes + kNarrowXBytes;
constexpr int kNarrowLoads = kNarrowDyLoads + kNarrowBK / 8;  // per wavefront and K tile
constexpr int kNarrowLdsBytes = kNarrowStages * kNarrowStageBytes + kNarrowBM * kNarrowBK * 2;

struct NarrowSet {
    const uint16_t* dY;  // T x m, leading dimension ldy
    int64_t ldy;
    const int32_t* idx;  // `rows` column numbers of dY
    int rows;            // selected rows of this set (<= 128 per row tile; several tiles allowed)
    int chunks;          // 16-byte chunks per row of dY (m / 8)
    int off;             // first row of this set in the partial tiles
    int tile0;           // number of row tiles of the sets before this one
};
struct NarrowArgs {
    NarrowSet set[GRASS_MAX_GROUP];
    int count;
    const uint16_t* X;
    int64_t ldx, n;
    float* P;            // partial tiles [splits][Mp][Np]
    int64_t Mp, Np, ktiles;
    int tiles_m, tiles_n, splits, ktiles_per_split;
};

__global__ __launch_bounds__(256) void tn_gemm_gather_narrow_kernel(NarrowArgs g) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t narrow_lds[];
    constexpr int KT = kNarrowBK;
    uint16_t* compact = narrow_lds + kNarrowStages * kNarrowStageBytes / 2;

    // consecutive items share a K slice; XCD x receives a contiguous run of items (as in the
    // other GEMM kernels), so the tiles that read the same rows of dY and X share an L2
    const int64_t items = static_cast<int64_t>(g.tiles_m) * g.tiles_n * g.splits;
    const int64_t chunk_items = (items + kNumXcd - 1) / kNumXcd;
    const int64_t item = static_cast<int64_t>(blockIdx.x % kNumXcd) * chunk_items + blockIdx.x / kNumXcd;
    if (item >= items) return;
    const int tiles = g.tiles_m * g.tiles_n;
    const int split = static_cast<int>(item / tiles);
    const int tile = static_cast<int>(item % tiles);
    const int tm = tile % g.tiles_m, tn = tile / g.tiles_m;
    int si = 0;
#pragma unroll
    for (int i = 1; i < GRASS_MAX_GROUP; ++i)
        if (i < g.count && tm >= g.set[i].tile0) si = i;
    const NarrowSet& sg = g.set[si];
    const int row0 = (tm - sg.tile0) * kNarrowBM;  // first selected row of this tile within its set
    const int64_t n0 = static_cast<int64_t>(tn) * kNarrowBN;
    const int64_t kt_begin = static_cast<int64_t>(split) * g.ktiles_per_split;
    int64_t kt_end = kt_begin + g.ktiles_per_split;
    if (kt_end > g.ktiles) kt_end = g.ktiles;
    const int ntiles = kt_end > kt_begin ? static_cast<int>(kt_end - kt_begin) : 0;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- global -> LDS: per-lane byte offsets inside one K tile.  Chunk number c of the flat
    // copy of the 16 rows is chunk c % chunks of row c / chunks; load q of wavefront w covers
    // chunks 64 (4 q + w) .. + 64.
    const int used = KT * sg.chunks;
    uint32_t laneDY[kNarrowDyLoads], laneX[KT / 8];
#pragma unroll
    for (int q = 0; q < kNarrowDyLoads; ++q) {
        int c = (q * 4 + wave) * 64 + lane;
        if (c >= used) c = 0;  // padding of the stage: any valid chunk
        const int row = c / sg.chunks, cc = c - row * sg.chunks;
        laneDY[q] = static_cast<uint32_t>((row * sg.ldy + cc * 8) * 2);
    }
    const int lrow = wave * 2 + (lane >> 5);
    int64_t colX = n0 + ((lane & 31) ^ (4 * (lrow & 3))) * 8;
    if (colX >= g.n) colX = 0;  // columns past the edge only feed outputs nobody reads
#pragma unroll
    for (int p = 0; p < KT / 8; ++p)
        laneX[p] = static_cast<uint32_t>(((p * 8 + lrow) * g.ldx + colX) * 2);
    const uint16_t* gY = sg.dY + kt_begin * KT * sg.ldy;
    const uint16_t* gX = g.X + kt_begin * KT * g.ldx;
    const int64_t stepY = static_cast<int64_t>(KT) * sg.ldy, stepX = static_cast<int64_t>(KT) * g.ldx;
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void_t*)narrow_lds));
    auto issue = [&](int i) {
        const uint32_t st = lds_base + (i % kNarrowStages) * kNarrowStageBytes;
#pragma unroll
        for (int q = 0; q < kNarrowDyLoads; ++q) load16_to_lds(gY, laneDY[q], st + (q * 4 + wave) * 1024);
#pragma unroll
        for (int p = 0; p < KT / 8; ++p)
            load16_to_lds(gX, laneX[p], st + kNarrowDyBytes + (p * 8 + wave * 2) * 512);
        gY += stepY;
        gX += stepX;
    };

    // ---- gather: this thread builds slot tid / 128 of compact row j = tid % 128
    const int j = tid & 127, cslot = tid >> 7;
    const int jsel = row0 + j;
    const int mycol = jsel < sg.rows ? sg.idx[jsel] : -1;  // rows past the set's end stay zero
    asm volatile("" ::"v"(mycol));  // in its register before the first tile load is issued
    const int row_pitch = sg.chunks * 8;  // elements per staged row
    const int cwrite = j * KT + (cslot ^ ((j >> 3) & 1)) * 8;
    // ---- MFMA operands: A from the compact block, B by the large-tile kernel's transposing reads
    const int L = lane & 15, g2 = (lane >> 4) & 1, h = lane >> 5;
    const int rrow = 8 * h + (L >> 2);
    const int swz = 4 * (L >> 2);
    const int lchunk = 2 * g2 + ((L & 3) >> 1);
    const int half = (L & 1) * 4;
    int offA[4], offB[2];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int row = a * 32 + (lane & 31);
        offA[a] = row * KT + (h ^ ((row >> 3) & 1)) * 8;
    }
#pragma unroll
    for (int b = 0; b < 2; ++b)
        offB[b] = rrow * 256 + ((((wave * 64 + b * 32) >> 3) ^ swz) + lchunk) * 8 + half;

    f32x16 acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int pre = ntiles < kNarrowStages - 1 ? ntiles : kNarrowStages - 1;
    for (int i = 0; i < pre; ++i) issue(i);
    for (int i = 0; i < ntiles; ++i) {
        // tile i has landed once only the loads of the one younger tile in flight are pending
        if (i + 1 < ntiles) wait_vmcnt<kNarrowLoads>(); else wait_vmcnt<0>();
        __syncthreads();  // every wavefront's part of tile i has landed; tile i-1 is used up
        asm volatile("" ::: "memory");
        if (i + kNarrowStages - 1 < ntiles) issue(i + kNarrowStages - 1);  // into the stage of tile i-1
        const uint16_t* st = narrow_lds + (i % kNarrowStages) * kNarrowStageBytes / 2;
        s16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            v[e] = mycol >= 0 ? static_cast<short>(st[(cslot * 8 + e) * row_pitch + mycol]) : short{0};
        *reinterpret_cast<s16x8*>(compact + cwrite) = v;
        __syncthreads();
        const uint16_t* xs = st + kNarrowDyBytes / 2;
        bf16x8 fa[4], fb[2];
#pragma unroll
        for (int a = 0; a < 4; ++a)
            fa[a] = *reinterpret_cast<const lds_bf16x8*>((lds_void_t*)(compact + offA[a]));
#pragma unroll
        for (int b = 0; b < 2; ++b) fb[b] = read_frag_swz(xs + offB[b]);
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        __syncthreads();  // the compact block and the stage are free again
    }

    float* P = g.P + (static_cast<int64_t>(split) * g.Mp + sg.off + row0) * g.Np + n0 + wave * 64;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = a * 32 + 8 * (v / 4) + 4 * h + (v % 4);
            if (row0 + row < sg.rows) {
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    P[static_cast<int64_t>(row) * g.Np + b * 32 + (lane & 31)] = acc[a][b][v];
            }
        }
}

}  // namespace
}  // namespace grass
