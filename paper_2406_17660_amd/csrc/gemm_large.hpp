// bf16 MFMA GEMM with 256 x 256 tiles, load-to-LDS ring: the hot kernel.
// Included by cgrad.hip only (device code shares one translation unit with its launchers).
#pragma once
#include "common.hpp"
#include "gemm_common.hpp"
#include "gemm_small.hpp"  // GemmArgs

namespace grass {
namespace {

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
//
// kAPairs (with kARows): the rows of the left operand are fetched 64 values of k at a time, one
// whole 128-byte cache line per row and request instead of half a line per K tile (half-line
// requests make the loads of this operand twice as expensive as those of a packed panel).  The
// four A blocks of the ring then form two blocks of [256 rows][64 k] (128 bytes per row, 16-byte
// slot c of row j stored at slot c ^ ((j / 2) % 8)), each serving two consecutive K tiles: the
// pair (i, i+1), i even, is loaded during K tile i-2, right after the pair (i-2, i-1) has been
// used up.  B keeps its four single stages.  Needs an even number of K tiles per workgroup.
template <bool kDense, bool kRowStats = false, bool kARows = false, bool kAPairs = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void tn_gemm_bf16_direct_kernel(GemmArgs g) {
    static_assert(!kAPairs || kARows, "paired A stages are a form of the row-gathering kernel");
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
    // kAPairs: load q (0..7) of this wavefront fills rows 8 (4 q + wave) .. +8 of a pair block,
    // eight lanes per row; the lane that fills physical slot p of row j fetches logical slot
    // p ^ ((j / 2) % 8) of the 64 values of k.
    uint32_t lanePair[kAPairs ? 8 : 1];
    if (kAPairs) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int trow = 8 * (4 * q + wave) + (lane >> 3);
            int64_t j = m0 + trow;
            if (j >= g.Mcols) j = 0;
            const int64_t src = g.a_rows ? g.a_rows[j] : j;
            const int lslot = (lane & 7) ^ ((trow >> 1) & 7);
            lanePair[q] = static_cast<uint32_t>((src * g.lda + lslot * 8) * 2);
        }
    }
    const int64_t tileA = kARows ? kFastBK : kFastBK * g.lda, tileB = kFastBK * g.ldb;
    const int ldsrow = wave * 2;  // first LDS row this wavefront writes in a pass

    // Loads of K tile number `i` (counted from this workgroup's first tile) into its ring
    // stage, split into kFastLoadsPerTile single instructions (part = 0..7: A rows 8p.., then
    // B rows) so that the main loop can space them out between MFMA groups: the four
    // wavefronts of a workgroup share one address unit, and eight back-to-back 1 KiB loads
    // from each of them right after a barrier stall the last wavefront's MFMAs.
    const uint32_t ring_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void_t*)ring));
    // Element offsets of the A and B blocks of K tile i inside the ring.  Paired form: A pair
    // blocks at 0 and 32 KiB, the four B stages behind them.
    auto a_base = [&](int i) -> int {
        return kAPairs ? ((i >> 1) & 1) * 2 * kFastOperandElems : (i % kFastStages) * kFastStageElems;
    };
    auto b_base = [&](int i) -> int {
        return kAPairs ? (4 + i % kFastStages) * kFastOperandElems
                       : (i % kFastStages) * kFastStageElems + kFastOperandElems;
    };
    // paired form: load q of the pair that starts at K tile i (i even); B loads of K tile i
    auto issue_pair_part = [&](int i, int q) {
        load16_to_lds(gA, lanePair[kAPairs ? q : 0],
                      ring_base + (a_base(i) + (4 * q + wave) * 8 * 64) * 2);
    };
    auto issue_b_part = [&](int i, int part) {
        load16_to_lds(gB, laneB[part], ring_base + (b_base(i) + (ldsrow + part * 8) * 256) * 2);
    };
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
        if (kAPairs)  // row * 64 + (slot ^ ((row/2)%8)) * 8, slot = 4 (tile odd) + k16/8 + lane/32
            offA[i] = (wr * 128 + i * 32 + (lane & 31)) * 64 + ((h ^ (((lane & 31) >> 1) & 7)) * 8);
        else if (kARows)  // row wr*128 + 32i + lane%32, slot (k16/8 + lane/32) ^ ((row/4)%4); k16 added later
            offA[i] = (wr * 128 + i * 32 + (lane & 31)) * kFastBK + ((h ^ (((lane & 31) >> 2) & 3)) * 8);
        else
            offA[i] = rrow * 256 + ((((wr * 128 + i * 32) >> 3) ^ swz) + lchunk) * 8 + half;
        offB[i] = rrow * 256 + ((((wc * 128 + i * 32) >> 3) ^ swz) + lchunk) * 8 + half;
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
        if (kARows) {
            // slots 2, 3 hold k16 = 16: flipping bit 1 of the slot = element offset ^ 16; in the
            // paired form slots 4-7 hold the odd K tile of the pair: bit 2 of the slot, ^ 32
            const int flip = kAPairs ? k16 + 32 * (i & 1) : k16;
            const uint16_t* sa = ring + a_base(i) + (offA[a] ^ flip);
            return *reinterpret_cast<const lds_bf16x8*>((lds_void_t*)sa);
        }
        return read_frag_swz(ring + a_base(i) + k16 * 256 + offA[a]);
    };
    auto read_quarter = [&](Frags& f, int i, int k16, int part) {
        const uint16_t* st = ring + b_base(i) + k16 * 256;
        if (part == 0) { f.a[0] = read_a(i, k16, 0); f.b[0] = read_frag_swz(st + offB[0]); }
        else if (part == 1) { f.b[1] = read_frag_swz(st + offB[1]); f.b[2] = read_frag_swz(st + offB[2]); }
        else if (part == 2) { f.b[3] = read_frag_swz(st + offB[3]); f.a[1] = read_a(i, k16, 1); }
        else { f.a[2] = read_a(i, k16, 2); f.a[3] = read_a(i, k16, 3); }
    };
    auto read_frags = [&](Frags& f, int i, int k16) {
#pragma unroll
        for (int part = 0; part < 4; ++part) read_quarter(f, i, k16, part);
    };
    // Row `a` of the 4 x 4 fragment products of a slice.  Odd rows run through the columns
    // backwards, so that only one operand changes from the last instruction of a row to the
    // first of the next (fewer operand switches: measured 0.5 % faster; the kernel is bound
    // by power).
    auto mfma_row = [&](const Frags& f, int a) {
#pragma unroll
        for (int bb = 0; bb < 4; ++bb) {
            const int b = (a & 1) ? 3 - bb : bb;
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[a], f.b[b], acc[a][b], 0, 0, 0);
        }
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
    if constexpr (kAPairs) {
        // Paired A stages (ntiles is even).  Loads in program order:
        //   before the loop   A pair (0,1) x8, B(0) x4, B(1) x4, B(2) x4
        //   K tile i even     A pair (i+2, i+3) x8 during its first slice, B(i+3) x4 during its second
        //   K tile i odd      B(i+3) x4 during its second slice
        // so before an even tile 8 younger loads may still be in flight (its own pair was issued
        // two tiles earlier, followed by B x4 twice), before an odd tile 16 (B(i) was followed by
        // B x4 and a whole even tile's 12).
        auto slice_pair = [&](const Frags& cur, Frags& next, int next_tile, int next_k16, int kind,
                              int load_tile) {
#pragma unroll
            for (int part = 0; part < 4; ++part) {
                read_quarter(next, next_tile, next_k16, part);
                mfma_row(cur, part);
                interleave_hint4();
                __builtin_amdgcn_sched_barrier(0);
                if (kind == 1) {
                    issue_pair_part(load_tile, 2 * part);
                    issue_pair_part(load_tile, 2 * part + 1);
                } else if (kind == 2) {
                    issue_b_part(load_tile, part);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        auto issue_pair = [&](int i) {
#pragma unroll
            for (int q = 0; q < 8; ++q) issue_pair_part(i, q);
            gA += 2 * kFastBK;
        };
        auto issue_b = [&](int i) {
#pragma unroll
            for (int part = 0; part < 4; ++part) issue_b_part(i, part);
            gB += tileB;
        };
        if (ntiles > 0) {
            issue_pair(0);
            const int pre = ntiles < kAhead ? ntiles : kAhead;
            for (int t = 0; t < pre; ++t) issue_b(t);
            wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            read_frags(F, 0, 0);
            if (2 < ntiles) issue_pair(2);
            if (3 < ntiles) issue_b(3);
            read_frags(G, 0, 16);
            __builtin_amdgcn_sched_barrier(0);
            mfma16(F);
            __builtin_amdgcn_sched_barrier(0);
            int i = 1;
            for (; i + 4 < ntiles; i += 2) {
                // odd K tile i: its half of the pair arrived with tile i-1
                wait_vmcnt<16>();
                __builtin_amdgcn_s_waitcnt(0xC07F);
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                slice_pair(G, F, i, 0, 0, 0);
                slice_pair(F, G, i, 16, 2, i + 3);
                gB += tileB;
                // even K tile i+1: the pair (i+1, i+2) and B(i+1)
                wait_vmcnt<8>();
                __builtin_amdgcn_s_waitcnt(0xC07F);
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                slice_pair(G, F, i + 1, 0, 1, i + 3);
                slice_pair(F, G, i + 1, 16, 2, i + 4);
                gA += 2 * kFastBK;
                gB += tileB;
            }
            // drain: everything has been issued (the last even tile of the loop issued the
            // pair and the B tile that end the K range)
            for (; i < ntiles; ++i) {
                wait_vmcnt<0>();
                __builtin_amdgcn_s_waitcnt(0xC07F);
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                slice_pair(G, F, i, 0, 0, 0);
                slice_pair(F, G, i, 16, 0, 0);
            }
            mfma16(G);
        }
    } else if (ntiles > 0) {
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


}  // namespace
}  // namespace grass
