// Vector types, XCD count and tile numbering shared by the GEMM, packing and reduction kernels.
// Included by cgrad.hip only (device code shares one translation unit with its launchers).
#pragma once
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


}  // namespace
}  // namespace grass
