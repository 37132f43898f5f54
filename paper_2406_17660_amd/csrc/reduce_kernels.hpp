// Split-K and row-statistic reductions; the fp32 FMA GEMM of the reference-precision path.
// Included by cgrad.hip only (device code shares one translation unit with its launchers).
#pragma once
#include "common.hpp"
#include "gemm_common.hpp"

namespace grass {
namespace {

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


}  // namespace
}  // namespace grass
