// grass_probe_mfma_rate: a measurement aid, not a step of the method.
//
// What the matrix cores of THIS machine sustain when a kernel does nothing but issue
// v_mfma_f32_32x32x16_bf16 (the instruction of the compressed-gradient GEMM) on every compute
// unit, with non-zero operands held in registers and no memory traffic.  The datasheet peak
// assumes the maximum clock; under this load the chip runs at whatever clock its power budget
// allows, and that differs from box to box, so the benchmark reports this figure next to the
// GEMM's own rate.
#include "common.hpp"

namespace grass {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// One wavefront per SIMD (4 per workgroup, one workgroup per compute unit), 16 independent
// accumulators per wavefront: the same register footprint and issue pattern as the GEMM.
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* __restrict__ out, int iters) {
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[i][e] = static_cast<__bf16>(0.37f * static_cast<float>(threadIdx.x % 7 + i + e));
            b[i][e] = static_cast<__bf16>(0.37f * static_cast<float>(threadIdx.x % 5 + i * e + 1));
        }
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    out[static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x] = s;
}

}  // namespace

grass_status launch_probe_mfma_rate(float* out, int iters, hipStream_t s) {
    mfma_rate_kernel<<<kProbeWorkgroups, 256, 0, s>>>(out, iters);
    return launch_status();
}

}  // namespace grass
