// mfma_rate_probe: a measurement aid for the benchmark, not a step of the method and not part
// of the GRASS library (it is built into a library of its own, libgrass_probe.so).
//
// What the matrix cores of THIS machine sustain when a kernel does nothing but issue
// v_mfma_f32_32x32x16_bf16 (the instruction of the compressed-gradient GEMM) on every compute
// unit.  The datasheet peak assumes the maximum clock; under this load the chip runs at whatever
// clock its power budget allows, and the power of a matrix instruction depends on its operands,
// so the probe has three operand sources:
//   constants      small multiples of a constant held in registers (few bits change between
//                  consecutive instructions: the most favourable case)
//   registers      the caller's values (say, normal deviates like the GEMM's inputs), two sets
//                  of eight fragments held in registers and used alternately
//   LDS            the caller's values staged in LDS once; every group of 16 instructions reads
//                  its eight fragments from there, 16 bytes per lane and fragment, which is the
//                  LDS read traffic of the GEMM (no global memory traffic in the loop)
// The benchmark reports these next to the GEMM's own rate.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mfma_rate_probe.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int kProbeWorkgroups = 256;
constexpr int kProbeOperandBytes = 65536;
constexpr int kPoolElems = kProbeOperandBytes / 2;

// One wavefront per SIMD (4 per workgroup, one workgroup per compute unit), 16 independent
// accumulators per wavefront, two alternating sets of 4 + 4 operand fragments: the register
// footprint and issue pattern of the GEMM.  kSource: 0 constants, 1 registers, 2 LDS.
template <int kSource>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void mfma_rate_kernel(const uint16_t* __restrict__ pool, float* __restrict__ out, int iters) {
    __shared__ __attribute__((aligned(16))) uint16_t lds[kSource == 2 ? kPoolElems : 8];
    const int tid = threadIdx.x, lane = tid & 63;
    if (kSource == 2) {
        for (int i = tid; i < kPoolElems / 8; i += 256)
            *reinterpret_cast<s16x8*>(lds + i * 8) = *reinterpret_cast<const s16x8*>(pool + i * 8);
        __syncthreads();
    }
    bf16x8 a[2][4], b[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (kSource == 0) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    a[s][i][e] = static_cast<__bf16>(0.37f * static_cast<float>(tid % 7 + i + e));
                    b[s][i][e] = static_cast<__bf16>(0.37f * static_cast<float>(tid % 5 + i * e + 1));
                }
            } else {  // fragment f of set s: 16 bytes per thread at ((8 s + f) * 256 + tid) * 8
                a[s][i] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const s16x8*>(pool + ((s * 8 + i) * 256 + tid) * 8));
                b[s][i] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const s16x8*>(pool + ((s * 8 + 4 + i) * 256 + tid) * 8));
            }
        }
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    // LDS source: fragment k of the current group is this lane's 16 bytes of the 1 KiB row
    // starting at off + 512 k elements; off moves on after every group and wraps inside the pool
    // (it stays a multiple of 8, so a read never crosses the end).
    int off = lane * 8;
    auto read = [&](int k) -> bf16x8 {
        return __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const s16x8*>(lds + ((off + k * 512) & (kPoolElems - 1))));
    };
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int part = 0; part < 4; ++part) {
                if (kSource == 2) {  // two fragments of the other set per four instructions
                    if (part == 0) { a[s ^ 1][0] = read(0); b[s ^ 1][0] = read(1); }
                    else if (part == 1) { b[s ^ 1][1] = read(2); b[s ^ 1][2] = read(3); }
                    else if (part == 2) { b[s ^ 1][3] = read(4); a[s ^ 1][1] = read(5); }
                    else { a[s ^ 1][2] = read(6); a[s ^ 1][3] = read(7); }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[part][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s][part], b[s][j],
                                                                           acc[part][j], 0, 0, 0);
                if (kSource == 2) {
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // two MFMAs
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kSource == 2) off = (off + 4096 + 8) & (kPoolElems - 1);
        }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += acc[i][j][v];
    out[static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x] = sum;
}

}  // namespace

extern "C" int mfma_rate_probe(int source, const void* operands, size_t operand_bytes, float* out,
                               size_t out_floats, int iters, double* flops, void* stream) {
    if (!out || !flops) return MFMA_PROBE_ERR_NULL;
    if (source < MFMA_PROBE_CONSTANTS || source > MFMA_PROBE_LDS) return MFMA_PROBE_ERR_SOURCE;
    if (source != MFMA_PROBE_CONSTANTS) {
        if (!operands) return MFMA_PROBE_ERR_NULL;
        if (operand_bytes < static_cast<size_t>(kProbeOperandBytes) ||
            reinterpret_cast<uintptr_t>(operands) % 16 != 0)
            return MFMA_PROBE_ERR_SIZE;
    }
    if (iters < 1 || out_floats < static_cast<size_t>(kProbeWorkgroups) * 256) return MFMA_PROBE_ERR_SIZE;
    // 4 wavefronts per workgroup, 32 instructions of 32 x 32 x 16 multiply-adds per iteration
    *flops = static_cast<double>(kProbeWorkgroups) * 4.0 * iters * 32.0 * (2.0 * 32 * 32 * 16);
    const uint16_t* pool = static_cast<const uint16_t*>(operands);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (source == 0) mfma_rate_kernel<0><<<kProbeWorkgroups, 256, 0, s>>>(pool, out, iters);
    else if (source == 1) mfma_rate_kernel<1><<<kProbeWorkgroups, 256, 0, s>>>(pool, out, iters);
    else mfma_rate_kernel<2><<<kProbeWorkgroups, 256, 0, s>>>(pool, out, iters);
    return hipGetLastError() == hipSuccess ? MFMA_PROBE_OK : MFMA_PROBE_ERR_DEVICE;
}
