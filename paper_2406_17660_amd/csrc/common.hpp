// Shared device helpers for the gfx950 kernels: bf16 conversion, wavefront (64-lane)
// reductions and scans, launch-error mapping.  Nothing here is used by the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/grass.h"

namespace grass {

constexpr int kWave = 64;  // CDNA wavefront width

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// Round to nearest even; NaN stays NaN (quiet), as IEEE conversion does.
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

template <typename T>
__device__ __forceinline__ float load_as_f32(const T* p);
template <>
__device__ __forceinline__ float load_as_f32<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_as_f32<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }

template <typename T>
__device__ __forceinline__ void store_from_f32(T* p, float v);
template <>
__device__ __forceinline__ void store_from_f32<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_from_f32<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        const double w = __shfl_xor(v, o, kWave);
        v = w > v ? w : v;
    }
    return v;
}

// Inclusive prefix sum across the 64 lanes of a wavefront.
template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const T up = __shfl_up(v, o, kWave);
        if (lane >= o) v += up;
    }
    return v;
}

inline grass_status launch_status() {
    return hipGetLastError() == hipSuccess ? GRASS_OK : GRASS_ERR_DEVICE;
}

inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Value of a test hook (grass_set_test_option): 0 unless a test has forced a code path.
int test_option(grass_test_option which);

// Kernel launchers, one per translation unit.  All pointers are device pointers; shapes
// have been validated by the C entry points in api.hip before these are called.
grass_status launch_row_stats(const void* G, grass_dtype dt, int64_t m, int64_t n, int64_t ldg,
                              float* sumsq, hipStream_t s);
grass_status launch_select(const float* sumsq, int64_t m, int64_t r, grass_method method,
                           int replacement, grass_scale scale, uint64_t seed, uint64_t refresh_id,
                           int32_t* idx, float* rho, void* ws, hipStream_t s);
size_t select_workspace_bytes(int64_t m, int64_t r, grass_method method, int replacement);
// The same selection with the library's own static device scratch in place of `ws`; `status`:
// the caller's device status word, or nullptr.
size_t select_static_scratch_bytes();
grass_status launch_select_static(const float* sumsq, int64_t m, int64_t r, grass_method method,
                                  int replacement, grass_scale scale, uint64_t seed,
                                  uint64_t refresh_id, int32_t* idx, float* rho, int32_t* status,
                                  hipStream_t s);
// M and V have dtype sdt (fp32, or bf16 moments rounded once per step).
grass_status launch_adam_rows(const float* GC, int64_t ldgc, void* M, void* V, grass_dtype sdt,
                              int64_t r, int64_t n, float lr, float b1, float b2, float eps,
                              int64_t t, float* U, hipStream_t s);
grass_status launch_scatter(void* W, grass_dtype wdt, int64_t n, int64_t ldw, const int32_t* idx,
                            const float* rho, float alpha, const float* U, int64_t r,
                            hipStream_t s);
grass_status launch_scatter_cols(void* W, grass_dtype wdt, int64_t mrows, int64_t ldw,
                                 const int32_t* idx, const float* rho, float alpha, const float* U,
                                 int64_t r, hipStream_t s);
grass_status launch_adam_scatter(const float* GC, int64_t ldgc, void* M, void* V, grass_dtype sdt,
                                 int64_t r, int64_t n, float lr, float b1, float b2, float eps,
                                 int64_t t, void* W, grass_dtype wdt, int64_t ldw,
                                 const int32_t* idx, const float* rho, float alpha, hipStream_t s,
                                 const float* step_scalars = nullptr);
// {lr, 1/(1-b1^t), 1/(1-b2^t)}: what the Adam kernels read from device memory when a captured
// step is replayed (step_scalars != nullptr above; lr and t of the call are then ignored).
void adam_step_scalars(float lr, float b1, float b2, int64_t t, float out[3]);
grass_status launch_gather_rows(const void* G, grass_dtype gdt, int64_t n, int64_t ldg,
                                const int32_t* idx, const float* rho, int64_t r, float* out,
                                int64_t ldo, hipStream_t s);
// C[j, i] = scale_j * sum_t A[t, col_j] * B[t, i]  (cgrad: col_j = idx[j], scale_j = rho[j];
// dense: idx = rho = nullptr).  Output dtype odt, leading dimension ldc.
size_t gemm_workspace_bytes(int64_t T, int64_t mrows, int64_t n, grass_dtype dt,
                            grass_dy_layout layout, bool gathered);
// Tile edge and number of K slices the launcher plans for `count` gathered sets of `rows` rows in
// all (m: row length of dY, 0 when not known; tile 0 = the kernel that gathers inside the GEMM).
void gemm_plan_summary(int64_t T, int64_t m, int64_t rows, int count, int64_t n, grass_dtype dt,
                       grass_dy_layout layout, int* tile, int* k_slices);
grass_status launch_tn_gemm(const void* dY, grass_dy_layout layout, int64_t ldy, const void* X,
                            int64_t ldx, grass_dtype dt, int64_t T, int64_t mrows, int64_t n,
                            const int32_t* idx, const float* rho, void* C, grass_dtype odt,
                            int64_t ldc, void* ws, hipStream_t s, int64_t src_rows,
                            hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);

// What follows the compressed gradient in a regular step (Adam on r x n, update of the rows of
// W).  Given to the GEMM launcher, the split-K reduction, Adam and the update run as one kernel
// that reads the partial tiles directly; G_C is then only written when the segment names an
// output for it.
struct StepTail {
    void* M;
    void* V;
    grass_dtype sdt;
    float lr, beta1, beta2, eps;
    int64_t t;
    const float* step_scalars;  // device {lr, 1/(1-b1^t), 1/(1-b2^t)} or nullptr
    void* W;
    grass_dtype wdt;
    int64_t ldw;
    float alpha;
    // Column form (U != nullptr): the set's rows are columns of W.  Adam's output goes to U
    // (rows x n fp32, contiguous) and W (w_rows = n rows) gets W[:, idx[j]] += alpha rho_j U[j, :].
    // step_scalars is not supported in this form.
    float* U = nullptr;
    int64_t w_rows = 0;
};
// True when M, V, W or U (and GC, if given) allow the 16-byte accesses of the fused kernel.
bool reduce_adam_scatter_ok(const StepTail& t, int64_t n, const float* GC, int64_t ldgc);
// One row set of the fused tail.  part: partial tiles [slices][Mp][Np], already offset to this
// set's first row; GC: where to store the compressed gradient, or nullptr.
struct TailSet {
    const float* part;
    int64_t r;
    void* M;
    void* V;
    void* W;
    int64_t ldw;
    const int32_t* idx;
    const float* rho;
    float* GC;
    int64_t ldgc;
    float* U;  // column form: Adam's output (r x n, contiguous) instead of the update of W
};
struct TailSets {
    TailSet set[GRASS_MAX_GROUP];
};
// The fused tail for `count` row sets in one launch.  The sets share the partial-tile geometry,
// n, the dtypes, the form (row or column) and Adam's scalars, which are taken from `t` (its M, V,
// W, U are not read).  In column form the caller launches the column update afterwards.
// ev_start / ev_stop: optional events that receive the kernel's own start and stop times.
grass_status launch_reduce_adam_scatter(const TailSets& sets, int count, int slices, int64_t Mp,
                                        int64_t Np, int64_t n, const StepTail& t, hipStream_t s,
                                        hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);

// A kernel launch that, given events, has the runtime stamp them with the start and the end of
// this very dispatch (what a profiler's kernel trace reports), instead of events recorded as
// separate commands before and after it, which add the gaps between commands to the interval.
template <typename Kernel, typename... Args>
inline void launch_stamped(Kernel kernel, dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t s,
                           hipEvent_t ev_start, hipEvent_t ev_stop, Args... args) {
    if (ev_start || ev_stop)
        hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, s, ev_start, ev_stop, 0, args...);
    else
        kernel<<<grid, block, lds_bytes, s>>>(args...);
}

// The same product for several row sets that share X (one packed panel, one GEMM).
struct GemmSegment {
    const void* dY;      // this set's left operand
    int64_t ldy;
    const int32_t* idx;  // its selected rows (device), and their scales
    const float* rho;
    void* C;             // its rows x n output
    int64_t ldc;
    int64_t rows;
    int64_t src_rows;    // rows of dY's matrix that idx may name (m); bounds address arithmetic
    // regular step: Adam + update after (fused with) the reduction.  C must then be a valid
    // rows x n fp32 buffer in any case (the unfused route goes through it); c_wanted says
    // whether the caller asked for G_C, i.e. whether the fused kernel has to write it.
    const StepTail* tail = nullptr;
    bool c_wanted = true;
};
size_t gemm_group_workspace_bytes(int64_t T, const int64_t* rows, int count, int64_t n,
                                  grass_dtype dt, grass_dy_layout layout);
// ev_start / ev_stop: stamped with the start and the end of the matrix-multiply kernel (the
// large-tile kernel's own dispatch; for the other kernels, recorded before and after the
// launches); ev_tail_start / ev_tail_stop: the same for the fused tail of a regular step.
grass_status launch_tn_gemm_segments(const GemmSegment* seg, int count, grass_dy_layout layout,
                                     const void* X, int64_t ldx, grass_dtype dt, int64_t T,
                                     int64_t n, grass_dtype odt, void* ws, hipStream_t s,
                                     hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr,
                                     hipEvent_t ev_tail_start = nullptr,
                                     hipEvent_t ev_tail_stop = nullptr);

// Row statistic of G = dY^T X without storing G (fused into the GEMM when the shape allows).
size_t grad_row_stats_workspace_bytes(int64_t T, int64_t m, int64_t n, grass_dtype dt,
                                      grass_dy_layout layout, int64_t ldy, int64_t ldx);
grass_status launch_grad_row_stats(const void* dY, grass_dy_layout layout, int64_t ldy,
                                   const void* X, int64_t ldx, grass_dtype dt, int64_t T, int64_t m,
                                   int64_t n, float* sumsq, void* ws, size_t ws_bytes,
                                   hipStream_t s);

}  // namespace grass
