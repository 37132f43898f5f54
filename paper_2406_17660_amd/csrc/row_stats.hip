// grass_row_stats: squared 2-norm of every row of G (compute_P's statistic, Section 3.2).
//
// HBM-bound streaming reduction: m*n elements are read once, m floats written.  One
// 64-lane wavefront owns one row; lanes read 16-byte vectors (coalesced 1 KiB per wave
// load), accumulate in fp32 and combine with cross-lane shuffles.  Four wavefronts share
// a workgroup only to keep the grid small.
#include "common.hpp"

namespace grass {
namespace {

constexpr int kRowsPerBlock = 4;

template <typename T>
struct Vec16;
template <>
struct Vec16<float> {
    static constexpr int kElems = 4;
    __device__ static float sumsq(const uint4& v) {
        const float a = __uint_as_float(v.x), b = __uint_as_float(v.y);
        const float c = __uint_as_float(v.z), d = __uint_as_float(v.w);
        return a * a + b * b + c * c + d * d;
    }
};
template <>
struct Vec16<uint16_t> {
    static constexpr int kElems = 8;
    __device__ static float sumsq(const uint4& v) {
        float s = 0.f;
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = __uint_as_float(w[i] << 16);
            const float hi = __uint_as_float(w[i] & 0xFFFF0000u);
            s += lo * lo + hi * hi;
        }
        return s;
    }
};

template <typename T, bool kVector>
__global__ __launch_bounds__(kWave* kRowsPerBlock) void row_stats_kernel(
    const T* __restrict__ G, int64_t m, int64_t n, int64_t ldg, float* __restrict__ sumsq) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock + (threadIdx.x / kWave);
    if (row >= m) return;
    const T* g = G + row * ldg;
    float acc = 0.f;
    if (kVector) {
        constexpr int E = Vec16<T>::kElems;
        const int64_t nvec = n / E;
        const uint4* gv = reinterpret_cast<const uint4*>(g);
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        int64_t v = lane;
        for (; v + 3 * kWave < nvec; v += 4 * kWave) {  // four independent loads in flight
            const uint4 x0 = gv[v], x1 = gv[v + kWave], x2 = gv[v + 2 * kWave],
                        x3 = gv[v + 3 * kWave];
            a0 += Vec16<T>::sumsq(x0);
            a1 += Vec16<T>::sumsq(x1);
            a2 += Vec16<T>::sumsq(x2);
            a3 += Vec16<T>::sumsq(x3);
        }
        for (; v < nvec; v += kWave) a0 += Vec16<T>::sumsq(gv[v]);
        acc = (a0 + a1) + (a2 + a3);
        for (int64_t i = nvec * E + lane; i < n; i += kWave) {
            const float x = load_as_f32(g + i);
            acc += x * x;
        }
    } else {
        for (int64_t i = lane; i < n; i += kWave) {
            const float x = load_as_f32(g + i);
            acc += x * x;
        }
    }
    acc = wave_sum(acc);
    if (lane == 0) sumsq[row] = acc;
}

template <typename T>
grass_status launch_typed(const void* G, int64_t m, int64_t n, int64_t ldg, float* sumsq,
                          hipStream_t s) {
    const dim3 block(kWave * kRowsPerBlock);
    const dim3 grid(static_cast<unsigned>((m + kRowsPerBlock - 1) / kRowsPerBlock));
    const bool vec = aligned_to(G, 16) && (ldg * sizeof(T)) % 16 == 0;
    if (vec)
        row_stats_kernel<T, true><<<grid, block, 0, s>>>(static_cast<const T*>(G), m, n, ldg, sumsq);
    else
        row_stats_kernel<T, false><<<grid, block, 0, s>>>(static_cast<const T*>(G), m, n, ldg, sumsq);
    return launch_status();
}

}  // namespace

grass_status launch_row_stats(const void* G, grass_dtype dt, int64_t m, int64_t n, int64_t ldg,
                              float* sumsq, hipStream_t s) {
    if (m == 0) return GRASS_OK;
    return dt == GRASS_F32 ? launch_typed<float>(G, m, n, ldg, sumsq, s)
                           : launch_typed<uint16_t>(G, m, n, ldg, sumsq, s);
}

}  // namespace grass
