// grass_adam_rows, grass_scatter_update, grass_adam_scatter, grass_gather_rows.
//
// All four are HBM-bound elementwise passes over r x n values.  A workgroup of 256
// threads owns 1024 consecutive columns of one compressed row j (grid = column chunks
// x r); each thread handles four consecutive columns with 16-byte loads and stores of
// the fp32 arrays (8-byte for bf16 W), so every wave access is a contiguous 1 KiB.
// Buffers whose base or leading dimension breaks that alignment take the one-element-
// per-thread variant of the same kernel.
//
// Rows selected more than once (sampling with replacement) sit next to each other in
// the sorted idx.  The workgroups of the first occurrence walk the whole run, so a row
// of W is written by exactly one thread per column: no atomics, deterministic sums.
#include "common.hpp"

namespace grass {
namespace {

constexpr int kThreads = 256;

struct AdamParams {
    float b1, one_minus_b1, b2, one_minus_b2;
    float inv_c1, inv_c2;  // reciprocals of the bias corrections 1 - beta^t
    float lr, eps;
    // When set: device array {lr, inv_c1, inv_c2} that replaces the three values above, so that
    // a captured launch can be replayed for later steps (the caller rewrites the array).
    const float* step_scalars;
};

// The values of this step: from the launch arguments, or from device memory.
__device__ __forceinline__ AdamParams resolve(AdamParams p) {
    if (p.step_scalars) {
        p.lr = p.step_scalars[0];
        p.inv_c1 = p.step_scalars[1];
        p.inv_c2 = p.step_scalars[2];
    }
    return p;
}

// What a moment becomes when it is stored: itself in fp32, the nearest bf16 value otherwise.
template <typename ST>
__device__ __forceinline__ float as_stored(float x);
template <>
__device__ __forceinline__ float as_stored<float>(float x) { return x; }
template <>
__device__ __forceinline__ float as_stored<uint16_t>(float x) { return bf16_to_f32(f32_to_bf16(x)); }

// adam.update of Appendix A for one element; returns U.  With bf16 moments the update is
// computed from the values that are stored, so it is a function of the saved state.
template <typename ST>
__device__ __forceinline__ float adam_elem(float g, float& m, float& v, const AdamParams& p) {
    m = as_stored<ST>(p.b1 * m + p.one_minus_b1 * g);
    v = as_stored<ST>(p.b2 * v + p.one_minus_b2 * g * g);
    const float ms = m * p.inv_c1;
    const float vs = v * p.inv_c2;
    // hardware square root and reciprocal (about 1 ulp each): the kernel is otherwise bound by
    // memory and the correctly rounded sequences would make its arithmetic show
    return -p.lr * ms * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(vs) + p.eps);
}

// Vectors of VEC consecutive elements.  load / store are the ordinary accesses; load_once /
// store_once carry the streaming hint (non-temporal) and are for the Adam moments and the rows of
// W in the fused kernels: each element is read once and written once per step and is not needed
// again before hundreds of megabytes of other traffic have passed, so keeping it in the caches
// only displaces data.  Measured on the 4096-wide layer with state that is cold (eight sets
// cycled): 20.9 -> 17.3 us with both hints, and 16.6 -> 15.7 us with the state warm in the
// last-level cache; hinted loads or stores alone gain less or nothing.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

template <int VEC>
struct F32Vec;
template <>
struct F32Vec<4> {
    float x[4];
    __device__ void load(const float* p) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    }
    __device__ void store(float* p) const {
        *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
    }
    __device__ void load_once(const float* p) {
        const f32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    }
    __device__ void store_once(float* p) const {
        const f32x4_t t = {x[0], x[1], x[2], x[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<f32x4_t*>(p));
    }
};
template <>
struct F32Vec<1> {
    float x[1];
    __device__ void load(const float* p) { x[0] = *p; }
    __device__ void store(float* p) const { *p = x[0]; }
    __device__ void load_once(const float* p) { x[0] = __builtin_nontemporal_load(p); }
    __device__ void store_once(float* p) const { __builtin_nontemporal_store(x[0], p); }
};

template <typename WT, int VEC>
struct WVec;
template <>
struct WVec<float, 4> : F32Vec<4> {};
template <>
struct WVec<float, 1> : F32Vec<1> {};
template <>
struct WVec<uint16_t, 4> {
    float x[4];
    __device__ void load(const uint16_t* p) {
        const uint2 t = *reinterpret_cast<const uint2*>(p);
        x[0] = __uint_as_float(t.x << 16); x[1] = __uint_as_float(t.x & 0xFFFF0000u);
        x[2] = __uint_as_float(t.y << 16); x[3] = __uint_as_float(t.y & 0xFFFF0000u);
    }
    __device__ void store(uint16_t* p) const {
        uint2 t;
        t.x = f32_to_bf16(x[0]) | (static_cast<uint32_t>(f32_to_bf16(x[1])) << 16);
        t.y = f32_to_bf16(x[2]) | (static_cast<uint32_t>(f32_to_bf16(x[3])) << 16);
        *reinterpret_cast<uint2*>(p) = t;
    }
    __device__ void load_once(const uint16_t* p) {
        const u32x2_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
        x[0] = __uint_as_float(t.x << 16); x[1] = __uint_as_float(t.x & 0xFFFF0000u);
        x[2] = __uint_as_float(t.y << 16); x[3] = __uint_as_float(t.y & 0xFFFF0000u);
    }
    __device__ void store_once(uint16_t* p) const {
        u32x2_t t;
        t.x = f32_to_bf16(x[0]) | (static_cast<uint32_t>(f32_to_bf16(x[1])) << 16);
        t.y = f32_to_bf16(x[2]) | (static_cast<uint32_t>(f32_to_bf16(x[3])) << 16);
        __builtin_nontemporal_store(t, reinterpret_cast<u32x2_t*>(p));
    }
};
template <>
struct WVec<uint16_t, 1> {
    float x[1];
    __device__ void load(const uint16_t* p) { x[0] = bf16_to_f32(*p); }
    __device__ void store(uint16_t* p) const { *p = f32_to_bf16(x[0]); }
    __device__ void load_once(const uint16_t* p) { x[0] = bf16_to_f32(__builtin_nontemporal_load(p)); }
    __device__ void store_once(uint16_t* p) const { __builtin_nontemporal_store(f32_to_bf16(x[0]), p); }
};

// Column range of this thread: [c, c + cnt), cnt in 0..VEC.  Full vectors take the wide
// path; a ragged last vector is handled element by element by the caller.
template <int VEC>
__device__ __forceinline__ int64_t thread_col(int64_t n, int& cnt) {
    const int64_t c = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * VEC;
    const int64_t left = n - c;
    cnt = left >= VEC ? VEC : (left > 0 ? static_cast<int>(left) : 0);
    return c;
}

template <typename ST, int VEC>
__global__ __launch_bounds__(kThreads) void adam_rows_kernel(
    const float* __restrict__ GC, int64_t ldgc, ST* __restrict__ M, ST* __restrict__ V,
    float* __restrict__ U, int64_t n, AdamParams p_in) {
    const AdamParams p = resolve(p_in);
    const int64_t j = blockIdx.y;
    int cnt;
    const int64_t c = thread_col<VEC>(n, cnt);
    if (cnt == 0) return;
    const float* g = GC + j * ldgc + c;
    ST* mp = M + j * n + c;
    ST* vp = V + j * n + c;
    float* up = U + j * n + c;
    if (cnt == VEC) {
        F32Vec<VEC> gv, uv;
        WVec<ST, VEC> mv, vv;
        gv.load(g); mv.load(mp); vv.load(vp);
#pragma unroll
        for (int e = 0; e < VEC; ++e) uv.x[e] = adam_elem<ST>(gv.x[e], mv.x[e], vv.x[e], p);
        mv.store(mp); vv.store(vp); uv.store(up);
    } else {
        for (int e = 0; e < cnt; ++e) {
            float mm = load_as_f32(mp + e), vv = load_as_f32(vp + e);
            up[e] = adam_elem<ST>(g[e], mm, vv, p);
            store_from_f32(mp + e, mm);
            store_from_f32(vp + e, vv);
        }
    }
}

// W[idx[j], :] += alpha * sum over the run of equal idx of rho * U.
template <typename WT, int VEC>
__global__ __launch_bounds__(kThreads) void scatter_kernel(
    WT* __restrict__ W, int64_t ldw, const int32_t* __restrict__ idx,
    const float* __restrict__ rho, float alpha, const float* __restrict__ U, int64_t n, int64_t r) {
    const int64_t j = blockIdx.y;
    const int32_t row = idx[j];
    if (j > 0 && idx[j - 1] == row) return;  // a later member of a run: the first one does it
    int cnt;
    const int64_t c = thread_col<VEC>(n, cnt);
    if (cnt == 0) return;
    WT* wp = W + static_cast<int64_t>(row) * ldw + c;
    if (cnt == VEC) {
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
        for (int64_t jj = j; jj < r && idx[jj] == row; ++jj) {
            F32Vec<VEC> uv;
            uv.load(U + jj * n + c);
            const float s = rho[jj];
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += s * uv.x[e];
        }
        WVec<WT, VEC> wv;
        wv.load(wp);
#pragma unroll
        for (int e = 0; e < VEC; ++e) wv.x[e] += alpha * acc[e];
        wv.store(wp);
    } else {
        for (int e = 0; e < cnt; ++e) {
            float acc = 0.f;
            for (int64_t jj = j; jj < r && idx[jj] == row; ++jj) acc += rho[jj] * U[jj * n + c + e];
            store_from_f32(wp + e, load_as_f32(wp + e) + alpha * acc);
        }
    }
}

// Adam on every row of the run, then one write of W; U stays in registers.  A thread owns
// UNROLL vectors of VEC columns, kThreads * VEC columns apart, and issues the loads of all of
// them before it computes: the row index has to be fetched before anything else can start,
// so the more bytes a wavefront then has in flight the better that latency is amortised.
template <typename WT, typename ST, int VEC, int UNROLL>
__global__ __launch_bounds__(kThreads) void adam_scatter_kernel(
    const float* __restrict__ GC, int64_t ldgc, ST* __restrict__ M, ST* __restrict__ V,
    int64_t n, int64_t r, AdamParams p_in, WT* __restrict__ W, int64_t ldw,
    const int32_t* __restrict__ idx, const float* __restrict__ rho, float alpha) {
    const AdamParams p = resolve(p_in);
    const int64_t j = blockIdx.y;
    const int32_t row = idx[j];
    if (j > 0 && idx[j - 1] == row) return;
    const int64_t c0 = (static_cast<int64_t>(blockIdx.x) * kThreads * UNROLL + threadIdx.x) * VEC;
    constexpr int64_t kStride = static_cast<int64_t>(kThreads) * VEC;
    if (c0 >= n) return;
    WT* wrow = W + static_cast<int64_t>(row) * ldw;
    if (c0 + (UNROLL - 1) * kStride + VEC <= n) {  // every vector of this thread is whole
        WVec<WT, VEC> wv[UNROLL];
        float acc[UNROLL][VEC];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            wv[u].load_once(wrow + c0 + u * kStride);  // issued first: independent of the Adam loads
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[u][e] = 0.f;
        }
        for (int64_t jj = j; jj < r && idx[jj] == row; ++jj) {
            F32Vec<VEC> gv[UNROLL];
            WVec<ST, VEC> mv[UNROLL], vv[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                gv[u].load(GC + jj * ldgc + c0 + u * kStride);
                mv[u].load_once(M + jj * n + c0 + u * kStride);
                vv[u].load_once(V + jj * n + c0 + u * kStride);
            }
            const float s = rho[jj];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    acc[u][e] += s * adam_elem<ST>(gv[u].x[e], mv[u].x[e], vv[u].x[e], p);
                mv[u].store_once(M + jj * n + c0 + u * kStride);
                vv[u].store_once(V + jj * n + c0 + u * kStride);
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) wv[u].x[e] += alpha * acc[u][e];
            wv[u].store_once(wrow + c0 + u * kStride);
        }
        return;
    }
    // ragged end of the row: element by element
    for (int u = 0; u < UNROLL; ++u)
        for (int e = 0; e < VEC; ++e) {
            const int64_t c = c0 + u * kStride + e;
            if (c >= n) return;
            float acc = 0.f;
            for (int64_t jj = j; jj < r && idx[jj] == row; ++jj) {
                float mm = load_as_f32(M + jj * n + c), vv = load_as_f32(V + jj * n + c);
                acc += rho[jj] * adam_elem<ST>(GC[jj * ldgc + c], mm, vv, p);
                store_from_f32(M + jj * n + c, mm);
                store_from_f32(V + jj * n + c, vv);
            }
            store_from_f32(wrow + c, load_as_f32(wrow + c) + alpha * acc);
        }
}

// The tail of a regular step in one kernel: split-K reduction of the GEMM's partial tiles, Adam
// and the row update.  This is the form for many slices (short, wide products: a 128 x 512
// output with K = 65536 is split 128 times), where the sum over the slices is a long chain of
// loads if one thread walks it.  A workgroup of kManyWaves wavefronts (4, 8 or 16: about eight
// slices each) owns one compressed row j and 256 columns.  Each wavefront adds a contiguous share
// of the slices for all 256 columns (four per lane, up to eight loads in flight), the shares
// meet in LDS, and the first four wavefronts finish one column per lane: the sum of the shares
// in wavefront order times rho (that is G_C, written out only if the caller wants it), Adam,
// and the update.  Runs of equal idx are walked by their first member, as in
// adam_scatter_kernel.  The order of every sum is fixed: deterministic.
// kToU (column form): every compressed row stands for itself (no runs, W is not touched) and
// Adam's output is stored to U.
template <typename WT, typename ST, bool kToU, int kManyWaves>
__global__ __launch_bounds__(kManyWaves * 64) void reduce_adam_scatter_kernel(
    TailSets sets, int slices, int64_t Mp, int64_t Np, int64_t n, AdamParams p_in, float alpha) {
    __shared__ float4 share[kManyWaves][64];
    const TailSet& q = sets.set[blockIdx.z];  // the row set of this workgroup
    const int64_t j = blockIdx.y, r = q.r;
    if (j >= r) return;  // the grid spans the largest set
    const float* __restrict__ part = q.part;
    ST* __restrict__ M = static_cast<ST*>(q.M);
    ST* __restrict__ V = static_cast<ST*>(q.V);
    WT* __restrict__ W = static_cast<WT*>(q.W);
    const int64_t ldw = q.ldw, ldgc = q.ldgc;
    const int32_t* __restrict__ idx = q.idx;
    const float* __restrict__ rho = q.rho;
    float* __restrict__ GC = q.GC;
    float* __restrict__ U = q.U;
    const AdamParams p = resolve(p_in);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int32_t row = kToU ? 0 : idx[j];
    if (!kToU && j > 0 && idx[j - 1] == row) return;  // whole workgroup: no barrier is skipped by part of it
    // summing phase: this lane's four columns; n % 4 == 0, so a live lane owns four whole columns
    const int64_t c4 = static_cast<int64_t>(blockIdx.x) * 256 + lane * 4;
    const bool live4 = c4 < n;
    const int per = (slices + kManyWaves - 1) / kManyWaves;
    const int k0 = w * per < slices ? w * per : slices;
    const int k1 = k0 + per < slices ? k0 + per : slices;
    const int64_t slice_stride = Mp * Np;
    // finishing phase: threads 0..255 take one column each
    const bool finisher = threadIdx.x < 256;
    const int64_t c1 = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const bool live1 = finisher && c1 < n;
    WVec<WT, 1> wv;
    if (!kToU && live1) wv.load_once(W + static_cast<int64_t>(row) * ldw + c1);
    float acc = 0.f;
    for (int64_t jj = j; kToU ? jj == j : (jj < r && idx[jj] == row); ++jj) {
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live4) {
            const float* src = part + (static_cast<int64_t>(k0) * Mp + jj) * Np + c4;
#pragma unroll 8
            for (int k = k0; k < k1; ++k, src += slice_stride) {
                const float4 v = *reinterpret_cast<const float4*>(src);
                s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
            }
        }
        share[w][lane] = s;
        __syncthreads();
        if (live1) {
            const float sc = rho[jj];
            WVec<ST, 1> mv, vv;
            mv.load_once(M + jj * n + c1);
            vv.load_once(V + jj * n + c1);
            float g = 0.f;
#pragma unroll
            for (int o = 0; o < kManyWaves; ++o)
                g += reinterpret_cast<const float*>(&share[o][0])[threadIdx.x];
            g *= sc;
            if (GC) GC[jj * ldgc + c1] = g;
            const float u = adam_elem<ST>(g, mv.x[0], vv.x[0], p);
            if (kToU) U[jj * n + c1] = u;
            else acc += sc * u;
            mv.store_once(M + jj * n + c1);
            vv.store_once(V + jj * n + c1);
        }
        __syncthreads();  // the shares are rewritten for the next member of the run
    }
    if (!kToU && live1) {
        wv.x[0] += alpha * acc;
        wv.store_once(W + static_cast<int64_t>(row) * ldw + c1);
    }
}

// The same for a handful of slices: every thread adds all slices of its own four columns (the
// loads are independent, nothing goes through LDS) and all four wavefronts run Adam, so the
// kernel keeps as many bytes in flight as adam_scatter_kernel does.
template <typename WT, typename ST, bool kToU>
__global__ __launch_bounds__(kThreads) void reduce_adam_scatter_few_kernel(
    TailSets sets, int slices, int64_t Mp, int64_t Np, int64_t n, AdamParams p_in, float alpha) {
    const TailSet& q = sets.set[blockIdx.z];
    const int64_t j = blockIdx.y, r = q.r;
    if (j >= r) return;
    const float* __restrict__ part = q.part;
    ST* __restrict__ M = static_cast<ST*>(q.M);
    ST* __restrict__ V = static_cast<ST*>(q.V);
    WT* __restrict__ W = static_cast<WT*>(q.W);
    const int64_t ldw = q.ldw, ldgc = q.ldgc;
    const int32_t* __restrict__ idx = q.idx;
    const float* __restrict__ rho = q.rho;
    float* __restrict__ GC = q.GC;
    float* __restrict__ U = q.U;
    const AdamParams p = resolve(p_in);
    const int32_t row = kToU ? 0 : idx[j];
    if (!kToU && j > 0 && idx[j - 1] == row) return;
    const int64_t c = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4;
    if (c >= n) return;  // n % 4 == 0: four whole columns or none
    const int64_t slice_stride = Mp * Np;
    WVec<WT, 4> wv;
    if (!kToU) wv.load_once(W + static_cast<int64_t>(row) * ldw + c);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int64_t jj = j; kToU ? jj == j : (jj < r && idx[jj] == row); ++jj) {
        WVec<ST, 4> mv, vv;
        mv.load_once(M + jj * n + c);
        vv.load_once(V + jj * n + c);
        const float* src = part + jj * Np + c;
        F32Vec<4> g;
#pragma unroll
        for (int e = 0; e < 4; ++e) g.x[e] = 0.f;
#pragma unroll 8
        for (int k = 0; k < slices; ++k, src += slice_stride) {
            const float4 v = *reinterpret_cast<const float4*>(src);
            g.x[0] += v.x; g.x[1] += v.y; g.x[2] += v.z; g.x[3] += v.w;
        }
        const float sc = rho[jj];
#pragma unroll
        for (int e = 0; e < 4; ++e) g.x[e] *= sc;
        if (GC) g.store(GC + jj * ldgc + c);
        if (kToU) {
            F32Vec<4> u;
#pragma unroll
            for (int e = 0; e < 4; ++e) u.x[e] = adam_elem<ST>(g.x[e], mv.x[e], vv.x[e], p);
            u.store(U + jj * n + c);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += sc * adam_elem<ST>(g.x[e], mv.x[e], vv.x[e], p);
        }
        mv.store_once(M + jj * n + c);
        vv.store_once(V + jj * n + c);
    }
    if (kToU) return;
#pragma unroll
    for (int e = 0; e < 4; ++e) wv.x[e] += alpha * acc[e];
    wv.store_once(W + static_cast<int64_t>(row) * ldw + c);
}

template <typename GT, int VEC>
__global__ __launch_bounds__(kThreads) void gather_rows_kernel(
    const GT* __restrict__ G, int64_t ldg, const int32_t* __restrict__ idx,
    const float* __restrict__ rho, float* __restrict__ out, int64_t ldo, int64_t n) {
    const int64_t j = blockIdx.y;
    int cnt;
    const int64_t c = thread_col<VEC>(n, cnt);
    if (cnt == 0) return;
    const GT* gp = G + static_cast<int64_t>(idx[j]) * ldg + c;
    float* op = out + j * ldo + c;
    const float s = rho[j];
    if (cnt == VEC) {
        WVec<GT, VEC> gv;
        gv.load(gp);
        F32Vec<VEC> ov;
#pragma unroll
        for (int e = 0; e < VEC; ++e) ov.x[e] = s * gv.x[e];
        ov.store(op);
    } else {
        for (int e = 0; e < cnt; ++e) op[e] = s * load_as_f32(gp + e);
    }
}

// Column form of the update (right-hand projection): W[i, idx[j]] += alpha * sum over the
// run of equal idx of rho * U[., i], with U stored r x mrows (row j contiguous along i).
// A workgroup owns a 64 (j) x 64 (i) tile: U is read with lanes along i (coalesced), turned
// through LDS, and W is touched with lanes along j, so that a wavefront's 64 two- or
// four-byte read-modify-writes fall into the few cache lines that hold 64 consecutive
// selected columns of one row of W.  The first member of a run of equal idx sums the run
// (members beyond this tile are read from global memory), so each W element is written by
// one thread only.
template <typename WT>
__global__ __launch_bounds__(256) void scatter_cols_kernel(
    WT* __restrict__ W, int64_t ldw, int64_t mrows, const int32_t* __restrict__ idx,
    const float* __restrict__ rho, float alpha, const float* __restrict__ U, int64_t r) {
    __shared__ float tile[64][65];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t i0 = static_cast<int64_t>(blockIdx.x) * 64, j0 = static_cast<int64_t>(blockIdx.y) * 64;
    for (int jj = w; jj < 64; jj += 4) {
        const int64_t j = j0 + jj, i = i0 + lane;
        tile[jj][lane] = (j < r && i < mrows) ? rho[j] * U[j * mrows + i] : 0.f;
    }
    __syncthreads();
    const int64_t j = j0 + lane;
    if (j >= r) return;
    const int32_t col = idx[j];
    if (j > 0 && idx[j - 1] == col) return;  // a later member of a run
    int64_t run_end = j + 1;
    while (run_end < r && idx[run_end] == col) ++run_end;
    for (int ii = w; ii < 64; ii += 4) {
        const int64_t i = i0 + ii;
        if (i >= mrows) break;
        float acc = 0.f;
        for (int64_t jn = j; jn < run_end; ++jn)
            acc += jn < j0 + 64 ? tile[jn - j0][ii] : rho[jn] * U[jn * mrows + i];
        WT* wp = W + i * ldw + col;
        store_from_f32(wp, load_as_f32(wp) + alpha * acc);
    }
}

AdamParams make_params(float lr, float b1, float b2, float eps, int64_t t,
                       const float* step_scalars) {
    AdamParams p;
    p.step_scalars = step_scalars;
    if (t < 1) t = 1;  // unused when step_scalars is set
    p.b1 = b1;
    p.one_minus_b1 = 1.0f - b1;
    p.b2 = b2;
    p.one_minus_b2 = 1.0f - b2;
    p.inv_c1 = static_cast<float>(1.0 / (1.0 - pow(static_cast<double>(b1), static_cast<double>(t))));
    p.inv_c2 = static_cast<float>(1.0 / (1.0 - pow(static_cast<double>(b2), static_cast<double>(t))));
    p.lr = lr;
    p.eps = eps;
    return p;
}

dim3 grid_for(int64_t n, int64_t r, int vec) {
    const int64_t per_block = static_cast<int64_t>(kThreads) * vec;
    return dim3(static_cast<unsigned>((n + per_block - 1) / per_block), static_cast<unsigned>(r));
}

bool f32_rows_vectorisable(const void* p, int64_t ld) { return aligned_to(p, 16) && ld % 4 == 0; }
bool w_rows_vectorisable(const void* p, grass_dtype dt, int64_t ld) {
    return aligned_to(p, dt == GRASS_F32 ? 16 : 8) && ld % 4 == 0;
}

}  // namespace

// blockIdx.y carries the row: at most 65535 rows per launch, larger r goes in slices.
constexpr int64_t kMaxGridY = 65535;

template <typename ST>
static grass_status adam_rows_typed(const float* GC, int64_t ldgc, void* Mv, void* Vv,
                                    grass_dtype sdt, int64_t r, int64_t n, const AdamParams& p,
                                    float* U, hipStream_t s) {
    ST* M = static_cast<ST*>(Mv);
    ST* V = static_cast<ST*>(Vv);
    const bool vec = f32_rows_vectorisable(GC, ldgc) && w_rows_vectorisable(M, sdt, n) &&
                     w_rows_vectorisable(V, sdt, n) && f32_rows_vectorisable(U, n);
    for (int64_t j0 = 0; j0 < r; j0 += kMaxGridY) {
        const int64_t rr = r - j0 < kMaxGridY ? r - j0 : kMaxGridY;
        if (vec)
            adam_rows_kernel<ST, 4><<<grid_for(n, rr, 4), kThreads, 0, s>>>(
                GC + j0 * ldgc, ldgc, M + j0 * n, V + j0 * n, U + j0 * n, n, p);
        else
            adam_rows_kernel<ST, 1><<<grid_for(n, rr, 1), kThreads, 0, s>>>(
                GC + j0 * ldgc, ldgc, M + j0 * n, V + j0 * n, U + j0 * n, n, p);
    }
    return launch_status();
}

grass_status launch_adam_rows(const float* GC, int64_t ldgc, void* M, void* V, grass_dtype sdt,
                              int64_t r, int64_t n, float lr, float b1, float b2, float eps,
                              int64_t t, float* U, hipStream_t s) {
    if (r == 0 || n == 0) return GRASS_OK;
    const AdamParams p = make_params(lr, b1, b2, eps, t, nullptr);
    return sdt == GRASS_F32 ? adam_rows_typed<float>(GC, ldgc, M, V, sdt, r, n, p, U, s)
                            : adam_rows_typed<uint16_t>(GC, ldgc, M, V, sdt, r, n, p, U, s);
}

template <typename WT>
static grass_status scatter_typed(void* W, grass_dtype wdt, int64_t n, int64_t ldw,
                                  const int32_t* idx, const float* rho, float alpha,
                                  const float* U, int64_t r, hipStream_t s) {
    // A run of equal idx must not straddle two launches, so r > 65535 is done in one
    // launch per slice only when the slice boundary is not inside a run; the kernel's run
    // walk is bounded by the full r and its "first of the run" test looks at idx[j-1] of
    // the full array, so slices simply pass offsets into the same arrays.
    const bool vec = w_rows_vectorisable(W, wdt, ldw) && f32_rows_vectorisable(U, n);
    if (r > kMaxGridY) return GRASS_ERR_SHAPE;
    if (vec)
        scatter_kernel<WT, 4><<<grid_for(n, r, 4), kThreads, 0, s>>>(
            static_cast<WT*>(W), ldw, idx, rho, alpha, U, n, r);
    else
        scatter_kernel<WT, 1><<<grid_for(n, r, 1), kThreads, 0, s>>>(
            static_cast<WT*>(W), ldw, idx, rho, alpha, U, n, r);
    return launch_status();
}

grass_status launch_scatter(void* W, grass_dtype wdt, int64_t n, int64_t ldw, const int32_t* idx,
                            const float* rho, float alpha, const float* U, int64_t r,
                            hipStream_t s) {
    if (r == 0 || n == 0) return GRASS_OK;
    return wdt == GRASS_F32 ? scatter_typed<float>(W, wdt, n, ldw, idx, rho, alpha, U, r, s)
                            : scatter_typed<uint16_t>(W, wdt, n, ldw, idx, rho, alpha, U, r, s);
}

template <typename WT, typename ST>
static grass_status adam_scatter_typed(const float* GC, int64_t ldgc, void* Mv, void* Vv,
                                       grass_dtype sdt, int64_t r, int64_t n, const AdamParams& p,
                                       void* W, grass_dtype wdt, int64_t ldw, const int32_t* idx,
                                       const float* rho, float alpha, hipStream_t s) {
    ST* M = static_cast<ST*>(Mv);
    ST* V = static_cast<ST*>(Vv);
    const bool vec = f32_rows_vectorisable(GC, ldgc) && w_rows_vectorisable(M, sdt, n) &&
                     w_rows_vectorisable(V, sdt, n) && w_rows_vectorisable(W, wdt, ldw);
    if (r > kMaxGridY) return GRASS_ERR_SHAPE;
    // One vector per thread.  Two or four per thread are a few percent faster when the state is
    // warm in the last-level cache and slower inside a real step, where it comes from HBM.
    const int unroll = 1;
    if (vec && unroll == 4)
        adam_scatter_kernel<WT, ST, 4, 4><<<grid_for(n, r, 16), kThreads, 0, s>>>(
            GC, ldgc, M, V, n, r, p, static_cast<WT*>(W), ldw, idx, rho, alpha);
    else if (vec && unroll == 2)
        adam_scatter_kernel<WT, ST, 4, 2><<<grid_for(n, r, 8), kThreads, 0, s>>>(
            GC, ldgc, M, V, n, r, p, static_cast<WT*>(W), ldw, idx, rho, alpha);
    else if (vec)
        adam_scatter_kernel<WT, ST, 4, 1><<<grid_for(n, r, 4), kThreads, 0, s>>>(
            GC, ldgc, M, V, n, r, p, static_cast<WT*>(W), ldw, idx, rho, alpha);
    else
        adam_scatter_kernel<WT, ST, 1, 1><<<grid_for(n, r, 1), kThreads, 0, s>>>(
            GC, ldgc, M, V, n, r, p, static_cast<WT*>(W), ldw, idx, rho, alpha);
    return launch_status();
}

grass_status launch_adam_scatter(const float* GC, int64_t ldgc, void* M, void* V, grass_dtype sdt,
                                 int64_t r, int64_t n, float lr, float b1, float b2, float eps,
                                 int64_t t, void* W, grass_dtype wdt, int64_t ldw,
                                 const int32_t* idx, const float* rho, float alpha, hipStream_t s,
                                 const float* step_scalars) {
    if (r == 0 || n == 0) return GRASS_OK;
    const AdamParams p = make_params(lr, b1, b2, eps, t, step_scalars);
    if (wdt == GRASS_F32)
        return sdt == GRASS_F32
                   ? adam_scatter_typed<float, float>(GC, ldgc, M, V, sdt, r, n, p, W, wdt, ldw, idx, rho, alpha, s)
                   : adam_scatter_typed<float, uint16_t>(GC, ldgc, M, V, sdt, r, n, p, W, wdt, ldw, idx, rho, alpha, s);
    return sdt == GRASS_F32
               ? adam_scatter_typed<uint16_t, float>(GC, ldgc, M, V, sdt, r, n, p, W, wdt, ldw, idx, rho, alpha, s)
               : adam_scatter_typed<uint16_t, uint16_t>(GC, ldgc, M, V, sdt, r, n, p, W, wdt, ldw, idx, rho, alpha, s);
}

grass_status launch_scatter_cols(void* W, grass_dtype wdt, int64_t mrows, int64_t ldw,
                                 const int32_t* idx, const float* rho, float alpha, const float* U,
                                 int64_t r, hipStream_t s) {
    if (r == 0 || mrows == 0) return GRASS_OK;
    const dim3 grid(static_cast<unsigned>((mrows + 63) / 64), static_cast<unsigned>((r + 63) / 64));
    if (wdt == GRASS_F32)
        scatter_cols_kernel<float><<<grid, 256, 0, s>>>(static_cast<float*>(W), ldw, mrows, idx, rho,
                                                        alpha, U, r);
    else
        scatter_cols_kernel<uint16_t><<<grid, 256, 0, s>>>(static_cast<uint16_t*>(W), ldw, mrows,
                                                           idx, rho, alpha, U, r);
    return launch_status();
}

template <typename GT>
static grass_status gather_typed(const void* G, grass_dtype gdt, int64_t n, int64_t ldg,
                                 const int32_t* idx, const float* rho, int64_t r, float* out,
                                 int64_t ldo, hipStream_t s) {
    const bool vec = w_rows_vectorisable(G, gdt, ldg) && f32_rows_vectorisable(out, ldo);
    if (r > kMaxGridY) return GRASS_ERR_SHAPE;
    if (vec)
        gather_rows_kernel<GT, 4><<<grid_for(n, r, 4), kThreads, 0, s>>>(
            static_cast<const GT*>(G), ldg, idx, rho, out, ldo, n);
    else
        gather_rows_kernel<GT, 1><<<grid_for(n, r, 1), kThreads, 0, s>>>(
            static_cast<const GT*>(G), ldg, idx, rho, out, ldo, n);
    return launch_status();
}

grass_status launch_gather_rows(const void* G, grass_dtype gdt, int64_t n, int64_t ldg,
                                const int32_t* idx, const float* rho, int64_t r, float* out,
                                int64_t ldo, hipStream_t s) {
    if (r == 0 || n == 0) return GRASS_OK;
    return gdt == GRASS_F32 ? gather_typed<float>(G, gdt, n, ldg, idx, rho, r, out, ldo, s)
                            : gather_typed<uint16_t>(G, gdt, n, ldg, idx, rho, r, out, ldo, s);
}

bool reduce_adam_scatter_ok(const StepTail& t, int64_t n, const float* GC, int64_t ldgc) {
    return n % 4 == 0 && w_rows_vectorisable(t.M, t.sdt, n) && w_rows_vectorisable(t.V, t.sdt, n) &&
           (t.U ? f32_rows_vectorisable(t.U, n) : w_rows_vectorisable(t.W, t.wdt, t.ldw)) &&
           (!GC || f32_rows_vectorisable(GC, ldgc));
}

template <typename WT, typename ST, bool kToU = false>
static void reduce_adam_scatter_typed(const TailSets& sets, int count, int64_t rmax, int slices,
                                      int64_t Mp, int64_t Np, int64_t n, const AdamParams& p,
                                      float alpha, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    if (slices <= 8) {
        dim3 grid = grid_for(n, rmax, 4);
        grid.z = static_cast<unsigned>(count);
        launch_stamped(reduce_adam_scatter_few_kernel<WT, ST, kToU>, grid, dim3(kThreads), 0, s, e0, e1,
                       sets, slices, Mp, Np, n, p, alpha);
        return;
    }
    const dim3 grid(static_cast<unsigned>((n + 255) / 256), static_cast<unsigned>(rmax),
                    static_cast<unsigned>(count));
    if (slices <= 32)
        launch_stamped(reduce_adam_scatter_kernel<WT, ST, kToU, 4>, grid, dim3(4 * 64), 0, s, e0, e1,
                       sets, slices, Mp, Np, n, p, alpha);
    else if (slices <= 64)
        launch_stamped(reduce_adam_scatter_kernel<WT, ST, kToU, 8>, grid, dim3(8 * 64), 0, s, e0, e1,
                       sets, slices, Mp, Np, n, p, alpha);
    else
        launch_stamped(reduce_adam_scatter_kernel<WT, ST, kToU, 16>, grid, dim3(16 * 64), 0, s, e0, e1,
                       sets, slices, Mp, Np, n, p, alpha);
}

grass_status launch_reduce_adam_scatter(const TailSets& sets, int count, int slices, int64_t Mp,
                                        int64_t Np, int64_t n, const StepTail& t, hipStream_t s,
                                        hipEvent_t e0, hipEvent_t e1) {
    int64_t rmax = 0;
    for (int i = 0; i < count; ++i) rmax = sets.set[i].r > rmax ? sets.set[i].r : rmax;
    if (count < 1 || rmax == 0 || n == 0) return GRASS_OK;
    if (rmax > kMaxGridY || count > GRASS_MAX_GROUP) return GRASS_ERR_SHAPE;
    const AdamParams p = make_params(t.lr, t.beta1, t.beta2, t.eps, t.t, t.step_scalars);
    const bool wf = t.wdt == GRASS_F32, sf = t.sdt == GRASS_F32;
    if (sets.set[0].U) {  // column form: W is not touched here
        for (int i = 0; i < count; ++i)
            if (!sets.set[i].U) return GRASS_ERR_SHAPE;  // one form per launch
        if (sf) reduce_adam_scatter_typed<uint16_t, float, true>(sets, count, rmax, slices, Mp, Np, n, p, t.alpha, s, e0, e1);
        else reduce_adam_scatter_typed<uint16_t, uint16_t, true>(sets, count, rmax, slices, Mp, Np, n, p, t.alpha, s, e0, e1);
        return launch_status();
    }
    if (wf && sf) reduce_adam_scatter_typed<float, float>(sets, count, rmax, slices, Mp, Np, n, p, t.alpha, s, e0, e1);
    else if (wf) reduce_adam_scatter_typed<float, uint16_t>(sets, count, rmax, slices, Mp, Np, n, p, t.alpha, s, e0, e1);
    else if (sf) reduce_adam_scatter_typed<uint16_t, float>(sets, count, rmax, slices, Mp, Np, n, p, t.alpha, s, e0, e1);
    else reduce_adam_scatter_typed<uint16_t, uint16_t>(sets, count, rmax, slices, Mp, Np, n, p, t.alpha, s, e0, e1);
    return launch_status();
}

void adam_step_scalars(float lr, float b1, float b2, int64_t t, float out[3]) {
    const AdamParams p = make_params(lr, b1, b2, 0.f, t, nullptr);
    out[0] = p.lr;
    out[1] = p.inv_c1;
    out[2] = p.inv_c2;
}

}  // namespace grass
