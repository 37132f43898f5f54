// C entry points declared in include/grass.h: host-side argument validation, then the
// kernel launchers.  Validation touches no device memory and makes no HIP call, so a call
// that fails validation has no side effect (and can be exercised on a machine without a
// GPU).
#include <atomic>

#include "common.hpp"

using namespace grass;

namespace {

constexpr int kNumTestOptions = 6;
std::atomic<int> g_test_options[kNumTestOptions];  // zero-initialised: the library decides

constexpr int64_t kMaxGridRows = 65535;  // rows are carried in blockIdx.y

// A pointer may be NULL only when the array it names has no elements.
bool present(const void* p, int64_t elems) { return p != nullptr || elems <= 0; }
// Every size of the interface is below 2^31, so that products of two of them fit 64 bits.
bool small(int64_t v) { return v < (int64_t{1} << 31); }
bool dtype_ok(grass_dtype d) { return d == GRASS_F32 || d == GRASS_BF16; }
bool layout_ok(grass_dy_layout l) { return l == GRASS_DY_TxM || l == GRASS_DY_MxT; }
hipStream_t as_stream(void* s) { return static_cast<hipStream_t>(s); }

grass_status check_products(const void* dY, grass_dy_layout layout, int64_t ldy, const void* X,
                            int64_t ldx, grass_dtype dt, int64_t T, int64_t m, int64_t n) {
    if (T < 0 || m < 0 || n < 0 || ldx < n) return GRASS_ERR_SHAPE;
    // sizes first: the products below then fit 64 bits
    if (!small(m) || !small(n) || !small(T)) return GRASS_ERR_SHAPE;
    if (!present(dY, T * m) || !present(X, T * n)) return GRASS_ERR_NULL;
    if (!dtype_ok(dt) || !layout_ok(layout)) return GRASS_ERR_DTYPE;
    if (ldy < (layout == GRASS_DY_TxM ? m : T)) return GRASS_ERR_SHAPE;
    return GRASS_OK;
}

grass_status check_adam(const float* GC, int64_t ldgc, const void* M, const void* V,
                        grass_dtype sdt, int64_t r, int64_t n, float beta1, float beta2, int64_t t) {
    if (r < 0 || n < 0 || ldgc < n || t < 1 || !small(r) || !small(n)) return GRASS_ERR_SHAPE;
    if (!present(GC, r * n) || !present(M, r * n) || !present(V, r * n)) return GRASS_ERR_NULL;
    if (!dtype_ok(sdt)) return GRASS_ERR_DTYPE;
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return GRASS_ERR_SHAPE;
    return GRASS_OK;
}

grass_status check_rows_of_w(const void* W, grass_dtype wdt, int64_t m, int64_t n, int64_t ldw,
                             const int32_t* idx, const float* rho, int64_t r) {
    if (m < 0 || n < 0 || r < 0 || ldw < n || r > kMaxGridRows || !small(m) || !small(n))
        return GRASS_ERR_SHAPE;
    if (!present(W, m * n) || !present(idx, r) || !present(rho, r)) return GRASS_ERR_NULL;
    if (!dtype_ok(wdt)) return GRASS_ERR_DTYPE;
    if (r > 0 && m == 0) return GRASS_ERR_SHAPE;
    return GRASS_OK;
}

}  // namespace

namespace grass {
int test_option(grass_test_option which) {
    return g_test_options[which].load(std::memory_order_relaxed);
}
}  // namespace grass

extern "C" {

const char* grass_status_string(grass_status s) {
    switch (s) {
        case GRASS_OK: return "ok";
        case GRASS_ERR_NULL: return "null pointer";
        case GRASS_ERR_SHAPE: return "bad shape or size";
        case GRASS_ERR_DTYPE: return "unsupported dtype or option";
        case GRASS_ERR_WORKSPACE: return "workspace missing or too small";
        case GRASS_ERR_NONFINITE: return "row statistics are not finite and non-negative";
        case GRASS_ERR_DEVICE: return "HIP launch failed";
    }
    return "unknown status";
}

grass_status grass_row_stats(const void* G, grass_dtype dt, int64_t m, int64_t n, int64_t ldg,
                             float* sumsq, void* stream) {
    if (m < 0 || n < 0 || ldg < n || !small(m) || !small(n)) return GRASS_ERR_SHAPE;
    if (!present(G, m * n) || !present(sumsq, m)) return GRASS_ERR_NULL;
    if (!dtype_ok(dt)) return GRASS_ERR_DTYPE;
    return launch_row_stats(G, dt, m, n, ldg, sumsq, as_stream(stream));
}

size_t grass_select_workspace(int64_t m, int64_t r, grass_method method, int replacement) {
    return select_workspace_bytes(m, r, method, replacement);
}

static grass_status check_select(const float* sumsq, int64_t m, int64_t r, grass_method method,
                                 int replacement, grass_scale scale, const int32_t* idx,
                                 const float* rho) {
    if (m < 0 || r < 0) return GRASS_ERR_SHAPE;
    if (!present(sumsq, m) || !present(idx, r) || !present(rho, r)) return GRASS_ERR_NULL;
    if (method < GRASS_SEL_TOPR || method > GRASS_SEL_MULTI_NORM2) return GRASS_ERR_DTYPE;
    if (scale < GRASS_SCALE_PAPER || scale > GRASS_SCALE_INV_SQRT_RQ) return GRASS_ERR_DTYPE;
    if (method == GRASS_SEL_TOPR && scale == GRASS_SCALE_INV_SQRT_RQ) return GRASS_ERR_DTYPE;
    if (!small(m) || !small(r)) return GRASS_ERR_SHAPE;
    const bool with_repl = method != GRASS_SEL_TOPR && replacement;
    if (!with_repl && r > m) return GRASS_ERR_SHAPE;
    if (r > 0 && m == 0) return GRASS_ERR_SHAPE;
    return GRASS_OK;
}

grass_status grass_select_rows(const float* sumsq, int64_t m, int64_t r, grass_method method,
                               int replacement, grass_scale scale, uint64_t seed,
                               uint64_t refresh_id, int32_t* idx, float* rho, void* ws,
                               size_t ws_bytes, void* stream) {
    const grass_status st = check_select(sumsq, m, r, method, replacement, scale, idx, rho);
    if (st != GRASS_OK) return st;
    if (!ws || ws_bytes < select_workspace_bytes(m, r, method, replacement))
        return GRASS_ERR_WORKSPACE;
    return launch_select(sumsq, m, r, method, replacement, scale, seed, refresh_id, idx, rho, ws,
                         as_stream(stream));
}

size_t grass_select_static_capacity(void) { return select_static_scratch_bytes(); }

grass_status grass_select_rows_static(const float* sumsq, int64_t m, int64_t r,
                                      grass_method method, int replacement, grass_scale scale,
                                      uint64_t seed, uint64_t refresh_id, int32_t* idx, float* rho,
                                      int32_t* status, void* stream) {
    const grass_status st = check_select(sumsq, m, r, method, replacement, scale, idx, rho);
    if (st != GRASS_OK) return st;
    if (select_workspace_bytes(m, r, method, replacement) > select_static_scratch_bytes())
        return GRASS_ERR_WORKSPACE;  // beyond the built-in scratch: use grass_select_rows
    return launch_select_static(sumsq, m, r, method, replacement, scale, seed, refresh_id, idx, rho,
                                status, as_stream(stream));
}

size_t grass_cgrad_workspace(int64_t T, int64_t m, int64_t n, int64_t r, grass_dtype dt,
                             grass_dy_layout layout) {
    (void)m;
    if (T < 0 || n < 0 || r < 0 || !small(T) || !small(n) || !small(r)) return 0;
    return gemm_workspace_bytes(T, r, n, dt, layout, true);
}

grass_status grass_cgrad_plan(int64_t T, int64_t m, int64_t n, int64_t rows, int count,
                              grass_dtype dt, grass_dy_layout layout, int* tile, int* k_slices) {
    if (!tile || !k_slices) return GRASS_ERR_NULL;
    if (T < 0 || m < 0 || n < 0 || rows < 0 || !small(T) || !small(m) || !small(n) ||
        rows > kMaxGridRows || count < 1 || count > GRASS_MAX_GROUP)
        return GRASS_ERR_SHAPE;
    if (!dtype_ok(dt) || !layout_ok(layout)) return GRASS_ERR_DTYPE;
    gemm_plan_summary(T, m, rows, count, n, dt, layout, tile, k_slices);
    return GRASS_OK;
}

grass_status grass_compressed_grad(const void* dY, grass_dy_layout layout, int64_t ldy,
                                   const void* X, int64_t ldx, grass_dtype dt, int64_t T,
                                   int64_t m, int64_t n, int64_t r, const int32_t* idx,
                                   const float* rho, float* GC, int64_t ldgc, void* ws,
                                   size_t ws_bytes, void* stream) {
    return grass_compressed_grad_timed(dY, layout, ldy, X, ldx, dt, T, m, n, r, idx, rho, GC, ldgc,
                                       ws, ws_bytes, stream, nullptr, nullptr);
}

grass_status grass_compressed_grad_timed(const void* dY, grass_dy_layout layout, int64_t ldy,
                                         const void* X, int64_t ldx, grass_dtype dt, int64_t T,
                                         int64_t m, int64_t n, int64_t r, const int32_t* idx,
                                         const float* rho, float* GC, int64_t ldgc, void* ws,
                                         size_t ws_bytes, void* stream, void* ev_gemm_start,
                                         void* ev_gemm_stop) {
    const grass_status st = check_products(dY, layout, ldy, X, ldx, dt, T, m, n);
    if (st != GRASS_OK) return st;
    if (r < 0 || r > kMaxGridRows || ldgc < n || (r > 0 && m == 0)) return GRASS_ERR_SHAPE;
    if (!present(idx, r) || !present(rho, r) || !present(GC, r * n)) return GRASS_ERR_NULL;
    const size_t need = gemm_workspace_bytes(T, r, n, dt, layout, true);
    if (need > 0 && (!ws || ws_bytes < need)) return GRASS_ERR_WORKSPACE;
    return launch_tn_gemm(dY, layout, ldy, X, ldx, dt, T, r, n, idx, rho, GC, GRASS_F32, ldgc, ws,
                          as_stream(stream), m, static_cast<hipEvent_t>(ev_gemm_start),
                          static_cast<hipEvent_t>(ev_gemm_stop));
}

size_t grass_cgrad_group_workspace(int64_t T, int64_t n, int count, const int64_t* r,
                                   grass_dtype dt, grass_dy_layout layout) {
    if (T < 0 || n < 0 || !small(T) || !small(n) || count < 1 || count > GRASS_MAX_GROUP || !r)
        return 0;
    for (int i = 0; i < count; ++i)
        if (r[i] < 0 || r[i] > kMaxGridRows) return 0;
    return gemm_group_workspace_bytes(T, r, count, n, dt, layout);
}

grass_status grass_compressed_grad_group(int count, const void* const* dY, grass_dy_layout layout,
                                         const int64_t* ldy, const void* X, int64_t ldx,
                                         grass_dtype dt, int64_t T, const int64_t* m, int64_t n,
                                         const int64_t* r, const int32_t* const* idx,
                                         const float* const* rho, float* const* GC,
                                         const int64_t* ldgc, void* ws, size_t ws_bytes,
                                         void* stream) {
    if (count < 1 || count > GRASS_MAX_GROUP) return GRASS_ERR_SHAPE;
    if (!dY || !ldy || !m || !r || !idx || !rho || !GC || !ldgc) return GRASS_ERR_NULL;
    GemmSegment seg[GRASS_MAX_GROUP];
    for (int i = 0; i < count; ++i) {
        const grass_status st = check_products(dY[i], layout, ldy[i], X, ldx, dt, T, m[i], n);
        if (st != GRASS_OK) return st;
        if (r[i] < 0 || r[i] > kMaxGridRows || ldgc[i] < n || (r[i] > 0 && m[i] == 0))
            return GRASS_ERR_SHAPE;
        if (!present(idx[i], r[i]) || !present(rho[i], r[i]) || !present(GC[i], r[i] * n))
            return GRASS_ERR_NULL;
        seg[i] = GemmSegment{dY[i], ldy[i], idx[i], rho[i], GC[i], ldgc[i], r[i], m[i]};
    }
    const size_t need = gemm_group_workspace_bytes(T, r, count, n, dt, layout);
    if (need > 0 && (!ws || ws_bytes < need)) return GRASS_ERR_WORKSPACE;
    return launch_tn_gemm_segments(seg, count, layout, X, ldx, dt, T, n, GRASS_F32, ws,
                                   as_stream(stream));
}

grass_status grass_adam_rows(const float* GC, int64_t ldgc, float* M, float* V, int64_t r,
                             int64_t n, float lr, float beta1, float beta2, float eps, int64_t t,
                             float* U, void* stream) {
    return grass_adam_rows_state(GC, ldgc, M, V, GRASS_F32, r, n, lr, beta1, beta2, eps, t, U,
                                 stream);
}

grass_status grass_adam_rows_state(const float* GC, int64_t ldgc, void* M, void* V,
                                   grass_dtype sdt, int64_t r, int64_t n, float lr, float beta1,
                                   float beta2, float eps, int64_t t, float* U, void* stream) {
    const grass_status st = check_adam(GC, ldgc, M, V, sdt, r, n, beta1, beta2, t);
    if (st != GRASS_OK) return st;
    if (!present(U, r * n)) return GRASS_ERR_NULL;
    return launch_adam_rows(GC, ldgc, M, V, sdt, r, n, lr, beta1, beta2, eps, t, U,
                            as_stream(stream));
}

grass_status grass_scatter_update(void* W, grass_dtype wdt, int64_t m, int64_t n, int64_t ldw,
                                  const int32_t* idx, const float* rho, float alpha,
                                  const float* U, int64_t r, void* stream) {
    const grass_status st = check_rows_of_w(W, wdt, m, n, ldw, idx, rho, r);
    if (st != GRASS_OK) return st;
    if (!present(U, r * n)) return GRASS_ERR_NULL;
    return launch_scatter(W, wdt, n, ldw, idx, rho, alpha, U, r, as_stream(stream));
}

grass_status grass_scatter_update_cols(void* W, grass_dtype wdt, int64_t m, int64_t n, int64_t ldw,
                                       const int32_t* idx, const float* rho, float alpha,
                                       const float* U, int64_t r, void* stream) {
    if (m < 0 || n < 0 || r < 0 || ldw < n || !small(m) || !small(n) || !small(r) ||
        (r + 63) / 64 > kMaxGridRows || (r > 0 && n == 0))
        return GRASS_ERR_SHAPE;
    if (!present(W, m * n) || !present(idx, r) || !present(rho, r) || !present(U, r * m))
        return GRASS_ERR_NULL;
    if (!dtype_ok(wdt)) return GRASS_ERR_DTYPE;
    return launch_scatter_cols(W, wdt, m, ldw, idx, rho, alpha, U, r, as_stream(stream));
}

grass_status grass_adam_scatter(const float* GC, int64_t ldgc, float* M, float* V, int64_t r,
                                int64_t n, float lr, float beta1, float beta2, float eps,
                                int64_t t, void* W, grass_dtype wdt, int64_t m, int64_t ldw,
                                const int32_t* idx, const float* rho, float alpha, void* stream) {
    return grass_adam_scatter_state(GC, ldgc, M, V, GRASS_F32, r, n, lr, beta1, beta2, eps, t, W,
                                    wdt, m, ldw, idx, rho, alpha, stream);
}

grass_status grass_adam_scatter_state(const float* GC, int64_t ldgc, void* M, void* V,
                                      grass_dtype sdt, int64_t r, int64_t n, float lr, float beta1,
                                      float beta2, float eps, int64_t t, void* W, grass_dtype wdt,
                                      int64_t m, int64_t ldw, const int32_t* idx, const float* rho,
                                      float alpha, void* stream) {
    grass_status st = check_adam(GC, ldgc, M, V, sdt, r, n, beta1, beta2, t);
    if (st != GRASS_OK) return st;
    st = check_rows_of_w(W, wdt, m, n, ldw, idx, rho, r);
    if (st != GRASS_OK) return st;
    return launch_adam_scatter(GC, ldgc, M, V, sdt, r, n, lr, beta1, beta2, eps, t, W, wdt, ldw,
                               idx, rho, alpha, as_stream(stream));
}

static size_t scratch_gc_bytes(int64_t r, int64_t n) {
    return (static_cast<size_t>(r) * n * 4 + 255) / 256 * 256;
}

size_t grass_step_group_workspace(int64_t T, int64_t n, int count, const int64_t* r,
                                  grass_dtype dt, grass_dy_layout layout) {
    if (T < 0 || n < 0 || !small(T) || !small(n) || count < 1 || count > GRASS_MAX_GROUP || !r)
        return 0;
    size_t extra = 256;  // a G_C for every layer that does not name one (the two-kernel route)
    for (int i = 0; i < count; ++i) {
        if (r[i] < 0 || r[i] > kMaxGridRows) return 0;
        extra += scratch_gc_bytes(r[i], n);
    }
    return gemm_group_workspace_bytes(T, r, count, n, dt, layout) + extra;
}

grass_status grass_step_group(int count, const grass_step_layer* layers, grass_dy_layout layout,
                              const void* X, int64_t ldx, grass_dtype dt, int64_t T, int64_t n,
                              grass_dtype sdt, grass_dtype wdt, float lr, float beta1, float beta2,
                              float eps, int64_t t, const float* step_scalars, float alpha,
                              void* ws, size_t ws_bytes, void* stream, void* ev_gemm_start,
                              void* ev_gemm_stop) {
    return grass_step_group_timed(count, layers, layout, X, ldx, dt, T, n, sdt, wdt, lr, beta1, beta2,
                                  eps, t, step_scalars, alpha, ws, ws_bytes, stream, ev_gemm_start,
                                  ev_gemm_stop, nullptr, nullptr);
}

grass_status grass_step_group_timed(int count, const grass_step_layer* layers,
                                    grass_dy_layout layout, const void* X, int64_t ldx,
                                    grass_dtype dt, int64_t T, int64_t n, grass_dtype sdt,
                                    grass_dtype wdt, float lr, float beta1, float beta2, float eps,
                                    int64_t t, const float* step_scalars, float alpha, void* ws,
                                    size_t ws_bytes, void* stream, void* ev_gemm_start,
                                    void* ev_gemm_stop, void* ev_tail_start, void* ev_tail_stop) {
    if (count < 1 || count > GRASS_MAX_GROUP) return GRASS_ERR_SHAPE;
    if (!layers) return GRASS_ERR_NULL;
    GemmSegment seg[GRASS_MAX_GROUP];
    StepTail tail[GRASS_MAX_GROUP];
    int64_t rows[GRASS_MAX_GROUP];
    for (int i = 0; i < count; ++i) {
        const grass_step_layer& L = layers[i];
        grass_status st = check_products(L.dY, layout, L.ldy, X, ldx, dt, T, L.m, n);
        if (st != GRASS_OK) return st;
        if (L.r < 0 || L.r > kMaxGridRows || (L.GC && L.ldgc < n)) return GRASS_ERR_SHAPE;
        // any non-null stand-in passes the presence test of G_C when the layer does not name one
        st = check_adam(L.GC ? L.GC : reinterpret_cast<const float*>(L.M), L.GC ? L.ldgc : n, L.M,
                        L.V, sdt, L.r, n, beta1, beta2, step_scalars ? 1 : t);
        if (st != GRASS_OK) return st;
        st = check_rows_of_w(L.W, wdt, L.m, n, L.ldw, L.idx, L.rho, L.r);
        if (st != GRASS_OK) return st;
        rows[i] = L.r;
    }
    const size_t gemm_bytes = gemm_group_workspace_bytes(T, rows, count, n, dt, layout);
    size_t need = gemm_bytes + 256;
    for (int i = 0; i < count; ++i) need += scratch_gc_bytes(rows[i], n);
    if (!ws || ws_bytes < need) return GRASS_ERR_WORKSPACE;
    char* scratch = static_cast<char*>(ws) + gemm_bytes;
    scratch += (256 - reinterpret_cast<uintptr_t>(scratch) % 256) % 256;
    for (int i = 0; i < count; ++i) {
        const grass_step_layer& L = layers[i];
        tail[i] = StepTail{L.M, L.V, sdt, lr, beta1, beta2, eps, step_scalars ? 1 : t,
                           step_scalars, L.W, wdt, L.ldw, alpha};
        seg[i] = GemmSegment{L.dY, L.ldy, L.idx, L.rho, L.GC ? static_cast<void*>(L.GC) : scratch,
                             L.GC ? L.ldgc : n, L.r, L.m, &tail[i], L.GC != nullptr};
        if (!L.GC) scratch += scratch_gc_bytes(L.r, n);
    }
    return launch_tn_gemm_segments(seg, count, layout, X, ldx, dt, T, n, GRASS_F32, ws,
                                   as_stream(stream), static_cast<hipEvent_t>(ev_gemm_start),
                                   static_cast<hipEvent_t>(ev_gemm_stop),
                                   static_cast<hipEvent_t>(ev_tail_start),
                                   static_cast<hipEvent_t>(ev_tail_stop));
}

size_t grass_step_cols_workspace(int64_t T, int64_t m, int64_t n, int64_t r, grass_dtype dt) {
    if (T < 0 || m < 0 || n < 0 || r < 0 || !small(T) || !small(m) || !small(n) || r > kMaxGridRows)
        return 0;
    // the transposed problem: r selected rows of an n x m gradient, plus room for an unnamed G_C
    return gemm_workspace_bytes(T, r, m, dt, GRASS_DY_TxM, true) + 256 + scratch_gc_bytes(r, m);
}

grass_status grass_step_cols(const void* dY, int64_t ldy, const void* X, int64_t ldx,
                             grass_dtype dt, int64_t T, int64_t m, int64_t n, int64_t r,
                             const int32_t* idx, const float* rho, float* GC, int64_t ldgc,
                             void* M, void* V, grass_dtype sdt, float* U, void* W,
                             grass_dtype wdt, int64_t ldw, float lr, float beta1, float beta2,
                             float eps, int64_t t, float alpha, void* ws, size_t ws_bytes,
                             void* stream, void* ev_gemm_start, void* ev_gemm_stop) {
    grass_status st = check_products(dY, GRASS_DY_TxM, ldy, X, ldx, dt, T, m, n);
    if (st != GRASS_OK) return st;
    if (r < 0 || r > kMaxGridRows || (GC && ldgc < m) || (r > 0 && n == 0)) return GRASS_ERR_SHAPE;
    st = check_adam(GC ? GC : reinterpret_cast<const float*>(M), GC ? ldgc : m, M, V, sdt, r, m,
                    beta1, beta2, t);
    if (st != GRASS_OK) return st;
    if (ldw < n) return GRASS_ERR_SHAPE;
    if (!present(W, m * n) || !present(idx, r) || !present(rho, r) || !present(U, r * m))
        return GRASS_ERR_NULL;
    if (!dtype_ok(wdt)) return GRASS_ERR_DTYPE;
    if (!aligned_to(U, 16)) return GRASS_ERR_SHAPE;
    const size_t gemm_bytes = gemm_workspace_bytes(T, r, m, dt, GRASS_DY_TxM, true);
    if (!ws || ws_bytes < gemm_bytes + 256 + scratch_gc_bytes(r, m)) return GRASS_ERR_WORKSPACE;
    char* scratch = static_cast<char*>(ws) + gemm_bytes;
    scratch += (256 - reinterpret_cast<uintptr_t>(scratch) % 256) % 256;
    StepTail tail{M, V, sdt, lr, beta1, beta2, eps, t, nullptr, W, wdt, ldw, alpha};
    tail.U = U;
    tail.w_rows = m;
    // rows of the transposed problem: the r selected columns of X are gathered, dY is the
    // dense operand
    const GemmSegment seg{X, ldx, idx, rho, GC ? static_cast<void*>(GC) : scratch, GC ? ldgc : m,
                          r, n, &tail, GC != nullptr};
    return launch_tn_gemm_segments(&seg, 1, GRASS_DY_TxM, dY, ldy, dt, T, m, GRASS_F32, ws,
                                   as_stream(stream), static_cast<hipEvent_t>(ev_gemm_start),
                                   static_cast<hipEvent_t>(ev_gemm_stop));
}

grass_status grass_adam_step_scalars(float lr, float beta1, float beta2, int64_t t,
                                     float* scalars) {
    if (!scalars) return GRASS_ERR_NULL;
    if (t < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f))
        return GRASS_ERR_SHAPE;
    adam_step_scalars(lr, beta1, beta2, t, scalars);
    return GRASS_OK;
}

grass_status grass_adam_scatter_replayable(const float* GC, int64_t ldgc, void* M, void* V,
                                           grass_dtype sdt, int64_t r, int64_t n, float beta1,
                                           float beta2, float eps, const float* step_scalars,
                                           void* W, grass_dtype wdt, int64_t m, int64_t ldw,
                                           const int32_t* idx, const float* rho, float alpha,
                                           void* stream) {
    if (!step_scalars) return GRASS_ERR_NULL;
    grass_status st = check_adam(GC, ldgc, M, V, sdt, r, n, beta1, beta2, 1);
    if (st != GRASS_OK) return st;
    st = check_rows_of_w(W, wdt, m, n, ldw, idx, rho, r);
    if (st != GRASS_OK) return st;
    return launch_adam_scatter(GC, ldgc, M, V, sdt, r, n, 0.f, beta1, beta2, eps, 1, W, wdt, ldw,
                               idx, rho, alpha, as_stream(stream), step_scalars);
}

size_t grass_dense_workspace(int64_t T, int64_t m, int64_t n, grass_dtype dt,
                             grass_dy_layout layout) {
    if (T < 0 || m < 0 || n < 0 || !small(T) || !small(m) || !small(n)) return 0;
    return gemm_workspace_bytes(T, m, n, dt, layout, false);
}

grass_status grass_dense_grad(const void* dY, grass_dy_layout layout, int64_t ldy, const void* X,
                              int64_t ldx, grass_dtype dt, int64_t T, int64_t m, int64_t n,
                              void* G, grass_dtype gdt, int64_t ldg, void* ws, size_t ws_bytes,
                              void* stream) {
    const grass_status st = check_products(dY, layout, ldy, X, ldx, dt, T, m, n);
    if (st != GRASS_OK) return st;
    if (ldg < n || m > kMaxGridRows) return GRASS_ERR_SHAPE;
    if (!present(G, m * n)) return GRASS_ERR_NULL;
    if (!dtype_ok(gdt)) return GRASS_ERR_DTYPE;
    const size_t need = gemm_workspace_bytes(T, m, n, dt, layout, false);
    if (need > 0 && (!ws || ws_bytes < need)) return GRASS_ERR_WORKSPACE;
    return launch_tn_gemm(dY, layout, ldy, X, ldx, dt, T, m, n, nullptr, nullptr, G, gdt, ldg, ws,
                          as_stream(stream), m);
}

size_t grass_grad_row_stats_workspace(int64_t T, int64_t m, int64_t n, grass_dtype dt,
                                      grass_dy_layout layout, int64_t ldy, int64_t ldx) {
    if (T < 0 || m < 0 || n < 0 || !small(T) || !small(m) || !small(n)) return 0;
    return grad_row_stats_workspace_bytes(T, m, n, dt, layout, ldy, ldx);
}

grass_status grass_grad_row_stats(const void* dY, grass_dy_layout layout, int64_t ldy,
                                  const void* X, int64_t ldx, grass_dtype dt, int64_t T, int64_t m,
                                  int64_t n, float* sumsq, void* ws, size_t ws_bytes,
                                  void* stream) {
    const grass_status st = check_products(dY, layout, ldy, X, ldx, dt, T, m, n);
    if (st != GRASS_OK) return st;
    if (!present(sumsq, m)) return GRASS_ERR_NULL;
    if (m > kMaxGridRows) return GRASS_ERR_SHAPE;
    if (!ws || ws_bytes < grad_row_stats_workspace_bytes(T, m, n, dt, layout, ldy, ldx))
        return GRASS_ERR_WORKSPACE;
    return launch_grad_row_stats(dY, layout, ldy, X, ldx, dt, T, m, n, sumsq, ws, ws_bytes,
                                 as_stream(stream));
}

grass_status grass_gather_rows(const void* G, grass_dtype gdt, int64_t m, int64_t n, int64_t ldg,
                               const int32_t* idx, const float* rho, int64_t r, float* out,
                               int64_t ldo, void* stream) {
    if (m < 0 || n < 0 || r < 0 || ldg < n || ldo < n || r > kMaxGridRows || !small(m) ||
        !small(n) || (r > 0 && m == 0))
        return GRASS_ERR_SHAPE;
    if (!present(G, m * n) || !present(idx, r) || !present(rho, r) || !present(out, r * n))
        return GRASS_ERR_NULL;
    if (!dtype_ok(gdt)) return GRASS_ERR_DTYPE;
    return launch_gather_rows(G, gdt, n, ldg, idx, rho, r, out, ldo, as_stream(stream));
}

grass_status grass_set_test_option(grass_test_option option, int value) {
    const int which = static_cast<int>(option);
    if (which < 0 || which >= kNumTestOptions) return GRASS_ERR_DTYPE;
    g_test_options[which].store(value, std::memory_order_relaxed);
    return GRASS_OK;
}

}  // extern "C"
