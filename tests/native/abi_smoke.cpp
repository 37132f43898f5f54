// Stand-alone user of the C ABI: no Python, no torch.  Allocates with hipMalloc, runs one
// refresh (row statistic, selection) and one regular step (compressed gradient, fused Adam +
// row update) of a small bf16 layer through libgrass.so, and checks every result against the
// fp64 oracle library (libgrass_ref.so).  Exit status 0 = all checks passed.
//
// Built by paper_2406_17660_amd/build.py (hipcc, host code only); run by tests/test_gpu_native.py.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/grass.h"

extern "C" {  // the oracle (test infrastructure): plain C, fp64
int grass_ref_full_grad(const void* dY, int layout, int64_t ldy, const void* X, int64_t ldx, int dt,
                        int64_t T, int64_t m, int64_t n, double* G);
int grass_ref_row_stats(const void* G, int dt, int64_t m, int64_t n, int64_t ldg, double* sumsq);
int grass_ref_compressed_grad(const void* dY, int layout, int64_t ldy, const void* X, int64_t ldx,
                              int dt, int64_t T, int64_t m, int64_t n, int64_t r,
                              const int32_t* idx, const float* rho, double* GC);
int grass_ref_adam_rows(const double* GC, int64_t ldgc, double* M, double* V, int64_t r, int64_t n,
                        double lr, double beta1, double beta2, double eps, int64_t t, double* U);
int grass_ref_scatter_update(double* W, int64_t m, int64_t n, int64_t ldw, const int32_t* idx,
                             const float* rho, double alpha, const double* U, int64_t r);
int grass_ref_select_rows(const float* sumsq, int64_t m, int64_t r, int method, int replacement,
                          int scale, uint64_t seed, uint64_t refresh_id, int32_t* idx, float* rho,
                          double* rho_unrounded);
}

#define HIP_OK(x)                                                                        \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
            return 2;                                                                    \
        }                                                                                \
    } while (0)
#define GRASS_OK_OR_FAIL(x)                                                              \
    do {                                                                                 \
        grass_status s_ = (x);                                                           \
        if (s_ != GRASS_OK) {                                                            \
            std::printf("%s failed: %s\n", #x, grass_status_string(s_));                 \
            return 3;                                                                    \
        }                                                                                \
    } while (0)

static uint16_t to_bf16(float f) {  // round to nearest even
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u += 0x7FFF + ((u >> 16) & 1);
    return static_cast<uint16_t>(u >> 16);
}
static double from_bf16(uint16_t b) {
    uint32_t u = static_cast<uint32_t>(b) << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}
static uint64_t rng_state = 0x2406176600ull;
static float uniform_pm1() {  // xorshift64*: inputs only, not part of the method
    rng_state ^= rng_state >> 12;
    rng_state ^= rng_state << 25;
    rng_state ^= rng_state >> 27;
    return static_cast<float>((rng_state * 0x2545F4914F6CDD1Dull) >> 40) / 8388608.0f - 1.0f;
}
static double rel_fro(const std::vector<double>& got, const std::vector<double>& want) {
    double num = 0, den = 0;
    for (size_t i = 0; i < got.size(); ++i) {
        num += (got[i] - want[i]) * (got[i] - want[i]);
        den += want[i] * want[i];
    }
    return den > 0 ? std::sqrt(num / den) : std::sqrt(num);
}

int main() {
    const int64_t T = 1056, m = 320, n = 264, r = 72;
    const float lr = 1e-3f, b1 = 0.9f, b2 = 0.999f, eps = 1e-8f, alpha = 0.25f;
    std::vector<uint16_t> dY(T * m), X(T * n), W(m * n);
    for (auto& v : dY) v = to_bf16(0.1f * uniform_pm1());
    for (auto& v : X) v = to_bf16(uniform_pm1());
    for (auto& v : W) v = to_bf16(0.02f * uniform_pm1());

    void *d_dY, *d_X, *d_W, *d_ws_stat, *d_ws_sel, *d_ws_gemm;
    float *d_ss, *d_rho, *d_GC, *d_M, *d_V;
    int32_t* d_idx;
    HIP_OK(hipMalloc(&d_dY, dY.size() * 2));
    HIP_OK(hipMalloc(&d_X, X.size() * 2));
    HIP_OK(hipMalloc(&d_W, W.size() * 2));
    HIP_OK(hipMalloc(&d_ss, m * 4));
    HIP_OK(hipMalloc(&d_idx, r * 4));
    HIP_OK(hipMalloc(&d_rho, r * 4));
    HIP_OK(hipMalloc(&d_GC, r * n * 4));
    HIP_OK(hipMalloc(&d_M, r * n * 4));
    HIP_OK(hipMalloc(&d_V, r * n * 4));
    HIP_OK(hipMemcpy(d_dY, dY.data(), dY.size() * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_X, X.data(), X.size() * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_W, W.data(), W.size() * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemset(d_M, 0, r * n * 4));
    HIP_OK(hipMemset(d_V, 0, r * n * 4));
    const size_t b_stat = grass_grad_row_stats_workspace(T, m, n, GRASS_BF16, GRASS_DY_TxM, m, n);
    const size_t b_sel = grass_select_workspace(m, r, GRASS_SEL_MULTI_NORM, 0);
    const size_t b_gemm = grass_cgrad_workspace(T, m, n, r, GRASS_BF16, GRASS_DY_TxM);
    HIP_OK(hipMalloc(&d_ws_stat, b_stat));
    HIP_OK(hipMalloc(&d_ws_sel, b_sel));
    HIP_OK(hipMalloc(&d_ws_gemm, b_gemm));
    hipStream_t s;
    HIP_OK(hipStreamCreate(&s));

    // The oracle's statistic first: nothing the GPU computes goes into the oracle, so the rows
    // are selected, on both sides, from the oracle's statistic rounded once to fp32.
    std::vector<double> G(m * n), ss_ref(m);
    if (grass_ref_full_grad(dY.data(), 0, m, X.data(), n, 1, T, m, n, G.data()) != 0) return 4;
    if (grass_ref_row_stats(G.data(), 2, m, n, n, ss_ref.data()) != 0) return 4;
    std::vector<float> ss32(ss_ref.begin(), ss_ref.end());
    float* d_ss32 = nullptr;
    HIP_OK(hipMalloc(&d_ss32, m * 4));
    HIP_OK(hipMemcpy(d_ss32, ss32.data(), m * 4, hipMemcpyHostToDevice));

    // refresh: row statistic of G (G itself is never stored), then selection without replacement
    GRASS_OK_OR_FAIL(grass_grad_row_stats(d_dY, GRASS_DY_TxM, m, d_X, n, GRASS_BF16, T, m, n, d_ss,
                                          d_ws_stat, b_stat, s));
    GRASS_OK_OR_FAIL(grass_select_rows(d_ss32, m, r, GRASS_SEL_MULTI_NORM, 0, GRASS_SCALE_PAPER, 77, 0,
                                       d_idx, d_rho, d_ws_sel, b_sel, s));
    // regular step
    GRASS_OK_OR_FAIL(grass_compressed_grad(d_dY, GRASS_DY_TxM, m, d_X, n, GRASS_BF16, T, m, n, r,
                                           d_idx, d_rho, d_GC, n, d_ws_gemm, b_gemm, s));
    GRASS_OK_OR_FAIL(grass_adam_scatter(d_GC, n, d_M, d_V, r, n, lr, b1, b2, eps, 1, d_W, GRASS_BF16,
                                        m, n, d_idx, d_rho, alpha, s));
    HIP_OK(hipStreamSynchronize(s));

    std::vector<float> ss(m), rho(r), GC(r * n), M(r * n), V(r * n);
    std::vector<int32_t> idx(r);
    std::vector<uint16_t> Wn(m * n);
    int32_t sel_status = -1;
    HIP_OK(hipMemcpy(ss.data(), d_ss, m * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(idx.data(), d_idx, r * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(rho.data(), d_rho, r * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(GC.data(), d_GC, r * n * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(M.data(), d_M, r * n * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(V.data(), d_V, r * n * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(Wn.data(), d_W, m * n * 2, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&sel_status, d_ws_sel, 4, hipMemcpyDeviceToHost));

    int failures = 0;
    auto check = [&](bool ok, const char* what, double value) {
        std::printf("%-34s %s (%.3g)\n", what, ok ? "ok" : "FAILED", value);
        if (!ok) ++failures;
    };
    check(sel_status == GRASS_OK, "selection status word", sel_status);
    check(rel_fro(std::vector<double>(ss.begin(), ss.end()), ss_ref) <= 1e-5, "row statistic", 0);
    std::vector<int32_t> idx_ref(r);
    std::vector<float> rho_ref(r);
    if (grass_ref_select_rows(ss32.data(), m, r, 2, 0, 0, 77, 0, idx_ref.data(), rho_ref.data(), nullptr) != 0)
        return 4;
    check(idx == idx_ref && rho == rho_ref, "selected rows and scales, bit-exact", r);
    std::vector<double> GC_ref(r * n), Mr(r * n, 0.0), Vr(r * n, 0.0), U(r * n), Wr(m * n);
    if (grass_ref_compressed_grad(dY.data(), 0, m, X.data(), n, 1, T, m, n, r, idx_ref.data(),
                                  rho_ref.data(), GC_ref.data()) != 0)
        return 4;
    const double e_gc = rel_fro(std::vector<double>(GC.begin(), GC.end()), GC_ref);
    check(e_gc <= 2e-5, "compressed gradient", e_gc);
    if (grass_ref_adam_rows(GC_ref.data(), n, Mr.data(), Vr.data(), r, n, lr, b1, b2, eps, 1, U.data()) != 0)
        return 4;
    for (int64_t i = 0; i < m * n; ++i) Wr[i] = from_bf16(W[i]);
    if (grass_ref_scatter_update(Wr.data(), m, n, n, idx_ref.data(), rho_ref.data(), alpha, U.data(), r) != 0)
        return 4;
    check(rel_fro(std::vector<double>(M.begin(), M.end()), Mr) <= 1e-5, "first moment", 0);
    check(rel_fro(std::vector<double>(V.begin(), V.end()), Vr) <= 1e-5, "second moment", 0);
    std::vector<double> Wsel_got, Wsel_want;
    bool untouched_same = true;
    std::vector<char> selected(m, 0);
    for (int32_t k : idx_ref) selected[k] = 1;
    for (int64_t k = 0; k < m; ++k)
        for (int64_t i = 0; i < n; ++i) {
            if (selected[k]) {
                Wsel_got.push_back(from_bf16(Wn[k * n + i]));
                Wsel_want.push_back(Wr[k * n + i]);
            } else if (Wn[k * n + i] != W[k * n + i]) {
                untouched_same = false;
            }
        }
    const double e_w = rel_fro(Wsel_got, Wsel_want);
    check(e_w <= 1e-2, "updated rows of W", e_w);
    check(untouched_same, "other rows of W bit-identical", 0);
    std::printf(failures ? "FAILED: %d check(s)\n" : "all checks passed\n", failures);
    return failures ? 1 : 0;
}
