/*
 * grass_ref.c - CPU oracle for the GRASS per-layer step.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of what the GPU library computes, written
 * from the paper's definitions so that it can be checked against them by eye.
 * It shares no code, header, table or helper with the HIP path.  Only the test
 * suite, the smoke check and the benchmark's cpu_baseline leg may call it; the
 * product never does.
 *
 * Inputs are the same bits the GPU consumes (fp32 or bf16), widened exactly to
 * double one element at a time.  All arithmetic is IEEE double except the
 * selection rule, which is defined on integers (see grass_ref_select_rows).
 * OpenMP is used only as "parallel for" over independent output rows; every
 * single output value is produced by one sequential loop in the order the
 * definition states.
 *
 * Pins (tests/test_oracle_*.py): brute-force loops and hand-worked cases for the
 * two matrix products; closed forms for Adam at t = 1, 2 and a library Adam;
 * exhaustive subset search for Top-r; unbiasedness, the closed-form total
 * variance and the printed 97.66 % coverage figure for the samplers; exact
 * enumeration for sampling without replacement; published known-answer vectors
 * for Philox4x32-10.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { REF_OK = 0, REF_ERR_NULL = 1, REF_ERR_SHAPE = 2, REF_ERR_DTYPE = 3, REF_ERR_NONFINITE = 5 };
enum { DT_F32 = 0, DT_BF16 = 1, DT_F64 = 2 };
enum { SEL_TOPR = 0, SEL_UNIFORM = 1, SEL_MULTI_NORM = 2, SEL_MULTI_NORM2 = 3 };
enum { SCALE_PAPER = 0, SCALE_ONE = 1, SCALE_INV_SQRT_RQ = 2 };
enum { DY_TxM = 0, DY_MxT = 1 };

/* Exact widening of one stored element to double. */
static double elem(const void* p, int dt, int64_t i) {
    if (dt == DT_F32) return (double)((const float*)p)[i];
    if (dt == DT_F64) return ((const double*)p)[i];
    /* bf16 = the upper 16 bits of an IEEE float */
    uint32_t bits = (uint32_t)((const uint16_t*)p)[i] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

static int dtype_ok(int dt) { return dt == DT_F32 || dt == DT_BF16 || dt == DT_F64; }

/* dY[t, k] under either storage order. */
static double dy_at(const void* dY, int layout, int64_t ldy, int dt, int64_t t, int64_t k) {
    return layout == DY_TxM ? elem(dY, dt, t * ldy + k) : elem(dY, dt, k * ldy + t);
}

/* Full gradient, Section 3.1 / Appendix F:  G = (grad_y L)^T X,
 * G[k, i] = sum_t dY[t, k] * X[t, i].  G is dense m x n doubles. */
int grass_ref_full_grad(const void* dY, int layout, int64_t ldy, const void* X, int64_t ldx,
                        int dt, int64_t T, int64_t m, int64_t n, double* G) {
    if (!dY || !X || !G) return REF_ERR_NULL;
    if (!dtype_ok(dt)) return REF_ERR_DTYPE;
    if (T < 0 || m < 0 || n < 0 || ldx < n) return REF_ERR_SHAPE;
#pragma omp parallel for schedule(dynamic)
    for (int64_t k = 0; k < m; ++k)
        for (int64_t i = 0; i < n; ++i) {
            double s = 0.0;
            for (int64_t t = 0; t < T; ++t)
                s += dy_at(dY, layout, ldy, dt, t, k) * elem(X, dt, t * ldx + i);
            G[k * n + i] = s;
        }
    return REF_OK;
}

/* Row statistic used by compute_P (Section 3.2): sumsq[k] = ||G_k||_2^2. */
int grass_ref_row_stats(const void* G, int dt, int64_t m, int64_t n, int64_t ldg, double* sumsq) {
    if (!G || !sumsq) return REF_ERR_NULL;
    if (!dtype_ok(dt)) return REF_ERR_DTYPE;
    if (m < 0 || n < 0 || ldg < n) return REF_ERR_SHAPE;
    for (int64_t k = 0; k < m; ++k) {
        double s = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double g = elem(G, dt, k * ldg + i);
            s += g * g;
        }
        sumsq[k] = s;
    }
    return REF_OK;
}

/* Compressed gradient, Section 3.1: P^T G = rho ((B dY^T) X), i.e.
 * GC[j, i] = rho_j * sum_t dY[t, sigma_j] * X[t, i].  GC is dense r x n doubles. */
int grass_ref_compressed_grad(const void* dY, int layout, int64_t ldy, const void* X, int64_t ldx,
                              int dt, int64_t T, int64_t m, int64_t n, int64_t r,
                              const int32_t* idx, const float* rho, double* GC) {
    if (!dY || !X || !GC || !idx || !rho) return REF_ERR_NULL;
    if (!dtype_ok(dt)) return REF_ERR_DTYPE;
    if (T < 0 || m < 0 || n < 0 || r < 0 || ldx < n) return REF_ERR_SHAPE;
    for (int64_t j = 0; j < r; ++j)
        if (idx[j] < 0 || idx[j] >= m) return REF_ERR_SHAPE;
#pragma omp parallel for schedule(dynamic)
    for (int64_t j = 0; j < r; ++j)
        for (int64_t i = 0; i < n; ++i) {
            double s = 0.0;
            for (int64_t t = 0; t < T; ++t)
                s += dy_at(dY, layout, ldy, dt, t, idx[j]) * elem(X, dt, t * ldx + i);
            GC[j * n + i] = (double)rho[j] * s;
        }
    return REF_OK;
}

/* adam.update of Appendix A, in the order printed there.  M, V, U dense r x n. */
int grass_ref_adam_rows(const double* GC, int64_t ldgc, double* M, double* V, int64_t r, int64_t n,
                        double lr, double beta1, double beta2, double eps, int64_t t, double* U) {
    if (!GC || !M || !V || !U) return REF_ERR_NULL;
    if (r < 0 || n < 0 || ldgc < n || t < 1) return REF_ERR_SHAPE;
    if (!(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0)) return REF_ERR_SHAPE;
    const double c1 = 1.0 - pow(beta1, (double)t);
    const double c2 = 1.0 - pow(beta2, (double)t);
    for (int64_t j = 0; j < r; ++j)
        for (int64_t i = 0; i < n; ++i) {
            const double g = GC[j * ldgc + i];
            const double mn = beta1 * M[j * n + i] + (1.0 - beta1) * g;
            const double vn = beta2 * V[j * n + i] + (1.0 - beta2) * g * g;
            M[j * n + i] = mn;
            V[j * n + i] = vn;
            const double ms = mn / c1;
            const double vs = vn / c2;
            U[j * n + i] = -lr * ms / (sqrt(vs) + eps);
        }
    return REF_OK;
}

/* Nearest bf16 value (8 significant bits, ties to even) of a double, as a double. */
double grass_ref_round_bf16(double x) {
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);       /* |x| in [2^(e-1), 2^e) */
    int q = e - 8;            /* spacing of bf16 values there is 2^q */
    if (q < -133) q = -133;   /* subnormal range: fixed spacing 2^-133 */
    const double y = ldexp(nearbyint(ldexp(x, -q)), q); /* default rounding mode: ties to even */
    return fabs(y) >= ldexp(1.0, 128) ? copysign(INFINITY, x) : y;
}

/* adam.update of Appendix A with the moments KEPT IN bf16 (the pure-bf16 optimizer state of
 * the paper's memory accounting, Appendix "Optimizer State Memory Calculation"): the new
 * moments are rounded once to bf16, stored, and the update is computed from the stored
 * values, so that U is a function of the state a checkpoint would hold.  M and V are
 * double arrays whose values are bf16-representable on entry and on exit. */
int grass_ref_adam_rows_bf16state(const double* GC, int64_t ldgc, double* M, double* V, int64_t r,
                                  int64_t n, double lr, double beta1, double beta2, double eps,
                                  int64_t t, double* U) {
    if (!GC || !M || !V || !U) return REF_ERR_NULL;
    if (r < 0 || n < 0 || ldgc < n || t < 1) return REF_ERR_SHAPE;
    if (!(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0)) return REF_ERR_SHAPE;
    const double c1 = 1.0 - pow(beta1, (double)t);
    const double c2 = 1.0 - pow(beta2, (double)t);
    for (int64_t j = 0; j < r; ++j)
        for (int64_t i = 0; i < n; ++i) {
            const double g = GC[j * ldgc + i];
            const double mn = grass_ref_round_bf16(beta1 * M[j * n + i] + (1.0 - beta1) * g);
            const double vn = grass_ref_round_bf16(beta2 * V[j * n + i] + (1.0 - beta2) * g * g);
            M[j * n + i] = mn;
            V[j * n + i] = vn;
            const double ms = mn / c1;
            const double vs = vn / c2;
            U[j * n + i] = -lr * ms / (sqrt(vs) + eps);
        }
    return REF_OK;
}

/* Weight update of Algorithm 1 with P = (rho B)^T:  W += alpha * P * U, i.e. row
 * sigma_j of W receives alpha * rho_j * U_j; a row selected several times receives
 * the sum (that is what the product P U does). */
int grass_ref_scatter_update(double* W, int64_t m, int64_t n, int64_t ldw, const int32_t* idx,
                             const float* rho, double alpha, const double* U, int64_t r) {
    if (!W || !idx || !rho || !U) return REF_ERR_NULL;
    if (m < 0 || n < 0 || r < 0 || ldw < n) return REF_ERR_SHAPE;
    for (int64_t j = 0; j < r; ++j)
        if (idx[j] < 0 || idx[j] >= m) return REF_ERR_SHAPE;
    for (int64_t j = 0; j < r; ++j)
        for (int64_t i = 0; i < n; ++i)
            W[(int64_t)idx[j] * ldw + i] += alpha * (double)rho[j] * U[j * n + i];
    return REF_OK;
}

/* Right-hand (column) projection, used when the input dimension is the smaller one
 * (Section 4.1 projects whichever dimension of G is smaller): the r selected columns of
 * W receive the update, W[:, sigma_j] += alpha * rho_j * U[j, :]^T with U of shape r x m.
 * This is W + alpha * (P U)^T for the n x r projection P = (rho B)^T. */
int grass_ref_scatter_update_cols(double* W, int64_t m, int64_t n, int64_t ldw, const int32_t* idx,
                                  const float* rho, double alpha, const double* U, int64_t r) {
    if (!W || !idx || !rho || !U) return REF_ERR_NULL;
    if (m < 0 || n < 0 || r < 0 || ldw < n) return REF_ERR_SHAPE;
    for (int64_t j = 0; j < r; ++j)
        if (idx[j] < 0 || idx[j] >= n) return REF_ERR_SHAPE;
    for (int64_t j = 0; j < r; ++j)
        for (int64_t i = 0; i < m; ++i)
            W[i * ldw + idx[j]] += alpha * (double)rho[j] * U[j * m + i];
    return REF_OK;
}

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
 * 1, 2, 3", SC'11): ten rounds of two 32x32->64 multiplications, a word
 * permutation and key injection; the key is advanced by Weyl constants between
 * rounds. */
void grass_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u; /* golden ratio */
            k1 += 0xBB67AE85u; /* sqrt(3) - 1  */
        }
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 64-bit random word of draw j: key = seed, counter = (j, refresh_id), low
 * 32-bit halves first; the word is output[0] + 2^32 * output[1]. */
uint64_t grass_ref_draw_word(uint64_t seed, uint64_t refresh_id, uint64_t j) {
    uint32_t ctr[4] = {(uint32_t)j, (uint32_t)(j >> 32), (uint32_t)refresh_id,
                       (uint32_t)(refresh_id >> 32)};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    grass_ref_philox4x32_10(ctr, key, out);
    return (uint64_t)out[0] | ((uint64_t)out[1] << 32);
}

/* floor(a * b / 2^64) */
uint64_t grass_ref_mulhi64(uint64_t a, uint64_t b) {
    return (uint64_t)(((unsigned __int128)a * (unsigned __int128)b) >> 64);
}

/* Integer sampling weights.  w_k = ||G_k|| (Theorem 3.1), ||G_k||^2 (Norm^2) or 1
 * (uniform); quantised relative to the largest one on a 2^40 grid, plus 1 so
 * that every q_k > 0 (the unbiasedness theorem of Appendix D needs that). */
int grass_ref_sampling_weights(const float* sumsq, int64_t m, int method, uint64_t* wq) {
    if (!sumsq || !wq) return REF_ERR_NULL;
    if (method != SEL_UNIFORM && method != SEL_MULTI_NORM && method != SEL_MULTI_NORM2)
        return REF_ERR_DTYPE;
    double wmax = 0.0;
    for (int64_t k = 0; k < m; ++k) {
        const double s = (double)sumsq[k];
        if (!(s >= 0.0) || isinf(s)) return REF_ERR_NONFINITE;
        const double w = method == SEL_UNIFORM ? 1.0 : method == SEL_MULTI_NORM ? sqrt(s) : s;
        if (w > wmax) wmax = w;
    }
    for (int64_t k = 0; k < m; ++k) {
        const double s = (double)sumsq[k];
        const double w = method == SEL_UNIFORM ? 1.0 : method == SEL_MULTI_NORM ? sqrt(s) : s;
        wq[k] = wmax == 0.0 ? 1u : (uint64_t)floor(w / wmax * 1099511627776.0) + 1u;
    }
    return REF_OK;
}

static int cmp_i32(const void* a, const void* b) {
    const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

typedef struct { uint32_t key; int32_t row; } keyed_row;

/* larger key first; equal keys: lower row first */
static int cmp_keyed(const void* a, const void* b) {
    const keyed_row* x = (const keyed_row*)a;
    const keyed_row* y = (const keyed_row*)b;
    if (x->key != y->key) return x->key > y->key ? -1 : 1;
    return (x->row > y->row) - (x->row < y->row);
}

/* compute_P of Section 3.2.  Output idx ascending, rho as float (rho_d, if given,
 * receives the unrounded doubles). */
int grass_ref_select_rows(const float* sumsq, int64_t m, int64_t r, int method, int replacement,
                          int scale, uint64_t seed, uint64_t refresh_id, int32_t* idx, float* rho,
                          double* rho_d) {
    if (!sumsq || (r > 0 && (!idx || !rho))) return REF_ERR_NULL;
    if (m < 0 || r < 0 || m >= 2147483648LL) return REF_ERR_SHAPE;
    if (method < SEL_TOPR || method > SEL_MULTI_NORM2) return REF_ERR_DTYPE;
    if (scale < SCALE_PAPER || scale > SCALE_INV_SQRT_RQ) return REF_ERR_DTYPE;
    if (method == SEL_TOPR && scale == SCALE_INV_SQRT_RQ) return REF_ERR_DTYPE;
    const int with_repl = (method != SEL_TOPR) && replacement;
    if (!with_repl && r > m) return REF_ERR_SHAPE;
    if (r > 0 && m == 0) return REF_ERR_SHAPE;
    for (int64_t k = 0; k < m; ++k) {
        const double s = (double)sumsq[k];
        if (!(s >= 0.0) || isinf(s)) return REF_ERR_NONFINITE;
    }
    if (r == 0) return REF_OK;

    if (method == SEL_TOPR) {
        /* Deterministic construction: the r rows of largest norm, rho = 1.  Norms
         * are compared through sumsq (sqrt is monotone); non-negative floats order
         * like their bit patterns; -0 counts as 0. */
        keyed_row* a = (keyed_row*)malloc((size_t)m * sizeof(keyed_row));
        for (int64_t k = 0; k < m; ++k) {
            uint32_t bits;
            memcpy(&bits, &sumsq[k], 4);
            a[k].key = sumsq[k] == 0.0f ? 0u : bits;
            a[k].row = (int32_t)k;
        }
        qsort(a, (size_t)m, sizeof(keyed_row), cmp_keyed);
        for (int64_t j = 0; j < r; ++j) idx[j] = a[j].row;
        free(a);
        qsort(idx, (size_t)r, sizeof(int32_t), cmp_i32);
        for (int64_t j = 0; j < r; ++j) {
            rho[j] = 1.0f;
            if (rho_d) rho_d[j] = 1.0;
        }
        return REF_OK;
    }

    /* Stochastic construction: sigma_j ~ Multinomial(1, q), q_k = wq_k / total. */
    uint64_t* wq = (uint64_t*)malloc((size_t)m * sizeof(uint64_t));
    uint64_t* w0 = (uint64_t*)malloc((size_t)m * sizeof(uint64_t));
    int rc = grass_ref_sampling_weights(sumsq, m, method, wq);
    if (rc != REF_OK) { free(wq); free(w0); return rc; }
    memcpy(w0, wq, (size_t)m * sizeof(uint64_t));
    uint64_t total = 0;
    for (int64_t k = 0; k < m; ++k) total += wq[k];

    uint64_t remaining = total;
    for (int64_t j = 0; j < r; ++j) {
        const uint64_t x = grass_ref_draw_word(seed, refresh_id, (uint64_t)j);
        const uint64_t target = grass_ref_mulhi64(x, remaining);
        /* first k whose inclusive prefix sum of the current weights exceeds target */
        uint64_t c = 0;
        int64_t pick = -1;
        for (int64_t k = 0; k < m; ++k) {
            c += wq[k];
            if (c > target) { pick = k; break; }
        }
        idx[j] = (int32_t)pick; /* pick >= 0 because target < remaining = sum wq */
        if (!replacement) { remaining -= wq[pick]; wq[pick] = 0; }
    }
    qsort(idx, (size_t)r, sizeof(int32_t), cmp_i32);

    const int rescale = scale == SCALE_INV_SQRT_RQ || (scale == SCALE_PAPER && replacement);
    for (int64_t j = 0; j < r; ++j) {
        double rj = 1.0;
        if (rescale) {
            const double q = (double)w0[idx[j]] / (double)total;
            rj = 1.0 / sqrt((double)r * q);
        }
        rho[j] = (float)rj;
        if (rho_d) rho_d[j] = rj;
    }
    free(wq);
    free(w0);
    return REF_OK;
}
