/*
 * grass.h - C ABI of the GRASS structured-sparse gradient step for one linear layer
 *           on one AMD MI355X (gfx950).
 *
 * Notation (paper, Sections 2 and 3.1): a linear layer has weight W (m x n), input
 * activations X (T x n) and output gradient dY (T x m), T being the token batch
 * (the paper's b).  The full weight gradient is G = dY^T X (m x n).  GRASS uses a
 * sparse projection P (m x r) with one nonzero per column, stored as
 * P^T = rho * B: `idx[j]` (the paper's sigma_j) is the row of G that column j of P
 * selects and `rho[j]` its scale.  One optimisation step (Algorithm 1) is
 *
 *     refresh, every K steps:  sumsq = row norms^2 of G;  (idx, rho) = compute_P(sumsq)
 *     every step:              G_C = P^T G = rho * ((B dY^T) X)          (r x n)
 *                              (M, V, U) = Adam(M, V, G_C)               (r x n)
 *                              W += alpha * P * U                        (r rows of W)
 *
 * Conventions that hold for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller, unless the
 *     argument is documented as a host value.  The library allocates no memory;
 *     scratch memory is sized by the *_workspace queries and passed in by the caller.
 *     It keeps no state that a result depends on.  What it does keep, per process: one
 *     flag per device and kernel recording that the kernel's LDS limit has been raised
 *     (set once, atomically), and the test hooks of grass_set_test_option (initially
 *     off).
 *   - Matrices are row-major with an explicit leading dimension counted in
 *     ELEMENTS (ld >= number of columns).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it; no call synchronises with the host.
 *   - Arguments are validated on the host before anything is launched.  A call
 *     that returns an argument error (NULL, SHAPE, DTYPE, WORKSPACE) has launched
 *     nothing and written nothing.  GRASS_ERR_DEVICE reports a launch the HIP runtime
 *     refused; kernels the call enqueued before it still run, and the outputs are
 *     then unspecified.  A pointer may be NULL only when the array it names has no
 *     elements.
 *   - Calls that walk the compressed rows in the grid (compressed_grad,
 *     scatter_update, adam_scatter, gather_rows, dense_grad's m) accept at most
 *     65535 rows and return GRASS_ERR_SHAPE beyond that.
 *   - r = 0, n = 0 or T = 0 are legal where they make sense (see each call) and
 *     produce the empty / zero result.  Every size (T, m, n, r) is below 2^31;
 *     GRASS_ERR_SHAPE (0 from a workspace query) beyond that.
 *   - Index arrays (idx) live in device memory, so their VALUES cannot be validated
 *     before the launch: every entry must lie inside the dimension it indexes
 *     (grass_select_rows writes such arrays).  Entries outside it make the kernels
 *     read or write outside the caller's buffers.
 *   - No call records a memset or an event (the _timed call excepted) or allocates, so
 *     calls can be captured into a HIP graph.
 */
#ifndef GRASS_H
#define GRASS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GRASS_OK = 0,
    GRASS_ERR_NULL = 1,      /* a required pointer is NULL                              */
    GRASS_ERR_SHAPE = 2,     /* negative size, r > m where forbidden, ld too small ...  */
    GRASS_ERR_DTYPE = 3,     /* dtype / enum value not supported by this call           */
    GRASS_ERR_WORKSPACE = 4, /* workspace pointer NULL or smaller than the query says   */
    GRASS_ERR_NONFINITE = 5, /* sumsq holds NaN, Inf or a negative value (select only)  */
    GRASS_ERR_DEVICE = 6     /* a HIP launch failed                                     */
} grass_status;

typedef enum { GRASS_F32 = 0, GRASS_BF16 = 1 } grass_dtype;

/* compute_P rules of Section 3.2.  The sampling rules draw sigma_j from
 * Multinomial(1, q) with q_k = 1/m (UNIFORM), q_k ~ ||G_k|| (MULTI_NORM, Theorem 3.1)
 * or q_k ~ ||G_k||^2 (MULTI_NORM2); TOPR takes the r rows of largest norm. */
typedef enum {
    GRASS_SEL_TOPR = 0,
    GRASS_SEL_UNIFORM = 1,
    GRASS_SEL_MULTI_NORM = 2,
    GRASS_SEL_MULTI_NORM2 = 3
} grass_method;

/* How rho is set.  PAPER follows Section 3.2: 1/sqrt(r*q_sigma) when sampling
 * with replacement, 1 for sampling without replacement and for Top-r.  ONE and
 * INV_SQRT_RQ force one of the two rules whatever the method (INV_SQRT_RQ uses
 * the q of the initial distribution; with TOPR it is rejected). */
typedef enum {
    GRASS_SCALE_PAPER = 0,
    GRASS_SCALE_ONE = 1,
    GRASS_SCALE_INV_SQRT_RQ = 2
} grass_scale;

/* Storage of the output gradient: GRASS_DY_TxM is dY[t*ldy + k] (what a backward
 * pass produces, Section 3.1), GRASS_DY_MxT is its transpose dY[k*ldy + t]. */
typedef enum { GRASS_DY_TxM = 0, GRASS_DY_MxT = 1 } grass_dy_layout;

/* Readable name of a status code.  Returns a static string; never NULL. */
const char* grass_status_string(grass_status s);

/* ---------------------------------------------------------------------------
 * compute_P, part 1 (Section 3.2; cost "mn" in the FLOP table of Appendix F):
 *   sumsq[k] = sum_j G[k, j]^2,  the squared 2-norm of row k of G.
 * G: m x n, dtype `dt`, leading dimension ldg.  sumsq: m floats (fp32
 * accumulation).  m = 0 is a no-op; n = 0 writes zeros.
 * Errors: NULL, SHAPE (m, n < 0, ldg < n), DTYPE. */
grass_status grass_row_stats(const void* G, grass_dtype dt, int64_t m, int64_t n, int64_t ldg,
                             float* sumsq, void* stream);

/* ---------------------------------------------------------------------------
 * compute_P, part 2 (Section 3.2): choose idx[r] and rho[r] from sumsq[m].
 *
 * TOPR: the r rows with the largest sumsq; ties go to the lower row index.
 * Sampling rules: integer weights wq_k = floor(w_k / max_i w_i * 2^40) + 1 with
 *   w_k = sqrt(sumsq_k) (MULTI_NORM), sumsq_k (MULTI_NORM2) or 1 (UNIFORM), all in
 *   IEEE double (if every w_k is 0 all wq_k are 1); q_k = wq_k / sum_i wq_i.
 *   Draw j uses the 64-bit word x_j = Philox4x32-10(key = seed,
 *   counter = (j, refresh_id)), low word first, and target = floor(x_j * S / 2^64).
 *   With replacement (replacement != 0): S = sum wq, sigma_j is the first k whose
 *   inclusive prefix sum exceeds target.  Without: draws are sequential, S is the
 *   weight still present, the drawn row's weight is set to 0 afterwards.
 * Output: idx sorted ascending (duplicates adjacent; only possible with
 *   replacement); rho per `scale`, rounded from double to float.
 * Requirements: 0 <= r; r <= m unless sampling with replacement; m < 2^31.
 * `ws` must hold grass_select_workspace(...) bytes.  Its first 4 bytes are a
 * device status word the caller may read back after the stream has finished:
 * GRASS_OK, or GRASS_ERR_NONFINITE when sumsq held NaN / Inf / a negative
 * value, in which case the placeholder idx[j] = floor(j*m/r), rho = 1 is written
 * so that later calls stay in bounds.
 * Errors (host, before launch): NULL, SHAPE, DTYPE (bad enum, or
 * INV_SQRT_RQ with TOPR), WORKSPACE. */
size_t grass_select_workspace(int64_t m, int64_t r, grass_method method, int replacement);
grass_status grass_select_rows(const float* sumsq, int64_t m, int64_t r, grass_method method,
                               int replacement, grass_scale scale, uint64_t seed,
                               uint64_t refresh_id, int32_t* idx, float* rho, void* ws,
                               size_t ws_bytes, void* stream);

/* grass_select_rows for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same arithmetic, same idx and rho bit for bit; the scratch the kernels need
 * (status word, prefix sums and hit counters, or the sampling tree) lives in a static device
 * array inside the library: grass_select_static_capacity() bytes (1 MiB) on every GPU the
 * library runs on, held until the process ends.  The call allocates nothing and frees nothing.
 * Limit: grass_select_workspace(m, r, method, replacement) must not exceed the capacity
 * (m up to 65536 rows for every rule); larger problems return GRASS_ERR_WORKSPACE and launch
 * nothing: use grass_select_rows for them.
 * `status`: NULL, or a device int32 that receives what grass_select_rows leaves in the first
 * 4 bytes of its workspace (GRASS_OK, or GRASS_ERR_NONFINITE with the placeholder selection).
 * All calls on one GPU share that GPU's array: calls that may overlap in time (different
 * streams, different threads) race; calls on one stream are ordered and each call initialises
 * what it reads, so nothing of an earlier call is seen.  The first call on a device looks up
 * the array's address (hipGetSymbolAddress): make it outside any stream capture.
 * Errors: as grass_select_rows; WORKSPACE for sizes beyond the capacity; DEVICE if the address
 * lookup or a launch fails. */
size_t grass_select_static_capacity(void);
grass_status grass_select_rows_static(const float* sumsq, int64_t m, int64_t r,
                                      grass_method method, int replacement, grass_scale scale,
                                      uint64_t seed, uint64_t refresh_id, int32_t* idx, float* rho,
                                      int32_t* status, void* stream);

/* ---------------------------------------------------------------------------
 * Compressed gradient (Section 3.1, "Efficient Gradient Projection"; Algorithm 1
 * line "G_C <- P^T grad"):
 *   GC[j, i] = rho[j] * sum_t dY[t, idx[j]] * X[t, i],   j < r, i < n.
 * The full m x n gradient is never formed.  dY and X have dtype `dt` (bf16 inputs
 * are multiplied on the matrix cores with fp32 accumulation); GC is fp32, r x n,
 * leading dimension ldgc.  idx values must lie in [0, m) (not checked on the
 * device: idx comes from grass_select_rows); duplicates are allowed.
 * T = 0 writes zeros.  `ws` must hold grass_cgrad_workspace(...) bytes.
 * Errors: NULL, SHAPE, DTYPE, WORKSPACE. */
size_t grass_cgrad_workspace(int64_t T, int64_t m, int64_t n, int64_t r, grass_dtype dt,
                             grass_dy_layout layout);
grass_status grass_compressed_grad(const void* dY, grass_dy_layout layout, int64_t ldy,
                                   const void* X, int64_t ldx, grass_dtype dt, int64_t T,
                                   int64_t m, int64_t n, int64_t r, const int32_t* idx,
                                   const float* rho, float* GC, int64_t ldgc, void* ws,
                                   size_t ws_bytes, void* stream);

/* How the product above is planned for `count` sets of gathered rows that share X (count = 1:
 * one matrix), `rows` rows in all (r for one matrix; for a group call the sum of its r[i], each
 * rounded up to a multiple of 8; the sets are taken to be of equal size), m the row length of
 * dY (0: not given).  `*tile` receives the edge of the output tile (256, 128, or 64 for fp32
 * inputs), or 0 for narrow layers (bf16, T x m storage, m <= 512, r <= 128 per set, n <= 512, T
 * a multiple of 16), whose gather runs inside the matrix-multiply kernel (128 x 256 tiles, no
 * packed panel); `*k_slices` the number of slices the token dimension is split into (their
 * partial products are what the split-K reduction, or the fused tail of grass_step_group /
 * grass_step_cols, adds up; above 8 slices those kernels spread the slices over the wavefronts
 * of a workgroup).  A pure host function, for callers that want to know what a shape costs and
 * for tests that must reach every kernel.  Operands whose base or leading dimension is not
 * 16-byte aligned take the packed route with the 128 tile at launch whatever this reports.
 * Errors: NULL, SHAPE, DTYPE. */
grass_status grass_cgrad_plan(int64_t T, int64_t m, int64_t n, int64_t rows, int count,
                              grass_dtype dt, grass_dy_layout layout, int* tile, int* k_slices);

/* grass_compressed_grad with a timing hook: the two hipEvent_t handles (passed as
 * void*; created by the caller; either may be NULL) receive the start and the end of the
 * matrix-multiply kernel, so that a caller can time that kernel apart from the gather and
 * reduction passes around it.  For the large-tile kernel the runtime stamps the events with
 * the kernel dispatch's own start and end (the interval a profiler's kernel trace reports);
 * for the other kernels they are recorded on `stream` immediately before and after the
 * launch.  Everything else is identical. */
grass_status grass_compressed_grad_timed(const void* dY, grass_dy_layout layout, int64_t ldy,
                                         const void* X, int64_t ldx, grass_dtype dt, int64_t T,
                                         int64_t m, int64_t n, int64_t r, const int32_t* idx,
                                         const float* rho, float* GC, int64_t ldgc, void* ws,
                                         size_t ws_bytes, void* stream, void* ev_gemm_start,
                                         void* ev_gemm_stop);

/* ---------------------------------------------------------------------------
 * Compressed gradients of several weight matrices that read the same activations
 * (the query, key and value projections of an attention block, or the gate and up
 * projections of an MLP: Section 4 trains all linear layers of a block).  For set
 * i < count:
 *   GC[i][j, c] = rho[i][j] * sum_t dY[i][t, idx[i][j]] * X[t, c],  j < r[i], c < n,
 * exactly what grass_compressed_grad returns for (dY[i], idx[i], rho[i]) alone; the
 * selected rows of all sets are gathered into one panel and multiplied with X in a
 * single pass over X.
 * dY, ldy, m, r, idx, rho, GC, ldgc are HOST arrays of `count` entries (1 <= count
 * <= GRASS_MAX_GROUP); the entries of dY, idx, rho and GC are device pointers.  All
 * sets share T, n, dt, layout, X and the stream.  Each GC[i] is fp32, r[i] x n,
 * leading dimension ldgc[i]; the outputs must not overlap.  `ws` must hold
 * grass_cgrad_group_workspace(...) bytes.
 * Errors: NULL, SHAPE (also count out of range), DTYPE, WORKSPACE. */
#define GRASS_MAX_GROUP 8
size_t grass_cgrad_group_workspace(int64_t T, int64_t n, int count, const int64_t* r,
                                   grass_dtype dt, grass_dy_layout layout);
grass_status grass_compressed_grad_group(int count, const void* const* dY, grass_dy_layout layout,
                                         const int64_t* ldy, const void* X, int64_t ldx,
                                         grass_dtype dt, int64_t T, const int64_t* m, int64_t n,
                                         const int64_t* r, const int32_t* const* idx,
                                         const float* const* rho, float* const* GC,
                                         const int64_t* ldgc, void* ws, size_t ws_bytes,
                                         void* stream);

/* ---------------------------------------------------------------------------
 * opt.update = Adam on the r x n compressed gradient (Appendix A, adam.update):
 *   M <- b1*M + (1-b1)*g        V <- b2*V + (1-b2)*g^2
 *   U  = -lr * (M/(1-b1^t)) / (sqrt(V/(1-b2^t)) + eps)
 * GC (ld ldgc), M, V, U (dense r x n) are fp32; M and V are updated in place.
 * t >= 1 is the 1-based count of Adam updates since M, V were last zeroed (the
 * caller resets it together with the state, Section 3.3).  lr, beta1, beta2, eps
 * and t are host values.
 * Errors: NULL, SHAPE (also t < 1, beta outside [0,1)). */
grass_status grass_adam_rows(const float* GC, int64_t ldgc, float* M, float* V, int64_t r,
                             int64_t n, float lr, float beta1, float beta2, float eps,
                             int64_t t, float* U, void* stream);

/* ---------------------------------------------------------------------------
 * Sparse weight update (Section 3.1, "Efficient Weight Update"; Algorithm 1 line
 * "W <- W + alpha P Delta"):
 *   W[idx[j], :] += alpha * rho[j] * U[j, :]      for j < r.
 * idx must be sorted ascending (as grass_select_rows writes it).  Rows that occur
 * several times receive the sum of their updates, accumulated in fp32 in j order
 * and rounded once (to nearest even) to W's dtype.  Rows not in idx are not
 * touched.  W: m x n of dtype wdt, leading dimension ldw, updated in place.
 * U: dense r x n fp32.
 * Errors: NULL, SHAPE, DTYPE. */
grass_status grass_scatter_update(void* W, grass_dtype wdt, int64_t m, int64_t n, int64_t ldw,
                                  const int32_t* idx, const float* rho, float alpha,
                                  const float* U, int64_t r, void* stream);

/* Column form of the sparse weight update, for layers whose input dimension n is the
 * smaller one (Section 4.1 projects the smaller dimension of G).  With an n x r projection
 * the compressed gradient is G P = (rho (B X^T) dY)^T, i.e. grass_compressed_grad called
 * with X in the place of dY and dY in the place of X (result r x m), the statistic is the
 * row statistic of G^T (grass_grad_row_stats / grass_dense_grad with the same exchange),
 * Adam runs on r x m state, and the update goes to r COLUMNS of W:
 *   W[:, idx[j]] += alpha * rho[j] * U[j, :]^T      for j < r,   U dense r x m fp32.
 * idx sorted ascending, values in [0, n); duplicates are summed in fp32 in j order and
 * rounded once.  Columns not in idx are not touched.
 * Errors: NULL, SHAPE, DTYPE. */
grass_status grass_scatter_update_cols(void* W, grass_dtype wdt, int64_t m, int64_t n, int64_t ldw,
                                       const int32_t* idx, const float* rho, float alpha,
                                       const float* U, int64_t r, void* stream);

/* Fused form of grass_adam_rows followed by grass_scatter_update: same
 * arithmetic, but U is never written to memory.  This is the call the regular
 * step uses. */
grass_status grass_adam_scatter(const float* GC, int64_t ldgc, float* M, float* V, int64_t r,
                                int64_t n, float lr, float beta1, float beta2, float eps,
                                int64_t t, void* W, grass_dtype wdt, int64_t m, int64_t ldw,
                                const int32_t* idx, const float* rho, float alpha,
                                void* stream);

/* grass_adam_rows and grass_adam_scatter with the moments M, V stored in dtype `sdt`
 * (GRASS_F32: identical to the calls above; GRASS_BF16: the pure-bf16 optimizer state of
 * the paper's memory accounting, Appendix "Optimizer State Memory Calculation", 2 bytes
 * per moment).  With bf16 moments each new moment is computed in fp32 from the stored
 * value, rounded once to bf16 (nearest even), stored, and the update U is computed from
 * the rounded values, so U depends only on what a checkpoint of the state holds.
 * Errors: as the fp32 calls, plus DTYPE for a bad `sdt`. */
grass_status grass_adam_rows_state(const float* GC, int64_t ldgc, void* M, void* V,
                                   grass_dtype sdt, int64_t r, int64_t n, float lr, float beta1,
                                   float beta2, float eps, int64_t t, float* U, void* stream);
grass_status grass_adam_scatter_state(const float* GC, int64_t ldgc, void* M, void* V,
                                      grass_dtype sdt, int64_t r, int64_t n, float lr, float beta1,
                                      float beta2, float eps, int64_t t, void* W, grass_dtype wdt,
                                      int64_t m, int64_t ldw, const int32_t* idx, const float* rho,
                                      float alpha, void* stream);

/* ---------------------------------------------------------------------------
 * Full gradient G = dY^T X (m x n), Section 3.1.  This is what dense-projection
 * methods compute every step ("mbn" FLOPs, Appendix F) and what GRASS needs on a
 * refresh step to obtain row norms; it also serves as the naive comparator
 * (full G followed by a row gather).  G has dtype gdt (fp32 accumulation, one
 * rounding), leading dimension ldg.
 * Errors: NULL, SHAPE, DTYPE, WORKSPACE. */
size_t grass_dense_workspace(int64_t T, int64_t m, int64_t n, grass_dtype dt,
                             grass_dy_layout layout);
grass_status grass_dense_grad(const void* dY, grass_dy_layout layout, int64_t ldy, const void* X,
                              int64_t ldx, grass_dtype dt, int64_t T, int64_t m, int64_t n,
                              void* G, grass_dtype gdt, int64_t ldg, void* ws, size_t ws_bytes,
                              void* stream);

/* Refresh-step statistic in one pass (Section 3.2 needs only the row norms of G, and the
 * paper's memory table counts the full gradient as an intermittent cost of the projection
 * update): sumsq[k] = sum_i (sum_t dY[t,k] X[t,i])^2 without writing G to memory.  For
 * bf16 inputs in T x m layout with T a multiple of 32, m, n, ldy, ldx multiples of 8 and
 * 16-byte aligned bases, the squares are taken from the fp32 accumulators in the GEMM
 * epilogue and the workspace is a few hundred KB; other inputs form G in fp32 inside the
 * (then m*n*4 bytes larger) workspace and reduce it from there.  The query assumes aligned
 * bases; a call with misaligned bases and only the small workspace returns
 * GRASS_ERR_WORKSPACE.  Errors: NULL, SHAPE, DTYPE, WORKSPACE. */
size_t grass_grad_row_stats_workspace(int64_t T, int64_t m, int64_t n, grass_dtype dt,
                                      grass_dy_layout layout, int64_t ldy, int64_t ldx);
grass_status grass_grad_row_stats(const void* dY, grass_dy_layout layout, int64_t ldy,
                                  const void* X, int64_t ldx, grass_dtype dt, int64_t T, int64_t m,
                                  int64_t n, float* sumsq, void* ws, size_t ws_bytes,
                                  void* stream);

/* Row gather: out[j, :] = rho[j] * G[idx[j], :] (fp32 out, r x n, leading dimension ldo).
 * This is P^T G read from a stored full gradient: the second half of the naive comparator,
 * and the compressed gradient of a refresh step of Algorithm 1, where the full gradient has
 * just been formed for compute_P anyway (grass_dense_grad into an fp32 G, grass_row_stats,
 * grass_select_rows, this call, grass_adam_scatter: one matrix product for the whole step).
 * Errors: NULL, SHAPE, DTYPE. */
grass_status grass_gather_rows(const void* G, grass_dtype gdt, int64_t m, int64_t n, int64_t ldg,
                               const int32_t* idx, const float* rho, int64_t r, float* out,
                               int64_t ldo, void* stream);

/* ---------------------------------------------------------------------------
 * The regular step of Algorithm 1 in one call ("G_C <- P^T grad; Delta <- opt.update(G_C);
 * W <- W + alpha P Delta"), for `count` weight matrices that read the same activations X
 * (count = 1: one layer).  Per layer it computes exactly what grass_compressed_grad followed
 * by grass_adam_scatter_state computes; the split-K reduction of the matrix product, Adam and
 * the row update run as one kernel that reads the product's partial tiles directly, so G_C
 * is not written unless the layer asks for it (GC != NULL), and one launch and one pass over
 * r x n are saved per layer.
 *
 * `layers`: HOST array of `count` descriptors (1 <= count <= GRASS_MAX_GROUP); the pointers
 * inside are device pointers.  T, n, dt, layout, X, the moment dtype `sdt`, the weight dtype
 * `wdt`, the Adam scalars and alpha are shared.  `step_scalars`: NULL, or the device array of
 * grass_adam_step_scalars (lr and t are then ignored; for captured steps).
 * `ws` must hold grass_step_group_workspace(...) bytes.  ev_gemm_start / ev_gemm_stop: NULL, or
 * hipEvent_t handles recorded around the matrix-multiply kernel(s) as in
 * grass_compressed_grad_timed.
 * Errors: the union of those of the two calls it replaces. */
typedef struct {
    const void* dY;      /* T x m (or m x T), dtype dt                                   */
    int64_t ldy;
    int64_t m;           /* rows of W = features of dY                                   */
    int64_t r;           /* selected rows                                                */
    const int32_t* idx;  /* r ascending row indices                                      */
    const float* rho;    /* r scales                                                     */
    float* GC;           /* optional output, r x n fp32 (NULL: G_C is not stored)        */
    int64_t ldgc;        /* its leading dimension (ignored when GC is NULL)              */
    void* M;             /* r x n moments of dtype sdt, dense, updated in place          */
    void* V;
    void* W;             /* m x n weights of dtype wdt, updated in place                 */
    int64_t ldw;
} grass_step_layer;
size_t grass_step_group_workspace(int64_t T, int64_t n, int count, const int64_t* r,
                                  grass_dtype dt, grass_dy_layout layout);
grass_status grass_step_group(int count, const grass_step_layer* layers, grass_dy_layout layout,
                              const void* X, int64_t ldx, grass_dtype dt, int64_t T, int64_t n,
                              grass_dtype sdt, grass_dtype wdt, float lr, float beta1, float beta2,
                              float eps, int64_t t, const float* step_scalars, float alpha,
                              void* ws, size_t ws_bytes, void* stream, void* ev_gemm_start,
                              void* ev_gemm_stop);

/* grass_step_group with a second pair of timing hooks: ev_tail_start / ev_tail_stop (hipEvent_t
 * as void*, either may be NULL) receive the start and the end of the kernel that follows the
 * matrix multiply (split-K reduction + Adam + row update; with several layers, the launch that
 * serves them together, or the last layer's when the layers run one after the other), stamped
 * with that dispatch's own times.  For a benchmark that wants the step's tail as it runs inside
 * the step sequence.  Everything else is grass_step_group. */
grass_status grass_step_group_timed(int count, const grass_step_layer* layers,
                                    grass_dy_layout layout, const void* X, int64_t ldx,
                                    grass_dtype dt, int64_t T, int64_t n, grass_dtype sdt,
                                    grass_dtype wdt, float lr, float beta1, float beta2, float eps,
                                    int64_t t, const float* step_scalars, float alpha, void* ws,
                                    size_t ws_bytes, void* stream, void* ev_gemm_start,
                                    void* ev_gemm_stop, void* ev_tail_start, void* ev_tail_stop);

/* The regular step in column form, in one call (Section 4.1 projects the smaller dimension of
 * G; for a layer with m > n that is the input dimension, so r of the n COLUMNS of W are
 * trained): with dY (T x m) and X (T x n), both stored with t as the row index,
 *   G_C = rho ((B X^T) dY)            r x m   (= (G P)^T, P the n x r projection),
 *   Adam on r x m moments M, V        (U = its output, r x m fp32),
 *   W[:, idx[j]] += alpha * rho[j] * U[j, :]^T.
 * Exactly what grass_compressed_grad (X in the place of dY and dY in the place of X),
 * grass_adam_rows_state and grass_scatter_update_cols compute one after the other; the
 * split-K reduction of the product and Adam run as one kernel that reads the product's
 * partial tiles.  idx: r column indices in [0, n), ascending; GC: NULL, or r x m fp32 (leading
 * dimension ldgc) to receive G_C; U: r x m fp32, contiguous, 16-byte aligned (scratch the
 * caller owns; holds Adam's output afterwards); W: m x n of dtype wdt, leading dimension ldw;
 * ws: grass_step_cols_workspace(...) bytes.  Errors: NULL, SHAPE, DTYPE, WORKSPACE. */
size_t grass_step_cols_workspace(int64_t T, int64_t m, int64_t n, int64_t r, grass_dtype dt);
grass_status grass_step_cols(const void* dY, int64_t ldy, const void* X, int64_t ldx,
                             grass_dtype dt, int64_t T, int64_t m, int64_t n, int64_t r,
                             const int32_t* idx, const float* rho, float* GC, int64_t ldgc,
                             void* M, void* V, grass_dtype sdt, float* U, void* W,
                             grass_dtype wdt, int64_t ldw, float lr, float beta1, float beta2,
                             float eps, int64_t t, float alpha, void* ws, size_t ws_bytes,
                             void* stream, void* ev_gemm_start, void* ev_gemm_stop);

/* ---------------------------------------------------------------------------
 * The fused Adam + update for callers that capture a step into a HIP graph and replay it.
 * Adam's step count t and the learning rate change every step, and a captured launch keeps
 * its arguments; here the three values that depend on them are read from device memory:
 *   step_scalars[0] = lr,  [1] = 1 / (1 - beta1^t),  [2] = 1 / (1 - beta2^t).
 * grass_adam_step_scalars computes them on the host (`scalars`: host array of 3 floats, the
 * same double-precision evaluation the other Adam calls use); the caller copies them to the
 * device array before each replay (from pinned memory with a copy that is part of the graph,
 * or with a copy ahead of it on the same stream).  Everything else is grass_adam_scatter_state.
 * Errors: as grass_adam_scatter_state; NULL for a missing array; SHAPE for t < 1. */
grass_status grass_adam_step_scalars(float lr, float beta1, float beta2, int64_t t,
                                     float* scalars);
grass_status grass_adam_scatter_replayable(const float* GC, int64_t ldgc, void* M, void* V,
                                           grass_dtype sdt, int64_t r, int64_t n, float beta1,
                                           float beta2, float eps, const float* step_scalars,
                                           void* W, grass_dtype wdt, int64_t m, int64_t ldw,
                                           const int32_t* idx, const float* rho, float alpha,
                                           void* stream);

/* ---------------------------------------------------------------------------
 * Test hooks.  The launchers choose their kernels from the shapes and alignments of a call;
 * tests need to reach every kernel with small inputs, so a process-wide override exists for
 * each such choice.  value 0 (the initial state) leaves the choice to the library.  The
 * overrides are read when a call or a workspace query plans its launches: change them only
 * while no other thread is inside the library, and query workspaces after setting them.
 *   GRASS_TEST_GEMM_TILE     128 or 256: the matrix-multiply tile (the large tile still falls
 *                            back to the small one where alignment rules it out)
 *   GRASS_TEST_FUSED_STATS   1: grass_grad_row_stats takes the squares in the GEMM epilogue
 *                            whenever the shape allows, not only when the tiles fill the machine
 *   GRASS_TEST_PACK_MXT      1: dY stored m x T goes through the packing pass instead of the
 *                            row-gathering GEMM
 *   GRASS_TEST_NO_PAIRS      1: the row-gathering GEMM loads one K tile per request
 *   GRASS_TEST_MAX_K_SLICES  k > 0: the token dimension is split into at most k slices
 *   GRASS_TEST_NO_NARROW_GATHER  1: narrow layers take the packed route like all others (forcing
 *                            the tile with GRASS_TEST_GEMM_TILE does the same)
 * Errors: DTYPE for an unknown option. */
typedef enum {
    GRASS_TEST_GEMM_TILE = 0,
    GRASS_TEST_FUSED_STATS = 1,
    GRASS_TEST_PACK_MXT = 2,
    GRASS_TEST_NO_PAIRS = 3,
    GRASS_TEST_MAX_K_SLICES = 4,
    GRASS_TEST_NO_NARROW_GATHER = 5
} grass_test_option;
grass_status grass_set_test_option(grass_test_option option, int value);

#ifdef __cplusplus
}
#endif
#endif /* GRASS_H */
