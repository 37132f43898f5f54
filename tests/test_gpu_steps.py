"""GPU parity of whole GRASS steps (Algorithm 1) on the benchmark configurations.

Configurations 1-4 run with the paper-shaped layers but a shortened token batch so that the
fp64 oracle finishes in seconds; configuration 5 runs at full size in the launch
configuration bench.py times and is checked on sampled outputs.

Nothing the GPU computed is ever an input of the oracle.  On a refresh step the GPU's row
statistic is compared with the oracle's within tolerance; the rows are then selected, on both
sides, from the oracle's statistic rounded once to fp32 (the type the selection reads), and
must agree bit for bit.  What the GPU selects from its own statistic is checked for the
properties that hold whichever way a near-tie falls.
"""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2406_17660_amd import grass, workloads
from paper_2406_17660_amd.layer import AdamHyper, GrassLayer
from gpu_util import (DEV, TOL_BF16, TOL_F32, bf16_ulp, check_own_selection, gpu_select, rel_fro,
                      to_f64, to_np, tol_for)

pytestmark = pytest.mark.gpu
F = np.float32
REF_METHOD = {"topr": ref.TOPR, "uniform": ref.UNIFORM, "multi_norm": ref.MULTI_NORM,
              "multi_norm2": ref.MULTI_NORM2}


class OracleLayer:
    """The same Algorithm-1 bookkeeping as GrassLayer, but every step is the fp64 oracle."""

    def __init__(self, W0, r, method, replacement, scale, alpha, adam, seed, state_bf16=False):
        self.state_bf16 = state_bf16
        self.W = W0.copy()
        self.r, self.method, self.replacement, self.scale = r, method, replacement, scale
        self.alpha, self.adam, self.seed = alpha, adam, seed
        n = W0.shape[1]
        self.M = np.zeros((r, n))
        self.V = np.zeros((r, n))
        self.t = 0
        self.refresh_id = 0
        self.idx = self.rho = None

    def refresh(self, sumsq, reset=True):
        self.idx, self.rho, _ = ref.select_rows(sumsq, self.r, self.method, self.replacement,
                                                self.scale, self.seed, self.refresh_id)
        self.refresh_id += 1
        if reset:
            self.M[:] = 0
            self.V[:] = 0
            self.t = 0

    def step(self, dY, X):
        a = self.adam
        self.GC = ref.compressed_grad(dY, X, self.idx, self.rho)
        self.t += 1
        U = ref.adam_rows(self.GC, self.M, self.V, float(F(a.lr)), float(F(a.beta1)),
                          float(F(a.beta2)), float(F(a.eps)), self.t, state_bf16=self.state_bf16)
        ref.scatter_update(self.W, self.idx, self.rho, float(F(self.alpha)), U)


def run_config(cfg, layer, T, steps, refresh_every, method=None, replacement=None,
               scale=grass.SCALE_PAPER, g_dtype=None, materialise_G=False,
               state_dtype=torch.float32, one_product_refresh=False):
    L = cfg.layers[layer]
    method = method or cfg.method
    replacement = cfg.replacement if replacement is None else replacement
    adam = AdamHyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps)
    W = workloads.make_W(cfg, layer, DEV)
    W0_bits = to_np(W).copy()
    st = GrassLayer(L.m, L.n, cfg.r, T, cfg.dtype, method, replacement, scale, cfg.alpha, adam,
                    seed=workloads.BASE_SEED + layer, g_dtype=g_dtype, materialise_G=materialise_G,
                    state_dtype=state_dtype)
    orc = OracleLayer(to_f64(W), cfg.r, REF_METHOD[method], replacement, scale, cfg.alpha, adam,
                      workloads.BASE_SEED + layer, state_bf16=state_dtype == torch.bfloat16)
    tol = tol_for(cfg.dtype)
    touched = set()
    # Adam's update is ~ -lr * sign(g) early on, so an element of G_C that cancels to within
    # the fp32 accumulation error of zero has an ill-conditioned update (the oracle sees
    # -1.7e-6, fp32 sees 0).  Such elements are left out of the elementwise check of W only.
    well = np.ones((L.m, L.n), bool)
    for t in range(steps):
        dY = workloads.make_dY(cfg, layer, t, DEV, T=T)
        X = workloads.make_X(cfg, layer, t, DEV, T=T)
        dYh, Xh = to_np(dY), to_np(X)
        if t % refresh_every == 0:
            G = ref.full_grad(dYh, Xh)
            ref_ss = ref.row_stats(G)
            st.row_statistic(dY, X)  # the statistic as the GPU path takes it
            gpu_ss = st.sumsq.cpu().numpy()
            if materialise_G:
                assert rel_fro(to_f64(st.G), G) <= (TOL_BF16 if st.G.dtype == torch.bfloat16 else 2e-5)
                # of a G rounded to its stored type: the rounding errors (2^-9 relative, mean
                # zero) average out over the n squares of a row
                assert rel_fro(gpu_ss, ref_ss) <= min(tol, 1e-3)
            else:  # squares taken from the fp32 accumulators: G is never rounded to bf16
                assert st.G is None
                assert rel_fro(gpu_ss, ref_ss) <= TOL_F32
            own_idx, _, status = gpu_select(st.sumsq, st.r, st.method, st.replacement, st.scale,
                                            st.seed, st.refresh_id)
            assert status == grass.OK
            check_own_selection(own_idx.cpu().numpy(), ref_ss, st.r, st.method, st.replacement)
            # The rows are decided on one fp32 array on both sides: the oracle's statistic
            # rounded once to the type the selection reads (nothing the GPU computed goes into
            # the oracle).
            ss32 = ref_ss.astype(np.float32)
            if one_product_refresh:
                # the whole refresh step from one full gradient: its kept fp32 copy gives the
                # statistic's squares and, through the selected rows, this step's G_C
                st.refresh_step(dY, X, W, statistic=torch.from_numpy(ss32).to(DEV))
                assert rel_fro(to_f64(st.G32), G) <= 2e-5
            else:
                st.refresh(dY, X, statistic=torch.from_numpy(ss32).to(DEV))
            assert grass.select_status(st.ws_sel) == grass.OK
            orc.refresh(ss32)
            assert np.array_equal(st.idx.cpu().numpy(), orc.idx), f"rows differ at step {t}"
            assert np.array_equal(st.rho.cpu().numpy(), orc.rho)
        if not (one_product_refresh and t % refresh_every == 0):
            st.step(dY, X, W)
        orc.step(dYh, Xh)
        touched.update(orc.idx.tolist())
        shaky = np.abs(orc.GC) < 1e-4 * np.abs(orc.GC).mean(axis=1, keepdims=True)
        for j in np.nonzero(shaky.any(axis=1))[0]:
            well[orc.idx[j], shaky[j]] = False
        assert rel_fro(to_f64(st.GC), orc.GC) <= min(tol, 2e-5), f"G_C at step {t}"
        assert rel_fro(to_f64(st.M), orc.M) <= tol and rel_fro(to_f64(st.V), orc.V) <= tol
        assert st.adam_t == orc.t
    sel = np.array(sorted(touched))
    got = to_f64(W)
    assert rel_fro(got[sel], orc.W[sel]) <= tol
    if cfg.dtype == torch.bfloat16:
        # each step rounds W once (half an ulp of its current magnitude).  |U| <= 4 lr bounds
        # how far an element can have moved, hence the largest ulp it has been rounded at.
        W0 = to_f64(workloads.make_W(cfg, layer, DEV))[sel]
        row_scale = np.bincount(orc.idx, weights=orc.rho.astype(np.float64)).max()  # duplicates add up
        row_scale = max(row_scale, float(orc.rho.max()))
        reach = np.abs(W0) + steps * 4 * cfg.lr * cfg.alpha * row_scale
        ok = np.abs(got[sel] - orc.W[sel]) <= steps * bf16_ulp(reach)
        assert (ok | ~well[sel]).all()
        assert well[sel].mean() > 0.999
    else:
        assert rel_fro(got[sel] - to_f64(workloads.make_W(cfg, layer, DEV))[sel],
                       orc.W[sel] - to_f64(workloads.make_W(cfg, layer, DEV))[sel]) <= 1e-4
    rest = np.setdiff1d(np.arange(L.m), sel)
    assert np.array_equal(to_np(W)[rest], W0_bits[rest])
    return st, orc


def test_config1_fp32_single_layer_exact_size():
    """256 x 256, T = 512, r = 16, fp32, Top-r, Adam defaults, one step: the stated sizes."""
    cfg = workloads.CONFIGS[1]
    st, orc = run_config(cfg, 0, cfg.T, 1, 1, materialise_G=True)
    run_config(cfg, 0, cfg.T, 1, 1, materialise_G=False)


@pytest.mark.parametrize("layer", [0, 1, 2])
@pytest.mark.parametrize("scale", [grass.SCALE_PAPER, grass.SCALE_INV_SQRT_RQ])
def test_config2_llama60m_multinorm_nr(layer, scale):
    """bf16, r = 128, Multinomial-Norm without replacement; rho = 1 (the paper's rule) and the
    configuration's 1/sqrt(r q) rescaling; 10 steps, selection refreshed every 5.  One of the
    two runs stores G in bf16 on refresh steps, the other takes the statistic in the GEMM."""
    run_config(workloads.CONFIGS[2], layer, 2048, 10, 5, scale=scale,
               materialise_G=(scale == grass.SCALE_PAPER))


@pytest.mark.parametrize("config,layer,T", [(2, 0, 2048), (2, 2, 2048), (3, 1, 1024), (4, 2, 512)])
def test_refresh_step_from_one_full_gradient(config, layer, T):
    """Algorithm 1's refresh step with the full gradient formed once and kept: P from its row
    norms, the step's compressed gradient from its selected rows (no second product)."""
    cfg = workloads.CONFIGS[config]
    st, orc = run_config(cfg, layer, T=T, steps=7, refresh_every=3, one_product_refresh=True)
    # the statistic the kept gradient gives on its own (the run selected from the oracle's)
    dY = workloads.make_dY(cfg, layer, 6, DEV, T=T)
    X = workloads.make_X(cfg, layer, 6, DEV, T=T)
    W = workloads.make_W(cfg, layer, DEV)
    st.refresh_step(dY, X, W)
    ref_ss = ref.row_stats(ref.full_grad(to_np(dY), to_np(X)))
    assert rel_fro(st.sumsq.cpu().numpy(), ref_ss) <= TOL_F32
    check_own_selection(st.idx.cpu().numpy(), ref_ss, st.r, st.method, st.replacement)


@pytest.mark.parametrize("layer", [0, 2])
def test_config2_with_bf16_adam_moments(layer):
    """The same steps with the moments kept in bf16 (2 bytes each), rounded once per step."""
    st, _ = run_config(workloads.CONFIGS[2], layer, 2048, 6, 3, state_dtype=torch.bfloat16)
    assert st.M.dtype == torch.bfloat16 and st.V.dtype == torch.bfloat16


@pytest.mark.parametrize("layer", [0, 1, 2])
def test_config3_llama350m_heavy_tailed_topr(layer):
    """bf16, r = 256, Top-r, Student-t(3) activations; refresh in the middle of the run."""
    run_config(workloads.CONFIGS[3], layer, 1024, 4, 2)


@pytest.mark.parametrize("layer", [0, 1, 2])
@pytest.mark.parametrize("method,replacement", [("uniform", True), ("multi_norm", True),
                                                ("uniform", False), ("multi_norm", False)])
def test_config4_llama1b_lognormal_rows(layer, method, replacement):
    """bf16, r = 512, log-normal spread of the row norms; with-replacement draws give duplicate
    rows; the 5461-wide layers have rows that are not 16-byte aligned."""
    st, orc = run_config(workloads.CONFIGS[4], layer, 512, 2, 2, method, replacement)
    if replacement and method == "multi_norm":
        assert len(np.unique(orc.idx)) < len(orc.idx)  # the heavy rows are drawn repeatedly


def test_config4_norm_sampling_prefers_heavy_rows():
    """Sanity of the workload itself: norm-proportional draws pick rows of larger norm."""
    cfg = workloads.CONFIGS[4]
    st, orc = run_config(cfg, 0, 512, 1, 1, "multi_norm", True)
    ss = st.sumsq.cpu().numpy()
    assert np.sqrt(ss[orc.idx]).mean() > 1.5 * np.sqrt(ss).mean()


# ------------------------------------------------------------------------------ full size, sampled
@pytest.mark.parametrize("layer", [0, 1])
def test_config5_full_size_sampled(layer):
    """7B-shaped layers at T = 131072, r = 1024, exactly as bench.py launches them.  The oracle
    cannot form the whole gradient at this size, so: the GPU's row statistic is checked on
    sampled rows; the rows are selected, on both sides, from a seeded statistic of the spread the
    real one has; the compressed gradient, the moments and the updated weights are checked on a
    lattice of entries the oracle computes from the inputs alone; Adam and the row update are
    also checked in full on a seeded compressed gradient."""
    cfg = workloads.CONFIGS[5]
    L = cfg.layers[layer]
    T, m, n, r = cfg.T, L.m, L.n, cfg.r
    dY = workloads.make_dY(cfg, layer, 0, DEV)
    X = workloads.make_X(cfg, layer, 0, DEV)
    W = workloads.make_W(cfg, layer, DEV)
    W0 = to_f64(W)
    W0_bits = to_np(W).copy()
    adam = AdamHyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps)
    stored = layer == 0  # one layer with the two-call refresh (G stored), one with the fused one
    st = GrassLayer(m, n, r, T, cfg.dtype, cfg.method, cfg.replacement, alpha=cfg.alpha, adam=adam,
                    seed=workloads.BASE_SEED, materialise_G=stored)
    Xh = to_np(X)

    # refresh step: full gradient and its row statistic on sampled rows
    st.row_statistic(dY, X)
    rng = np.random.default_rng(5 + layer)
    rows = np.sort(rng.choice(m, 6, replace=False))
    dY_rows = to_np(dY[:, torch.from_numpy(rows).to(DEV)].contiguous())
    G_rows = ref.full_grad(dY_rows, Xh)
    gpu_ss = st.sumsq.cpu().numpy()
    if stored:
        assert rel_fro(to_f64(st.G[torch.from_numpy(rows).to(DEV)]), G_rows) <= TOL_BF16
        assert rel_fro(gpu_ss[rows], ref.row_stats(G_rows)) <= TOL_BF16
    else:
        assert st.G is None
        assert rel_fro(gpu_ss[rows], ref.row_stats(G_rows)) <= TOL_F32
    # every row of G is a sum of T n independent products of variance 1e-2: the statistic is
    # T n / 100 up to a relative spread of sqrt(2 / n)
    assert np.abs(gpu_ss / (T * n * 1e-2) - 1).max() < 8 * np.sqrt(2.0 / n) + 0.05

    # selection at full size: a seeded statistic with that mean and spread, the same array on
    # both sides
    ss = (T * n * 1e-2 * (1 + np.sqrt(2.0 / n) * rng.standard_normal(m))).astype(np.float32)
    st.refresh(dY, X, statistic=torch.from_numpy(ss).to(DEV))
    idx, rho, _ = ref.select_rows(ss, r, REF_METHOD[cfg.method], cfg.replacement,
                                  ref.SCALE_PAPER, workloads.BASE_SEED, 0)
    st.step(dY, X, W)
    torch.cuda.synchronize()
    assert grass.select_status(st.ws_sel) == grass.OK
    assert np.array_equal(st.idx.cpu().numpy(), idx)
    assert np.array_equal(st.rho.cpu().numpy(), rho)

    # compressed gradient on a lattice that touches every tile.  The lattice takes whole runs
    # of equal rows (draws with replacement repeat rows), so that the update of a sampled row of
    # W can be formed from the lattice alone.
    picked = np.unique(idx[np.arange(7, r, 53)])
    js = np.nonzero(np.isin(idx, picked))[0]
    cols = np.arange(11, n, 173)
    sel_cols = torch.from_numpy(idx[js].astype(np.int64)).to(DEV)
    dY_sel = to_np(dY[:, sel_cols].contiguous())
    want = ref.compressed_grad(dY_sel, np.ascontiguousarray(Xh[:, cols]),
                               np.arange(len(js), dtype=np.int32), rho[js])
    got = to_f64(st.GC)[np.ix_(js, cols)]
    assert rel_fro(got, want) <= 2e-5
    assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()

    # Adam and the row update on the same lattice, from the oracle's own compressed gradient
    M = np.zeros_like(want)
    V = np.zeros_like(want)
    U = ref.adam_rows(want, M, V, float(F(cfg.lr)), float(F(cfg.beta1)), float(F(cfg.beta2)),
                      float(F(cfg.eps)), 1)
    assert rel_fro(to_f64(st.M)[np.ix_(js, cols)], M) <= 2e-5
    assert rel_fro(to_f64(st.V)[np.ix_(js, cols)], V) <= 2e-5
    Wo = np.ascontiguousarray(W0[:, cols])
    ref.scatter_update(Wo, idx[js], rho[js], float(F(cfg.alpha)), U)
    gotW = to_f64(W)
    assert rel_fro(gotW[np.ix_(picked, cols)], Wo[picked]) <= TOL_BF16
    # an element of G_C that cancels to (nearly) zero has an ill-conditioned update (Adam's
    # first step is -lr sign(g)): those entries are left out of the elementwise bound
    shaky = np.zeros((m, len(cols)), bool)
    for j, row in zip(js, np.abs(want) < 1e-4 * np.abs(want).mean(axis=1, keepdims=True)):
        shaky[idx[j]] |= row
    slack = 4 * 2.0 ** -24 * (np.abs(W0[np.ix_(picked, cols)]) + np.abs(Wo[picked] - W0[np.ix_(picked, cols)]))
    ok = np.abs(gotW[np.ix_(picked, cols)] - Wo[picked]) <= 0.501 * bf16_ulp(Wo[picked]) + slack
    assert (ok | shaky[picked]).all() and shaky[picked].mean() < 0.02
    sel = np.unique(idx)
    rest = np.setdiff1d(np.arange(m), sel)
    assert np.array_equal(to_np(W)[rest], W0_bits[rest])
    assert not np.array_equal(to_np(W)[sel], W0_bits[sel])

    # bench.py's own launch configuration: the one-call step that never writes G_C.  Same
    # kernels minus one store, so state and weights must equal the run above bit for bit.
    st2 = GrassLayer(m, n, r, T, cfg.dtype, cfg.method, cfg.replacement, alpha=cfg.alpha, adam=adam,
                     seed=workloads.BASE_SEED, store_GC=False)
    W2 = workloads.make_W(cfg, layer, DEV)
    st2.GC.fill_(float("nan"))
    st2.refresh(dY, X, statistic=torch.from_numpy(ss).to(DEV))
    st2.step(dY, X, W2)
    assert torch.equal(st2.idx, st.idx) and torch.equal(st2.rho, st.rho)
    assert torch.equal(st2.M, st.M) and torch.equal(st2.V, st.V) and torch.equal(W2, W)
    assert bool(torch.isnan(st2.GC).all())  # and G_C was indeed not stored
    del st2, W2

    # bench.py's refresh step: the full gradient formed once and kept in fp32, the rows selected
    # from the same seeded statistic, G_C read from the selected rows of the kept gradient.
    # Against the oracle's values of the lattice above (from the inputs alone).
    st3 = GrassLayer(m, n, r, T, cfg.dtype, cfg.method, cfg.replacement, alpha=cfg.alpha, adam=adam,
                     seed=workloads.BASE_SEED)
    W3 = workloads.make_W(cfg, layer, DEV)
    st3.refresh_step(dY, X, W3, statistic=torch.from_numpy(ss).to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(st3.idx, st.idx) and torch.equal(st3.rho, st.rho) and st3.adam_t == 1
    assert rel_fro(to_f64(st3.G32[torch.from_numpy(rows).to(DEV)]), G_rows) <= 2e-5
    kept_ss = torch.empty(m, device=DEV)
    grass.row_stats(st3.G32, kept_ss)
    assert rel_fro(kept_ss.cpu().numpy()[rows], ref.row_stats(G_rows)) <= TOL_F32
    got3 = to_f64(st3.GC)[np.ix_(js, cols)]
    assert rel_fro(got3, want) <= 2e-5 and np.abs(got3 - want).max() <= 1e-4 * np.abs(want).max()
    assert rel_fro(to_f64(st3.M)[np.ix_(js, cols)], M) <= 2e-5
    assert rel_fro(to_f64(st3.V)[np.ix_(js, cols)], V) <= 2e-5
    gotW3 = to_f64(W3)
    ok = np.abs(gotW3[np.ix_(picked, cols)] - Wo[picked]) <= 0.501 * bf16_ulp(Wo[picked]) + slack
    assert (ok | shaky[picked]).all()
    assert np.array_equal(to_np(W3)[rest], W0_bits[rest])
    del st3, W3, kept_ss

    # Adam and the row update in full at this size, on a seeded compressed gradient
    g = torch.Generator(device=DEV)
    g.manual_seed(workloads.BASE_SEED + 77 + layer)
    GC = torch.randn((r, n), generator=g, device=DEV) * 3.0
    Mg = torch.zeros((r, n), device=DEV)
    Vg = torch.zeros((r, n), device=DEV)
    Wg = workloads.make_W(cfg, layer, DEV)
    grass.adam_scatter(GC, Mg, Vg, cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, 1, Wg, st.idx, st.rho,
                       cfg.alpha)
    M = np.zeros((r, n))
    V = np.zeros((r, n))
    U = ref.adam_rows(to_f64(GC), M, V, float(F(cfg.lr)), float(F(cfg.beta1)), float(F(cfg.beta2)),
                      float(F(cfg.eps)), 1)
    Wo = W0.copy()
    ref.scatter_update(Wo, idx, rho, float(F(cfg.alpha)), U)
    gotW = to_f64(Wg)
    assert rel_fro(to_f64(Mg), M) <= TOL_F32 and rel_fro(to_f64(Vg), V) <= TOL_F32
    assert rel_fro(gotW[sel], Wo[sel]) <= TOL_BF16
    # one bf16 rounding (half an ulp), plus the fp32 rounding of the sum (matters where W and its
    # update cancel)
    slack = 4 * 2.0 ** -24 * (np.abs(W0[sel]) + np.abs(Wo[sel] - W0[sel]))
    assert (np.abs(gotW[sel] - Wo[sel]) <= 0.501 * bf16_ulp(Wo[sel]) + slack).all()
    assert np.array_equal(to_np(Wg)[rest], W0_bits[rest])


def test_config5_full_size_row_gathering_gemm_sampled():
    """The 7B attention layer with dY stored m x T (bench.py --layout mxt): the GEMM gathers the
    selected rows itself.  Sampled entries against the oracle, and the whole r x n result
    against the T x m path (same products, different summation order)."""
    cfg = workloads.CONFIGS[5]
    L = cfg.layers[0]
    T, m, n, r = cfg.T, L.m, L.n, cfg.r
    dY = workloads.make_dY(cfg, 0, 0, DEV)
    X = workloads.make_X(cfg, 0, 0, DEV)
    rng = np.random.default_rng(55)
    idx = np.sort(rng.choice(m, r, replace=True)).astype(np.int32)  # duplicates included
    rho = rng.uniform(0.5, 2.0, r).astype(np.float32)
    d_idx, d_rho = torch.from_numpy(idx).to(DEV), torch.from_numpy(rho).to(DEV)
    GC_t = torch.empty((r, n), device=DEV)
    ws = grass.workspace(grass.cgrad_workspace(T, m, n, r, grass.BF16, grass.DY_MxT))
    dYt = dY.t().contiguous()
    grass.compressed_grad(dYt, X, d_idx, d_rho, GC_t, ws, grass.DY_MxT)
    js = np.arange(3, r, 61)
    cols = np.arange(5, n, 191)
    sel_cols = torch.from_numpy(idx[js].astype(np.int64)).to(DEV)
    want = ref.compressed_grad(to_np(dY[:, sel_cols].contiguous()),
                               np.ascontiguousarray(to_np(X)[:, cols]),
                               np.arange(len(js), dtype=np.int32), rho[js])
    got = to_f64(GC_t)[np.ix_(js, cols)]
    assert rel_fro(got, want) <= 2e-5
    assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()
    del dYt
    GC = torch.empty((r, n), device=DEV)
    ws = grass.workspace(grass.cgrad_workspace(T, m, n, r, grass.BF16))
    grass.compressed_grad(dY, X, d_idx, d_rho, GC, ws)
    assert rel_fro(to_f64(GC_t), to_f64(GC)) <= 2e-6


# ------------------------------------------------------------------------------ column projection
@pytest.mark.parametrize("one_product_refresh", [False, True])
@pytest.mark.parametrize("method,replacement", [("topr", False), ("multi_norm", True)])
def test_column_projection_steps(method, replacement, one_product_refresh):
    """A gate/up-shaped layer (m > n) with the r selected COLUMNS of W trained: the row form of
    the transposed layer.  The oracle runs the same exchange and the column update."""
    from paper_2406_17660_amd.layer import GrassLayer
    T, m, n, r, steps = 1024, 688, 256, 64, 3
    adam = AdamHyper()
    g = torch.Generator(device=DEV)
    g.manual_seed(77)
    W = (torch.randn((m, n), generator=g, device=DEV) * 0.02).to(torch.bfloat16)
    W0 = to_f64(W).copy()
    W0_bits = to_np(W).copy()
    st = GrassLayer(m, n, r, T, torch.bfloat16, method, replacement, alpha=0.25, adam=adam, seed=5,
                    side="cols")
    M = np.zeros((r, m))
    V = np.zeros((r, m))
    Wo = W0.copy()
    touched = set()
    for t in range(steps):
        dY = (torch.randn((T, m), generator=g, device=DEV) * 0.1).to(torch.bfloat16)
        X = torch.randn((T, n), generator=g, device=DEV).to(torch.bfloat16)
        dYh, Xh = to_np(dY), to_np(X)
        if t == 0:
            st.row_statistic(dY, X)
            gpu_ss = st.sumsq.cpu().numpy()
            Gt = ref.full_grad(Xh, dYh)  # G^T = X^T dY, n x m: its rows are the columns of G
            np.testing.assert_allclose(Gt, ref.full_grad(dYh, Xh).T, rtol=1e-12, atol=1e-12)
            ref_ss = ref.row_stats(Gt)
            assert rel_fro(gpu_ss, ref_ss) <= TOL_F32
            own_idx, _, status = gpu_select(st.sumsq, r, st.method, replacement, st.scale, 5, 0)
            assert status == grass.OK
            check_own_selection(own_idx.cpu().numpy(), ref_ss, r, st.method, replacement)
            ss32 = ref_ss.astype(np.float32)  # both sides select from the oracle's statistic
            if one_product_refresh:  # G^T kept, its selected rows are this step's G_C
                st.refresh_step(dY, X, W, statistic=torch.from_numpy(ss32).to(DEV))
                assert rel_fro(to_f64(st.G32), Gt) <= 2e-5
            else:
                st.refresh(dY, X, statistic=torch.from_numpy(ss32).to(DEV))
            assert grass.select_status(st.ws_sel) == grass.OK
            idx, rho, _ = ref.select_rows(ss32, r, REF_METHOD[method], replacement,
                                          ref.SCALE_PAPER, 5, 0)
            assert np.array_equal(st.idx.cpu().numpy(), idx)
            assert np.array_equal(st.rho.cpu().numpy(), rho)
        if not (one_product_refresh and t == 0):
            st.step(dY, X, W)
        GC = ref.compressed_grad(Xh, dYh, idx, rho)  # r x m
        assert rel_fro(to_f64(st.GC), GC) <= 2e-5
        U = ref.adam_rows(GC, M, V, float(F(adam.lr)), float(F(adam.beta1)), float(F(adam.beta2)),
                          float(F(adam.eps)), t + 1)
        ref.scatter_update_cols(Wo, idx, rho, float(F(0.25)), U)
        touched.update(idx.tolist())
        assert rel_fro(to_f64(st.M), M) <= TOL_BF16 and rel_fro(to_f64(st.V), V) <= TOL_BF16
    sel = np.array(sorted(touched))
    got = to_f64(W)
    assert rel_fro(got[:, sel], Wo[:, sel]) <= TOL_BF16
    rest = np.setdiff1d(np.arange(n), sel)
    assert np.array_equal(to_np(W)[:, rest], W0_bits[:, rest])
