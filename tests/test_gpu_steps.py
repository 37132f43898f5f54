"""GPU parity of whole GRASS steps (Algorithm 1) on the benchmark configurations.

Configurations 1-4 run with the paper-shaped layers but a shortened token batch so that the
fp64 oracle finishes in seconds; configuration 5 runs at full size in the launch
configuration bench.py times and is checked on sampled outputs.

Selection parity is per call: the oracle's compute_P is fed the row statistics the GPU
produced (same bits in, same rows out must hold exactly); the statistics themselves are
compared within tolerance.
"""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2406_17660_amd import grass, workloads
from paper_2406_17660_amd.layer import AdamHyper, GrassLayer
from gpu_util import DEV, TOL_BF16, TOL_F32, bf16_ulp, rel_fro, to_f64, to_np, tol_for

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

    def refresh(self, gpu_sumsq, reset=True):
        self.idx, self.rho, _ = ref.select_rows(gpu_sumsq, self.r, self.method, self.replacement,
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
               scale=grass.SCALE_PAPER, g_dtype=None, check_full_grad=True, materialise_G=False,
               state_dtype=torch.float32):
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
            st.refresh(dY, X)
            assert grass.select_status(st.ws_sel) == grass.OK
            gpu_ss = st.sumsq.cpu().numpy()
            if check_full_grad:
                G = ref.full_grad(dYh, Xh)
                if materialise_G:
                    assert rel_fro(to_f64(st.G), G) <= (TOL_BF16 if st.G.dtype == torch.bfloat16 else 2e-5)
                    assert rel_fro(gpu_ss, ref.row_stats(G)) <= tol
                    # the statistic of the matrix the GPU actually stored: fp32-accumulation accuracy
                    assert rel_fro(gpu_ss, ref.row_stats(to_np(st.G))) <= TOL_F32
                else:  # squares taken from the fp32 accumulators: G is never rounded to bf16
                    assert st.G is None
                    assert rel_fro(gpu_ss, ref.row_stats(G)) <= TOL_F32
            orc.refresh(gpu_ss)
            assert np.array_equal(st.idx.cpu().numpy(), orc.idx), f"rows differ at step {t}"
            assert np.array_equal(st.rho.cpu().numpy(), orc.rho)
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
    # end to end from the oracle's own fp64 statistics: same rows unless a near-tie decides
    dY = workloads.make_dY(cfg, 0, 0, DEV)
    X = workloads.make_X(cfg, 0, 0, DEV)
    ss = ref.row_stats(ref.full_grad(to_np(dY), to_np(X)))
    own, _, _ = ref.select_rows(ss.astype(np.float32), cfg.r, ref.TOPR)
    diff = set(own.tolist()) ^ set(orc.idx.tolist())
    if diff:
        kth = np.sort(ss)[-cfg.r]
        assert all(abs(ss[k] - kth) <= 1e-5 * kth for k in diff)


@pytest.mark.parametrize("layer", [0, 1, 2])
@pytest.mark.parametrize("scale", [grass.SCALE_PAPER, grass.SCALE_INV_SQRT_RQ])
def test_config2_llama60m_multinorm_nr(layer, scale):
    """bf16, r = 128, Multinomial-Norm without replacement; rho = 1 (the paper's rule) and the
    configuration's 1/sqrt(r q) rescaling; 10 steps, selection refreshed every 5.  One of the
    two runs stores G in bf16 on refresh steps, the other takes the statistic in the GEMM."""
    run_config(workloads.CONFIGS[2], layer, 2048, 10, 5, scale=scale,
               materialise_G=(scale == grass.SCALE_PAPER))


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
    st, orc = run_config(workloads.CONFIGS[4], layer, 512, 2, 2, method, replacement,
                         check_full_grad=(layer == 0))
    if replacement and method == "multi_norm":
        assert len(np.unique(orc.idx)) < len(orc.idx)  # the heavy rows are drawn repeatedly


def test_config4_norm_sampling_prefers_heavy_rows():
    """Sanity of the workload itself: norm-proportional draws pick rows of larger norm."""
    cfg = workloads.CONFIGS[4]
    st, orc = run_config(cfg, 0, 512, 1, 1, "multi_norm", True, check_full_grad=False)
    ss = st.sumsq.cpu().numpy()
    assert np.sqrt(ss[orc.idx]).mean() > 1.5 * np.sqrt(ss).mean()


# ------------------------------------------------------------------------------ full size, sampled
@pytest.mark.parametrize("layer", [0, 1])
def test_config5_full_size_sampled(layer):
    """7B-shaped layers at T = 131072, r = 1024, exactly as bench.py launches them.  The
    oracle evaluates sampled rows / entries; Adam and the scatter are checked in full."""
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
    st.refresh(dY, X)
    st.step(dY, X, W)
    torch.cuda.synchronize()
    assert grass.select_status(st.ws_sel) == grass.OK
    Xh = to_np(X)

    # refresh step: full gradient and its row statistic on sampled rows
    rng = np.random.default_rng(5 + layer)
    rows = np.sort(rng.choice(m, 6, replace=False))
    dY_rows = to_np(dY[:, torch.from_numpy(rows).to(DEV)].contiguous())
    G_rows = ref.full_grad(dY_rows, Xh)
    gpu_ss = st.sumsq.cpu().numpy()
    if stored:
        assert rel_fro(to_f64(st.G[torch.from_numpy(rows).to(DEV)]), G_rows) <= TOL_BF16
        assert rel_fro(gpu_ss[rows], ref.row_stats(G_rows)) <= TOL_BF16
        assert rel_fro(gpu_ss, ref.row_stats(to_np(st.G))) <= TOL_F32
    else:
        assert st.G is None
        assert rel_fro(gpu_ss[rows], ref.row_stats(G_rows)) <= TOL_F32

    # selection: same statistic in, same rows and scales out
    idx, rho, _ = ref.select_rows(gpu_ss, r, REF_METHOD[cfg.method], cfg.replacement,
                                  ref.SCALE_PAPER, workloads.BASE_SEED, 0)
    assert np.array_equal(st.idx.cpu().numpy(), idx)
    assert np.array_equal(st.rho.cpu().numpy(), rho)

    # compressed gradient on a lattice that touches every tile
    js = np.arange(7, r, 53)
    cols = np.arange(11, n, 173)
    sel_cols = torch.from_numpy(idx[js].astype(np.int64)).to(DEV)
    dY_sel = to_np(dY[:, sel_cols].contiguous())
    want = ref.compressed_grad(dY_sel, np.ascontiguousarray(Xh[:, cols]),
                               np.arange(len(js), dtype=np.int32), rho[js])
    got = to_f64(st.GC)[np.ix_(js, cols)]
    assert rel_fro(got, want) <= 2e-5
    assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()

    # Adam and scatter in full, fed with the compressed gradient the GPU produced
    GC = to_f64(st.GC)
    M = np.zeros((r, n))
    V = np.zeros((r, n))
    U = ref.adam_rows(GC, M, V, float(F(cfg.lr)), float(F(cfg.beta1)), float(F(cfg.beta2)),
                      float(F(cfg.eps)), 1)
    Wo = W0.copy()
    ref.scatter_update(Wo, idx, rho, float(F(cfg.alpha)), U)
    sel = np.unique(idx)
    gotW = to_f64(W)
    assert rel_fro(to_f64(st.M), M) <= TOL_F32 and rel_fro(to_f64(st.V), V) <= TOL_F32
    assert rel_fro(gotW[sel], Wo[sel]) <= TOL_BF16
    # one bf16 rounding, plus the fp32 rounding of the sum (matters where W and its update cancel)
    slack = 4 * 2.0 ** -24 * (np.abs(W0[sel]) + np.abs(Wo[sel] - W0[sel]))
    assert (np.abs(gotW[sel] - Wo[sel]) <= 1.01 * bf16_ulp(Wo[sel]) + slack).all()
    rest = np.setdiff1d(np.arange(m), sel)
    assert np.array_equal(to_np(W)[rest], W0_bits[rest])


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
@pytest.mark.parametrize("method,replacement", [("topr", False), ("multi_norm", True)])
def test_column_projection_steps(method, replacement):
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
            st.refresh(dY, X)
            assert grass.select_status(st.ws_sel) == grass.OK
            gpu_ss = st.sumsq.cpu().numpy()
            Gt = ref.full_grad(Xh, dYh)  # G^T = X^T dY, n x m: its rows are the columns of G
            np.testing.assert_allclose(Gt, ref.full_grad(dYh, Xh).T, rtol=1e-12, atol=1e-12)
            assert rel_fro(gpu_ss, ref.row_stats(Gt)) <= TOL_F32
            idx, rho, _ = ref.select_rows(gpu_ss, r, REF_METHOD[method], replacement,
                                          ref.SCALE_PAPER, 5, 0)
            assert np.array_equal(st.idx.cpu().numpy(), idx)
            assert np.array_equal(st.rho.cpu().numpy(), rho)
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
