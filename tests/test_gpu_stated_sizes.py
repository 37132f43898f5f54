"""GPU parity at the sizes the benchmark configurations state: the layers of configurations 2,
3 and 4 at T = 65536 tokens and the 13B-shaped layers of configuration 5 at T = 131072, in the
launch configuration bench.py times (the one-call step).

The oracle cannot form a whole gradient at these sizes, so each test follows the scheme of the
7B test in test_gpu_steps.py: the GPU's row statistic is checked on sampled rows; the rows are
selected, on both sides, from one seeded statistic; the compressed gradient, the moments and the
updated weights are checked on a lattice of entries that the oracle computes from the inputs
alone (whole runs of repeated rows, so that a sampled row of W is determined by the lattice);
rows that were not selected must keep their bits.  Nothing the GPU computed enters the oracle.

At these token counts the launcher splits K into 5 to 94 slices for the small models (above 8
slices the tail of the step is the kernel that spreads the slices over its wavefronts) and into
3 for the 13B layers (80-tile rounds that do not fill the machine evenly); the plan query pins
that down.
"""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2406_17660_amd import grass, workloads
from paper_2406_17660_amd.layer import AdamHyper, GrassLayer
from gpu_util import DEV, TOL_BF16, TOL_F32, bf16_ulp, rel_fro, to_f64, to_np

pytestmark = pytest.mark.gpu
F = np.float32
REF_METHOD = {"topr": ref.TOPR, "uniform": ref.UNIFORM, "multi_norm": ref.MULTI_NORM,
              "multi_norm2": ref.MULTI_NORM2}


def seeded_statistic(law, T, n, m, rng):
    """A statistic with the mean and the spread the real one has, drawn on the host."""
    z = rng.standard_normal(m)
    if law == "flat":  # rows of G are sums of T n products of variance 1e-2
        return (T * n * 1e-2 * (1 + np.sqrt(2.0 / n) * z)).astype(np.float32)
    if law == "lognormal":  # per-feature scales exp(z_k): squared norms spread like exp(2 z_k)
        return (T * n * 1e-2 * np.exp(2.0 * z)).astype(np.float32)
    raise ValueError(law)


def lattice(idx, r, n, row_step, col_step):
    """Whole runs of equal rows every `row_step` compressed rows, every `col_step`-th column."""
    picked = np.unique(idx[np.arange(min(7, r - 1), r, row_step)])
    js = np.nonzero(np.isin(idx, picked))[0]
    cols = np.arange(min(11, n - 1), n, col_step)
    return picked, js, cols


def check_on_lattice(dY, Xh, idx, rho, picked, js, cols, GC, M, V, W, W0, cfg, m):
    """G_C (if stored), the moments and the updated rows of W on the lattice, against the oracle
    run on the inputs alone; Adam's first step from zero moments."""
    sel_cols = torch.from_numpy(idx[js].astype(np.int64)).to(DEV)
    dY_sel = to_np(dY[:, sel_cols].contiguous())
    want = ref.compressed_grad(dY_sel, np.ascontiguousarray(Xh[:, cols]),
                               np.arange(len(js), dtype=np.int32), rho[js])
    if GC is not None:
        got = to_f64(GC)[np.ix_(js, cols)]
        assert rel_fro(got, want) <= 2e-5
        assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()
    Mo = np.zeros_like(want)
    Vo = np.zeros_like(want)
    U = ref.adam_rows(want, Mo, Vo, float(F(cfg.lr)), float(F(cfg.beta1)), float(F(cfg.beta2)),
                      float(F(cfg.eps)), 1)
    assert rel_fro(to_f64(M)[np.ix_(js, cols)], Mo) <= 2e-5
    assert rel_fro(to_f64(V)[np.ix_(js, cols)], Vo) <= 2e-5
    Wo = np.ascontiguousarray(W0[:, cols])
    ref.scatter_update(Wo, idx[js], rho[js], float(F(cfg.alpha)), U)
    gotW = to_f64(W)[np.ix_(picked, cols)]
    assert rel_fro(gotW, Wo[picked]) <= TOL_BF16
    # an element of G_C that cancels to (nearly) zero has an ill-conditioned first Adam step
    # (-lr sign(g)): those entries are left out of the elementwise bound
    shaky = np.zeros((m, len(cols)), bool)
    for j, row in zip(js, np.abs(want) < 1e-4 * np.abs(want).mean(axis=1, keepdims=True)):
        shaky[idx[j]] |= row
    W0l = W0[np.ix_(picked, cols)]
    slack = 4 * 2.0 ** -24 * (np.abs(W0l) + np.abs(Wo[picked] - W0l))
    # one rounding to bf16: half an ulp of the result; `slack` covers the fp32 rounding of the sum
    # before it (which can also decide on which side of a rounding boundary the sum falls)
    ok = np.abs(gotW - Wo[picked]) <= 0.501 * bf16_ulp(Wo[picked]) + slack
    assert (ok | shaky[picked]).all() and shaky[picked].mean() < 0.02


def run_layer(cfg, layer, method, replacement, stat_law, min_slices, max_slices, check_stat=True,
              T=None):
    L = cfg.layers[layer]
    T, m, n, r = T or cfg.T, L.m, L.n, cfg.r
    tile, slices = grass.cgrad_plan(T, n, r, grass.BF16, m=m)
    assert min_slices <= slices <= max_slices, (tile, slices)
    assert (tile == 0) == (cfg.cid == 2 and layer == 0)  # the 60M 512 x 512 layers gather inside the GEMM
    dY = workloads.make_dY(cfg, layer, 0, DEV, T=T)
    X = workloads.make_X(cfg, layer, 0, DEV, T=T)
    W = workloads.make_W(cfg, layer, DEV)
    W0 = to_f64(W)
    W0_bits = to_np(W).copy()
    adam = AdamHyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps)
    st = GrassLayer(m, n, r, T, cfg.dtype, method, replacement, alpha=cfg.alpha, adam=adam,
                    seed=workloads.BASE_SEED + layer)
    Xh = to_np(X)
    rng = np.random.default_rng(100 * cfg.cid + layer)

    if check_stat:  # refresh step: the statistic of the full gradient on sampled rows
        st.row_statistic(dY, X)
        rows = np.sort(rng.choice(m, 4, replace=False))
        dY_rows = to_np(dY[:, torch.from_numpy(rows).to(DEV)].contiguous())
        G_rows = ref.full_grad(dY_rows, Xh)
        assert st.G is None
        assert rel_fro(st.sumsq.cpu().numpy()[rows], ref.row_stats(G_rows)) <= TOL_F32
        del dY_rows, G_rows

    ss = seeded_statistic(stat_law, T, n, m, rng)
    st.refresh(dY, X, statistic=torch.from_numpy(ss).to(DEV))
    idx, rho, _ = ref.select_rows(ss, r, REF_METHOD[method], replacement, ref.SCALE_PAPER,
                                  workloads.BASE_SEED + layer, 0)
    st.GC.fill_(float("nan"))
    st.step(dY, X, W)
    torch.cuda.synchronize()
    assert grass.select_status(st.ws_sel) == grass.OK
    assert np.array_equal(st.idx.cpu().numpy(), idx)
    assert np.array_equal(st.rho.cpu().numpy(), rho)
    assert not bool(torch.isnan(st.GC).any())

    picked, js, cols = lattice(idx, r, n, max(r // 37, 1), 61 if n > 2000 else 17)
    check_on_lattice(dY, Xh, idx, rho, picked, js, cols, st.GC, st.M, st.V, W, W0, cfg, m)
    sel = np.unique(idx)
    rest = np.setdiff1d(np.arange(m), sel)
    assert np.array_equal(to_np(W)[rest], W0_bits[rest])
    assert not np.array_equal(to_np(W)[sel], W0_bits[sel])

    # bench.py's launch configuration: the same step without storing G_C.  Same kernels minus
    # one store: state and weights equal the run above bit for bit.
    st2 = GrassLayer(m, n, r, T, cfg.dtype, method, replacement, alpha=cfg.alpha, adam=adam,
                     seed=workloads.BASE_SEED + layer, store_GC=False)
    W2 = workloads.make_W(cfg, layer, DEV)
    st2.GC.fill_(float("nan"))
    st2.refresh(dY, X, statistic=torch.from_numpy(ss).to(DEV))
    st2.step(dY, X, W2)
    assert torch.equal(st2.idx, st.idx) and torch.equal(st2.rho, st.rho)
    assert torch.equal(st2.M, st.M) and torch.equal(st2.V, st.V) and torch.equal(W2, W)
    assert bool(torch.isnan(st2.GC).all())
    return st, idx


@pytest.mark.parametrize("layer,slices", [(0, (65, 128)), (1, (65, 128)), (2, (33, 64))])
def test_config2_llama60m_layers_at_65536_tokens(layer, slices):
    """512 x 512, 1376 x 512, 512 x 1376 at r = 128, Multinomial-Norm without replacement: K is
    split into several dozen slices (both the 16-wavefront and the 8-wavefront form of the tail)."""
    run_layer(workloads.CONFIGS[2], layer, "multi_norm", False, "flat", *slices)


@pytest.mark.parametrize("layer,slices", [(0, (32, 64)), (1, (32, 64)), (2, (12, 32))])
def test_config3_llama350m_layers_at_65536_tokens(layer, slices):
    """1024 x 1024, 2736 x 1024, 1024 x 2736 at r = 256, Top-r, Student-t activations."""
    run_layer(workloads.CONFIGS[3], layer, "topr", False, "flat", *slices)


@pytest.mark.parametrize("layer,method,slices", [(0, "multi_norm", (9, 32)), (1, "uniform", (9, 32)),
                                                 (2, "multi_norm", (2, 16))])
def test_config4_llama1b_layers_at_65536_tokens(layer, method, slices):
    """2048 x 2048, 5461 x 2048, 2048 x 5461 at r = 512, draws with replacement from a log-normal
    spread of the row norms (long runs of repeated rows); the 5461-wide activations are copied to
    16-byte-aligned rows first, and rows of the 5461-long dY start at every byte offset."""
    st, idx = run_layer(workloads.CONFIGS[4], layer, method, True, "lognormal", *slices)
    if method == "multi_norm":
        assert len(np.unique(idx)) < 0.9 * len(idx)  # the heavy rows are drawn over and over


@pytest.mark.parametrize("layer", [2, 3])
def test_config5_llama13b_layers_at_131072_tokens(layer):
    """5120 x 5120 and 13824 x 5120 at r = 1024: 80 output tiles, three K slices; the 13824-long
    rows of dY are gathered one row per workgroup."""
    run_layer(workloads.CONFIGS[5], layer, "multi_norm", True, "flat", 2, 8)


@pytest.mark.parametrize("cid,slices", [(2, (32, 128)), (3, (9, 64)), (4, (2, 16))])
def test_query_key_value_group_at_65536_tokens(cid, slices):
    """The three attention projections that read the same activations, as one grass_step_group
    call at the configuration's token batch: one packed panel, one GEMM, one fused tail over the
    three sets.  Each set against the oracle on its own lattice."""
    cfg = workloads.CONFIGS[cid]
    L = cfg.layers[0]
    T, m, n, r = cfg.T, L.m, L.n, cfg.r
    total = 3 * ((r + 7) // 8 * 8)
    tile, k_slices = grass.cgrad_plan(T, n, total, grass.BF16, m=m, count=3)
    assert slices[0] <= k_slices <= slices[1], (tile, k_slices)
    assert (tile == 0) == (cid == 2)  # the 60M group gathers inside the GEMM (one launch, no panel)
    X = workloads.make_X(cfg, 0, 0, DEV)
    Xh = to_np(X)
    rng = np.random.default_rng(700 + cid)
    law = "lognormal" if cid == 4 else "flat"
    dYs, Ws, W0s, idxs, rhos, d_idx, d_rho = [], [], [], [], [], [], []
    for i in range(3):
        dYs.append(workloads.make_dY(cfg, 0, 1 + i, DEV))  # three different gradients
        W = workloads.make_W(cfg, 0, DEV)
        Ws.append(W)
        W0s.append((to_f64(W), to_np(W).copy()))
        ss = seeded_statistic(law, T, n, m, rng)
        idx, rho, _ = ref.select_rows(ss, r, REF_METHOD[cfg.method], cfg.replacement,
                                      ref.SCALE_PAPER, 11 + i, 0)
        idxs.append(idx); rhos.append(rho)
        d_idx.append(torch.from_numpy(idx).to(DEV)); d_rho.append(torch.from_numpy(rho).to(DEV))
    Ms = [torch.zeros((r, n), device=DEV) for _ in range(3)]
    Vs = [torch.zeros((r, n), device=DEV) for _ in range(3)]
    GCs = [torch.full((r, n), float("nan"), device=DEV) for _ in range(3)]
    ws = grass.workspace(grass.step_group_workspace(T, n, [r] * 3, grass.BF16))
    grass.step_group(dYs, X, d_idx, d_rho, Ms, Vs, Ws, cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, 1,
                     cfg.alpha, ws, GCs=GCs)
    torch.cuda.synchronize()
    for i in range(3):
        picked, js, cols = lattice(idxs[i], r, n, max(r // 23, 1), 41 if n > 1000 else 17)
        check_on_lattice(dYs[i], Xh, idxs[i], rhos[i], picked, js, cols, GCs[i], Ms[i], Vs[i], Ws[i],
                         W0s[i][0], cfg, m)
        rest = np.setdiff1d(np.arange(m), np.unique(idxs[i]))
        assert np.array_equal(to_np(Ws[i])[rest], W0s[i][1][rest])
    # without storing G_C (what the block driver of bench.py does): the same bits
    M2 = [torch.zeros((r, n), device=DEV) for _ in range(3)]
    V2 = [torch.zeros((r, n), device=DEV) for _ in range(3)]
    W2 = [workloads.make_W(cfg, 0, DEV) for _ in range(3)]
    grass.step_group(dYs, X, d_idx, d_rho, M2, V2, W2, cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, 1,
                     cfg.alpha, ws)
    for i in range(3):
        assert torch.equal(M2[i], Ms[i]) and torch.equal(V2[i], Vs[i]) and torch.equal(W2[i], Ws[i])
