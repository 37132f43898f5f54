"""GPU parity of the block driver: layers that share activations are served by one grouped
compressed-gradient call, projections are recomputed every K steps with the Adam state zeroed,
and the learning rate follows the re-warm-up schedule.  Every layer is compared with the fp64
oracle run layer by layer."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2406_17660_amd import grass
from paper_2406_17660_amd.block import GrassBlock, RewarmSchedule
from paper_2406_17660_amd.layer import AdamHyper
from gpu_util import DEV, TOL_BF16, TOL_F32, check_own_selection, gpu_select, rel_fro, to_f64, to_np
from test_gpu_steps import OracleLayer, REF_METHOD

pytestmark = pytest.mark.gpu


def draw(shape, seed, scale=1.0):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return (torch.randn(shape, generator=g, device=DEV) * scale).to(torch.bfloat16)


@pytest.mark.parametrize("method,replacement,reset,layout,concurrent", [
    ("topr", False, True, grass.DY_TxM, False), ("multi_norm", False, False, grass.DY_TxM, False),
    ("multi_norm", True, True, grass.DY_TxM, True), ("multi_norm", True, True, grass.DY_MxT, False),
    ("topr", False, True, grass.DY_MxT, True)])
def test_block_training_steps_match_layerwise_oracle(method, replacement, reset, layout, concurrent):
    hidden, inter, T, r, K, steps = 128, 344, 640, 24, 3, 7
    shapes = {"q": (hidden, hidden), "k": (hidden, hidden), "v": (hidden, hidden),
              "o": (hidden, hidden), "gate": (inter, hidden), "up": (inter, hidden),
              "down": (hidden, inter)}
    groups = [("q", "k", "v"), ("gate", "up")]
    adam = AdamHyper(lr=1e-3)
    sched = RewarmSchedule(base_lr=2e-3, warmup=4, total=20, min_ratio=0.1, K=K, rewarm=3)
    blk = GrassBlock(shapes, groups, r, T, torch.bfloat16, method, replacement, alpha=0.25,
                     adam=adam, seed=77, reset_state=reset, layout=layout,
                     concurrent_groups=concurrent)
    W = {name: draw(s, 500 + i, 0.05) for i, (name, s) in enumerate(shapes.items())}
    W0 = {name: to_np(w).copy() for name, w in W.items()}
    orc = {name: OracleLayer(to_f64(W[name]), min(r, shapes[name][0]), REF_METHOD[method],
                             replacement, grass.SCALE_PAPER, 0.25, adam, 77 + i)
           for i, name in enumerate(shapes)}
    touched = {name: set() for name in shapes}
    assert set(blk.groups) == {("q", "k", "v"), ("gate", "up"), ("o",), ("down",)}
    for t in range(steps):
        X = {g: draw((T, shapes[g[0]][1]), 1000 + 10 * t + gi) for gi, g in enumerate(blk.groups)}
        dY = {name: draw((T, s[0]), 2000 + 10 * t + i, 0.1) for i, (name, s) in enumerate(shapes.items())}
        refreshed = sched.is_refresh(t)
        dY_dev = dY if layout == grass.DY_TxM else {k: v.t().contiguous() for k, v in dY.items()}
        stats = None
        if refreshed:
            # The GPU's own statistics are compared with the oracle's; the rows are then selected,
            # on both sides, from the oracle's statistics rounded once to fp32.
            stats, ref_ss = {}, {}
            for g in blk.groups:
                Xh = to_np(X[g])
                for name in g:
                    L = blk.layers[name]
                    ref_ss[name] = ref.row_stats(ref.full_grad(to_np(dY[name]), Xh))
                    L.row_statistic(dY_dev[name], X[g])
                    assert rel_fro(L.sumsq.cpu().numpy(), ref_ss[name]) <= TOL_F32, (name, t)
                    own, _, status = gpu_select(L.sumsq, L.r, L.method, L.replacement, L.scale,
                                                L.seed, L.refresh_id)
                    assert status == grass.OK
                    check_own_selection(own.cpu().numpy(), ref_ss[name], L.r, L.method, L.replacement)
                    stats[name] = torch.from_numpy(ref_ss[name].astype(np.float32)).to(DEV)
        blk.train_step(dY_dev, X, W, sched, statistics=stats)
        lr = sched.lr(t)
        for g in blk.groups:
            Xh = to_np(X[g])
            for name in g:
                L, o = blk.layers[name], orc[name]
                if refreshed:
                    o.refresh(ref_ss[name].astype(np.float32), reset=reset)
                    assert grass.select_status(L.ws_sel) == grass.OK
                    assert np.array_equal(L.idx.cpu().numpy(), o.idx), (name, t)
                    assert np.array_equal(L.rho.cpu().numpy(), o.rho)
                o.adam = AdamHyper(lr, adam.beta1, adam.beta2, adam.eps)
                o.step(to_np(dY[name]), Xh)
                touched[name].update(o.idx.tolist())
                assert rel_fro(to_f64(L.GC), o.GC) <= 2e-5, (name, t)
                assert rel_fro(to_f64(L.M), o.M) <= 1e-5 and rel_fro(to_f64(L.V), o.V) <= 1e-5
                assert L.adam_t == o.t
    expect_t = (steps - 1) % K + 1 if reset else steps
    assert all(l.adam_t == expect_t for l in blk.layers.values())
    for name, (m, n) in shapes.items():
        sel = np.array(sorted(touched[name]))
        got = to_f64(W[name])
        assert rel_fro(got[sel], orc[name].W[sel]) <= TOL_BF16
        rest = np.setdiff1d(np.arange(m), sel)
        assert np.array_equal(to_np(W[name])[rest], W0[name][rest])
        assert not np.array_equal(to_np(W[name])[sel], W0[name][sel])


@pytest.mark.parametrize("concurrent", [False, True])
def test_block_steps_replayed_from_a_graph_equal_eager_steps(concurrent):
    """The regular step captured once and replayed (learning rate and bias corrections fed
    through device memory), refresh steps eager in between: same bits as the all-eager run."""
    hidden, inter, T, r, K, steps = 128, 344, 640, 24, 3, 8
    shapes = {"q": (hidden, hidden), "k": (hidden, hidden), "v": (hidden, hidden),
              "o": (hidden, hidden), "gate": (inter, hidden), "up": (inter, hidden),
              "down": (hidden, inter)}
    groups = [("q", "k", "v"), ("gate", "up")]
    sched = RewarmSchedule(base_lr=2e-3, warmup=4, total=20, min_ratio=0.1, K=K, rewarm=3)

    def make():
        blk = GrassBlock(shapes, groups, r, T, torch.bfloat16, "multi_norm", True, alpha=0.25,
                         adam=AdamHyper(lr=1e-3), seed=9, concurrent_groups=concurrent)
        W = {name: draw(s, 600 + i, 0.05) for i, (name, s) in enumerate(shapes.items())}
        # inputs live in fixed buffers that are refilled every step (a graph replays addresses)
        X = {g: torch.empty((T, shapes[g[0]][1]), dtype=torch.bfloat16, device=DEV) for g in blk.groups}
        dY = {name: torch.empty((T, s[0]), dtype=torch.bfloat16, device=DEV) for name, s in shapes.items()}
        return blk, W, X, dY

    def fill(blk, X, dY, t):
        for gi, g in enumerate(blk.groups):
            X[g].copy_(draw(tuple(X[g].shape), 3000 + 10 * t + gi))
        for i, name in enumerate(shapes):
            dY[name].copy_(draw(tuple(dY[name].shape), 4000 + 10 * t + i, 0.1))

    eager, We, Xe, dYe = make()
    for t in range(steps):
        fill(eager, Xe, dYe, t)
        eager.train_step(dYe, Xe, We, sched)

    replayed, Wg, Xg, dYg = make()
    for t in range(steps):
        fill(replayed, Xg, dYg, t)
        replayed.train_step(dYg, Xg, Wg, sched)
        if t == 0:
            replayed.capture(dYg, Xg, Wg, slots=2)  # two slots: the ring wraps several times
    assert replayed.graph is not None
    torch.cuda.synchronize()
    for name in shapes:
        a, b = eager.layers[name], replayed.layers[name]
        assert a.adam_t == b.adam_t
        assert torch.equal(a.idx, b.idx) and torch.equal(a.M, b.M) and torch.equal(a.V, b.V), name
        assert torch.equal(We[name], Wg[name]), name
