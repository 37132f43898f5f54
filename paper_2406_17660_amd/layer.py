"""Per-layer driver of Algorithm 1 (memory-efficient subspace optimisation) on top of the C ABI.

Owns the buffers one linear layer needs (idx, rho, Adam moments, compressed gradient,
workspaces) and issues the library calls in the order of Algorithm 1.  No arithmetic of the
method happens here: every step is a HIP kernel behind `grass.*`.
"""
from dataclasses import dataclass

import torch

from . import grass

METHODS = {"topr": grass.SEL_TOPR, "uniform": grass.SEL_UNIFORM,
           "multi_norm": grass.SEL_MULTI_NORM, "multi_norm2": grass.SEL_MULTI_NORM2}


@dataclass
class AdamHyper:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8


class GrassLayer:
    """State of one m x n linear layer trained with GRASS at rank r.

    refresh() is `compute_P` + `update_state` of Algorithm 1 (lines under "if t = 0 mod K");
    step() is the regular part (G_C, opt.update, W += alpha P Delta).

    side="rows" selects r of the m rows of W (output features).  side="cols" is the right-hand
    form for layers whose input dimension is the smaller one: r of the n columns are selected.
    It is the row form of the transposed layer (G^T = X^T dY), so the same library calls are
    used with dY and X exchanged; only the final update differs (columns of W).
    """

    def __init__(self, m, n, r, T, dtype, method="topr", replacement=False,
                 scale=grass.SCALE_PAPER, alpha=0.25, adam=None, seed=0, g_dtype=None,
                 layout=grass.DY_TxM, device="cuda", materialise_G=False, side="rows",
                 state_dtype=torch.float32, store_GC=True):
        assert side in ("rows", "cols")
        self.side = side
        self.w_shape = (m, n)
        if side == "cols":  # work on the transposed problem: "rows" of G^T, state r x m
            assert layout == grass.DY_TxM
            m, n = n, m
        self.m, self.n, self.r, self.T = m, n, r, T
        self.dtype = dtype
        self.dt = grass.F32 if dtype == torch.float32 else grass.BF16
        self.method, self.replacement, self.scale = METHODS[method], replacement, scale
        self.alpha, self.adam, self.seed, self.layout = alpha, adam or AdamHyper(), seed, layout
        self.g_dtype = g_dtype or dtype
        dev = device
        self.idx = torch.zeros(r, dtype=torch.int32, device=dev)
        self.rho = torch.ones(r, dtype=torch.float32, device=dev)
        # Adam moments: fp32, or bf16 (2 bytes per moment, rounded once per step)
        self.M = torch.zeros((r, n), dtype=state_dtype, device=dev)
        self.V = torch.zeros((r, n), dtype=state_dtype, device=dev)
        self.GC = torch.empty((r, n), dtype=torch.float32, device=dev)
        self.sumsq = torch.empty(m, dtype=torch.float32, device=dev)
        self.ws_sel = grass.workspace(grass.select_workspace(m, r, self.method, replacement), dev)
        # one workspace serves both the separate calls and the one-call step
        ws_bytes = max(grass.cgrad_workspace(T, m, n, r, self.dt, layout),
                       grass.step_group_workspace(T, n, [r], self.dt, layout))
        if side == "cols":  # (m, n are those of the transposed problem here)
            ws_bytes = max(ws_bytes, grass.step_cols_workspace(T, n, m, r, self.dt))
            self.U = torch.empty((r, n), dtype=torch.float32, device=dev)  # Adam's output
        self.ws_gemm = grass.workspace(ws_bytes, dev)
        self.store_GC = store_GC  # False: the one-call step does not write G_C at all
        self.ws_dense = None  # allocated on first refresh: only refresh steps need it
        self.G = None
        self.G32 = self.ws_dense32 = None  # refresh_step(): the kept full gradient
        self.ws_stats = None
        self.materialise_G = materialise_G
        self.adam_t = 0
        self.refresh_id = 0

    # -- refresh step -----------------------------------------------------------------
    def _operands(self, dY, X):
        return (X, dY) if self.side == "cols" else (dY, X)

    def full_gradient(self, dY, X):
        dY, X = self._operands(dY, X)
        if self.G is None:
            self.G = torch.empty((self.m, self.n), dtype=self.g_dtype, device=X.device)
            self.ws_dense = grass.workspace(
                grass.dense_workspace(self.T, self.m, self.n, self.dt, self.layout), X.device)
        return grass.dense_grad(dY, X, self.G, self.ws_dense, self.layout)

    def row_statistic(self, dY, X):
        """Squared row norms of G for compute_P.  By default G is not stored: the squares are
        taken in the GEMM epilogue; with materialise_G the two-call form (full gradient, then
        grass_row_stats) is used instead."""
        if self.materialise_G:
            self.full_gradient(dY, X)
            return grass.row_stats(self.G, self.sumsq)
        dY, X = self._operands(dY, X)
        if self.ws_stats is None:
            ldy, ldx = dY.stride(0), X.stride(0)
            self.ws_stats = grass.workspace(grass.grad_row_stats_workspace(
                self.T, self.m, self.n, self.dt, self.layout, ldy, ldx), X.device)
        return grass.grad_row_stats(dY, X, self.sumsq, self.ws_stats, self.layout)

    def refresh(self, dY, X, reset_state=True, statistic=None):
        """compute_P and update_state.  `statistic`: an fp32 device array of m squared row norms
        to select from in place of this layer's own (one that was reduced elsewhere, say summed
        over data-parallel workers); dY and X are then not read."""
        if statistic is None:
            self.row_statistic(dY, X)
        else:
            assert statistic.dtype == torch.float32 and tuple(statistic.shape) == (self.m,)
            if statistic is not self.sumsq:
                self.sumsq.copy_(statistic)
        grass.select_rows(self.sumsq, self.r, self.method, self.replacement, self.scale, self.seed,
                          self.refresh_id, self.idx, self.rho, self.ws_sel)
        self.refresh_id += 1
        if reset_state:  # update_state: moments back to zero, Adam's t restarts
            self.M.zero_()
            self.V.zero_()
            self.adam_t = 0

    def share_refresh_buffers(self, G32, ws_dense):
        """Use the caller's buffers for refresh_step(): G32 holds at least m * n fp32 values and
        ws_dense at least grass.dense_workspace(T, m, n, ...) bytes.  The layers of a block take
        their refresh steps one after the other and can share one pair."""
        assert G32.dtype == torch.float32 and G32.numel() >= self.m * self.n
        self.G32 = G32.reshape(-1)[:self.m * self.n].view(self.m, self.n)
        self.ws_dense32 = ws_dense

    def refresh_step(self, dY, X, W, reset_state=True, statistic=None):
        """A whole refresh step of Algorithm 1 with one matrix product: the full gradient is
        formed once (fp32, kept until the step ends), P is computed from its row norms, and
        the step's compressed gradient P^T G is read from that same G (rho[j] times row idx[j])
        instead of being recomputed from dY and X; Adam and the update of W follow as in a
        regular step.  Costs m * n * 4 bytes of scratch during refresh steps only.
        `statistic` as in refresh()."""
        dYo, Xo = self._operands(dY, X)
        if self.G32 is None:
            self.G32 = torch.empty((self.m, self.n), dtype=torch.float32, device=Xo.device)
            self.ws_dense32 = grass.workspace(
                grass.dense_workspace(self.T, self.m, self.n, self.dt, self.layout), Xo.device)
        grass.dense_grad(dYo, Xo, self.G32, self.ws_dense32, self.layout)
        if statistic is None:
            grass.row_stats(self.G32, self.sumsq)
        self.refresh(None, None, reset_state, self.sumsq if statistic is None else statistic)
        grass.gather_rows(self.G32, self.idx, self.rho, self.GC)
        return self.adam_scatter(W)

    # -- regular step -----------------------------------------------------------------
    def compressed_grad(self, dY, X, gemm_events=None):
        dY, X = self._operands(dY, X)
        return grass.compressed_grad(dY, X, self.idx, self.rho, self.GC, self.ws_gemm, self.layout,
                                     gemm_events)

    def adam_scatter(self, W, step_scalars=None):
        """Adam on the compressed gradient and the update of W.  With `step_scalars` (device
        array written by the caller from grass.adam_step_scalars) the launch does not depend on
        this step's learning rate and count and can be replayed from a captured graph."""
        self.adam_t += 1
        a = self.adam
        assert tuple(W.shape) == self.w_shape
        if step_scalars is not None:
            assert self.side == "rows"
            return grass.adam_scatter_replayable(self.GC, self.M, self.V, a.beta1, a.beta2, a.eps,
                                                 step_scalars, W, self.idx, self.rho, self.alpha)
        if self.side == "cols":  # Adam on r x m, then the update of r columns of W
            grass.adam_rows(self.GC, self.M, self.V, a.lr, a.beta1, a.beta2, a.eps, self.adam_t,
                            self.U)
            return grass.scatter_update_cols(W, self.idx, self.rho, self.alpha, self.U)
        return grass.adam_scatter(self.GC, self.M, self.V, a.lr, a.beta1, a.beta2, a.eps,
                                  self.adam_t, W, self.idx, self.rho, self.alpha)

    def step(self, dY, X, W, gemm_events=None, tail_events=None):
        """The regular step in one library call (grass_step_group, or grass_step_cols when
        columns are selected): the reduction of the product and Adam are one kernel, which
        for selected rows also updates W."""
        self.adam_t += 1
        a = self.adam
        assert tuple(W.shape) == self.w_shape
        if self.side == "cols":
            return grass.step_cols(dY, X, self.idx, self.rho, self.M, self.V, self.U, W, a.lr, a.beta1,
                                   a.beta2, a.eps, self.adam_t, self.alpha, self.ws_gemm,
                                   GC=self.GC if self.store_GC else None, gemm_events=gemm_events)
        grass.step_group([dY], X, [self.idx], [self.rho], [self.M], [self.V], [W], a.lr, a.beta1,
                         a.beta2, a.eps, self.adam_t, self.alpha, self.ws_gemm, self.layout,
                         GCs=[self.GC] if self.store_GC else None, gemm_events=gemm_events,
                         tail_events=tail_events)
