"""Algorithm 1 over the linear layers of one transformer block, and the step schedule around it.

Layers that read the same activations (query/key/value; gate/up) form a group whose compressed
gradients come from one library call, `grass_compressed_grad_group`.  The schedule is the host
side of Section 3.3 ("Updating the Optimizer State") and Appendix "Pretraining" details: the
projection is recomputed every K steps, the Adam moments may be zeroed at that point, and the
learning rate is warmed up again after every recomputation.  Only call order and scalar
bookkeeping live here; all array arithmetic is in the HIP library.
"""
import math
from dataclasses import dataclass

import torch

from . import grass
from .layer import AdamHyper, GrassLayer


@dataclass
class RewarmSchedule:
    """Learning rate at optimiser step t (0-based).

    global part: linear warm-up over `warmup` steps to `base_lr`, then cosine decay to
    `min_ratio * base_lr` at `total` steps (the pretraining recipe of the paper's appendix:
    1000 warm-up steps, decay to 10 %).
    local part: after every projection update (steps t = 0, K, 2K, ...) the rate is ramped
    again over `rewarm` steps.  The paper gives the length of that ramp (200 steps) but not
    its shape; a linear ramp (s + 1) / rewarm, s = steps since the update, is used here.
    """
    base_lr: float = 1e-3
    warmup: int = 1000
    total: int = 10000
    min_ratio: float = 0.1
    K: int = 200
    rewarm: int = 200

    def global_factor(self, t: int) -> float:
        if self.warmup > 0 and t < self.warmup:
            return (t + 1) / self.warmup
        span = max(self.total - self.warmup, 1)
        x = min(max(t - self.warmup, 0), span) / span
        return self.min_ratio + (1.0 - self.min_ratio) * 0.5 * (1.0 + math.cos(math.pi * x))

    def local_factor(self, t: int) -> float:
        if self.rewarm <= 0 or self.K <= 0:
            return 1.0
        return min(1.0, (t % self.K + 1) / self.rewarm)

    def lr(self, t: int) -> float:
        return self.base_lr * self.global_factor(t) * self.local_factor(t)

    def is_refresh(self, t: int) -> bool:
        return self.K > 0 and t % self.K == 0


class GrassBlock:
    """The GRASS-trained linear layers of one block.

    shapes: {name: (m, n)}; groups: list of tuples of names, each tuple sharing one X (and so
    one n).  A layer outside every tuple is a group of its own.  All layers select rows.
    """

    def __init__(self, shapes, groups, r, T, dtype, method="topr", replacement=False,
                 scale=grass.SCALE_PAPER, alpha=0.25, adam=None, seed=0, device="cuda",
                 reset_state=True, layout=grass.DY_TxM, concurrent_groups=False, store_GC=True):
        # concurrent_groups: issue every group on a HIP stream of its own (default priority),
        # forked from and joined back into the caller's stream.  The groups are independent
        # (own inputs, state and workspaces); small layers, whose kernels do not fill the
        # machine, then overlap instead of queueing behind each other's launch gaps and tails.
        self.streams = None
        self.concurrent_groups = concurrent_groups
        self.store_GC = store_GC  # False: the compressed gradients are never written out
        self.adam = adam or AdamHyper()
        self.reset_state = reset_state
        self.layout = layout  # storage of every dY handed to refresh() / step()
        named = [n for g in groups for n in g]
        assert len(set(named)) == len(named) and set(named) <= set(shapes)
        self.groups = [tuple(g) for g in groups] + [(n,) for n in shapes if n not in named]
        self.layers = {}
        for k, (name, (m, n)) in enumerate(shapes.items()):
            self.layers[name] = GrassLayer(m, n, min(r, m), T, dtype, method, replacement, scale,
                                           alpha, self.adam, seed + k, device=device, layout=layout)
        self.ws = {}
        dt = grass.F32 if dtype == torch.float32 else grass.BF16
        for g in self.groups:
            ns = {self.layers[name].n for name in g}
            assert len(ns) == 1, "layers of a group read the same activations"
            rs = [self.layers[name].r for name in g]
            self.ws[g] = grass.workspace(grass.step_group_workspace(T, ns.pop(), rs, dt, layout),
                                         device)
        self.t = 0
        self.graph = None
        self.G32 = self.ws_dense = None  # refresh_step(): allocated on first use

    def refresh(self, dY, X, statistics=None):
        """compute_P (+ update_state) for every layer.  dY: {name: tensor}, X: {group: tensor};
        statistics: optional {name: fp32 device array} of row statistics to select from in
        place of a layer's own (see GrassLayer.refresh)."""
        for g in self.groups:
            for name in g:
                self.layers[name].refresh(dY[name], X[g], reset_state=self.reset_state,
                                          statistic=(statistics or {}).get(name))

    def refresh_step(self, dY, X, W, lr=None, statistics=None):
        """The refresh step of every layer with one matrix product per layer (see
        GrassLayer.refresh_step): the full gradient of a layer is kept while P is computed and
        its selected rows are the compressed gradient of this step.  One fp32 buffer of the
        largest layer's size serves all layers in turn."""
        if self.G32 is None:
            dev = next(iter(W.values())).device
            ls = self.layers.values()
            self.G32 = torch.empty(max(l.m * l.n for l in ls), dtype=torch.float32, device=dev)
            self.ws_dense = grass.workspace(
                max(grass.dense_workspace(l.T, l.m, l.n, l.dt, l.layout) for l in ls), dev)
            for l in ls:
                l.share_refresh_buffers(self.G32, self.ws_dense)
        for g in self.groups:
            for name in g:
                l = self.layers[name]
                if lr is not None:
                    l.adam = AdamHyper(lr, self.adam.beta1, self.adam.beta2, self.adam.eps)
                l.refresh_step(dY[name], X[g], W[name], reset_state=self.reset_state,
                               statistic=(statistics or {}).get(name))

    def _step_group(self, g, dY, X, W, lr, step_scalars=None):
        """One library call for the group: grouped G_C, Adam and the row updates."""
        members = [self.layers[name] for name in g]
        for l in members:
            if lr is not None:
                l.adam = AdamHyper(lr, self.adam.beta1, self.adam.beta2, self.adam.eps)
            l.adam_t += 1
        a, t = members[0].adam, members[0].adam_t
        assert all(l.adam_t == t for l in members)
        grass.step_group([dY[name] for name in g], X[g], [l.idx for l in members],
                         [l.rho for l in members], [l.M for l in members], [l.V for l in members],
                         [W[name] for name in g], a.lr, a.beta1, a.beta2, a.eps, t, members[0].alpha,
                         self.ws[g], self.layout,
                         GCs=[l.GC for l in members] if self.store_GC else None,
                         step_scalars=step_scalars)

    def step(self, dY, X, W, lr=None, step_scalars=None):
        """One regular step of every layer: grouped G_C, then Adam and the row update."""
        if not self.concurrent_groups:
            for g in self.groups:
                self._step_group(g, dY, X, W, lr, step_scalars)
            return
        if self.streams is None:
            self.streams = [torch.cuda.Stream() for _ in self.groups]
        main = torch.cuda.current_stream()
        fork = torch.cuda.Event()
        fork.record(main)
        for g, side in zip(self.groups, self.streams):
            side.wait_event(fork)
            with torch.cuda.stream(side):
                self._step_group(g, dY, X, W, lr, step_scalars)
                joined = torch.cuda.Event()
                joined.record(side)
            main.wait_event(joined)

    def train_step(self, dY, X, W, schedule: RewarmSchedule, statistics=None):
        """Step t of Algorithm 1 under `schedule`: when t = 0 mod K the refresh step (P from
        the full gradient, whose selected rows are also this step's compressed gradient), else
        the regular step."""
        if schedule.is_refresh(self.t):
            self.refresh_step(dY, X, W, schedule.lr(self.t), statistics)
        elif self.graph is not None:
            self.replay(schedule.lr(self.t))
        else:
            self.step(dY, X, W, schedule.lr(self.t))
        self.t += 1

    # -- the regular step as a HIP graph ---------------------------------------------------
    def capture(self, dY, X, W, slots=64):
        """Capture one regular step over the tensors given (they, the state and the workspaces
        must stay where they are) into a HIP graph.  Afterwards train_step() replays it; the
        refresh steps stay eager (they rewrite idx and rho in place, which the graph reads).
        Run one eager step first so that every lazily created handle exists.

        The learning rate and Adam's bias corrections reach the kernels through a 3-float
        device array.  Each replay is preceded by a copy into it from a pinned host slot of its
        own (a ring of `slots`, each guarded by an event), so the host can run ahead of the GPU.
        """
        dev = next(iter(W.values())).device
        self.scalars = torch.zeros(3, dtype=torch.float32, device=dev)
        self.slots = [torch.zeros(3, dtype=torch.float32).pin_memory() for _ in range(slots)]
        self.slot_events = [None] * slots
        self.slot = 0
        saved = {name: l.adam_t for name, l in self.layers.items()}
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step(dY, X, W, None, self.scalars)
        for name, l in self.layers.items():  # the capture itself runs nothing
            l.adam_t = saved[name]
        self.graph = graph

    def replay(self, lr):
        ts = {l.adam_t for l in self.layers.values()}
        assert len(ts) == 1, "all layers of a block share Adam's step count"
        t = ts.pop() + 1
        k = self.slot
        if self.slot_events[k] is not None:
            self.slot_events[k].synchronize()  # the copy that last read this slot has run
        vals = grass.adam_step_scalars(lr, self.adam.beta1, self.adam.beta2, t)
        for i in range(3):
            self.slots[k][i] = vals[i]
        self.scalars.copy_(self.slots[k], non_blocking=True)
        ev = torch.cuda.Event()
        ev.record()
        self.slot_events[k] = ev
        self.slot = (k + 1) % len(self.slots)
        self.graph.replay()
        for l in self.layers.values():
            l.adam_t = t
