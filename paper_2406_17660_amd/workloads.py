"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random tensors; it contains none of the method's
arithmetic and is the one piece of code that both the GPU tests/benchmark and
the CPU oracle's tests use.

The paper trains LLaMA models (dimensions in its Table 9) on C4 token batches;
neither the data nor the weights are available here, so each configuration below
takes the paper's layer shapes and token-batch sizes and fills dY and X from
stated distributions.  Every tensor has its own seed:

    seed = BASE_SEED + 100000*config + 1000*layer + 10*step + tensor_code

with tensor_code 0 = dY, 1 = X, 2 = W, 3 = auxiliary (per-feature scales).
Values are drawn in fp32 with a torch generator on the requested device and then
rounded once to the configuration's dtype; whoever needs them on the host copies
those exact bits back.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import torch

BASE_SEED = 2406176600


@dataclass(frozen=True)
class Layer:
    name: str
    m: int  # output features = rows of W and of G
    n: int  # input features


@dataclass(frozen=True)
class Config:
    cid: int
    name: str
    layers: Tuple[Layer, ...]
    T: int
    r: int
    dtype: torch.dtype
    dy_law: str  # "normal1" | "normal0.1" | "lognormal_rows"
    x_law: str  # "normal" | "student_t3"
    method: str
    replacement: bool
    steps: int
    refresh_every: int
    alpha: float
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8


def _llama(hidden, inter):
    return (Layer("attn_qkvo", hidden, hidden), Layer("mlp_gate_up", inter, hidden),
            Layer("mlp_down", hidden, inter))


CONFIGS = {
    1: Config(1, "single-256 fp32", (Layer("linear", 256, 256),), 512, 16, torch.float32,
              "normal1", "normal", "topr", False, 1, 1, 1.0),
    2: Config(2, "llama-60m bf16", _llama(512, 1376), 65536, 128, torch.bfloat16,
              "normal0.1", "normal", "multi_norm", False, 10, 5, 0.25),
    3: Config(3, "llama-350m bf16", _llama(1024, 2736), 65536, 256, torch.bfloat16,
              "normal0.1", "student_t3", "topr", False, 20, 10, 0.25),
    4: Config(4, "llama-1b bf16", _llama(2048, 5461), 65536, 512, torch.bfloat16,
              "lognormal_rows", "normal", "multi_norm", True, 2, 2, 0.25),
    5: Config(5, "llama-7b/13b bf16",
              (Layer("7b_attn", 4096, 4096), Layer("7b_mlp_gate_up", 11008, 4096),
               Layer("13b_attn", 5120, 5120), Layer("13b_mlp_gate_up", 13824, 5120)),
              131072, 1024, torch.bfloat16, "normal0.1", "normal", "multi_norm", True, 20, 200,
              0.25),
}


def tensor_seed(config: int, layer: int, step: int, code: int) -> int:
    return BASE_SEED + 100000 * config + 1000 * layer + 10 * step + code


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _randn(shape, device, seed, chunk_rows=8192, dtype=torch.float32, scale=1.0, col_scale=None):
    """N(0, scale^2) values, drawn in fp32 chunk by chunk and stored as `dtype`."""
    g = _gen(device, seed)
    out = torch.empty(shape, dtype=dtype, device=device)
    rows = shape[0]
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        z = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=g, device=device,
                        dtype=torch.float32)
        if scale != 1.0:
            z.mul_(scale)
        if col_scale is not None:
            z.mul_(col_scale)
        out[r0:r1] = z.to(dtype)
    return out


def make_dY(cfg: Config, layer: int, step: int, device, T=None, m=None):
    """dY (T x m): the loss gradient with respect to the layer's outputs."""
    T = cfg.T if T is None else T
    m = cfg.layers[layer].m if m is None else m
    seed = tensor_seed(cfg.cid, layer, step, 0)
    if cfg.dy_law == "normal1":
        return _randn((T, m), device, seed, dtype=cfg.dtype)
    if cfg.dy_law == "normal0.1":  # variance 1e-2
        return _randn((T, m), device, seed, dtype=cfg.dtype, scale=0.1)
    if cfg.dy_law == "lognormal_rows":
        # per-output-feature scale s_k = exp(z_k): the row norms of G spread log-normally
        z = torch.randn((m,), generator=_gen(device, tensor_seed(cfg.cid, layer, 0, 3)),
                        device=device, dtype=torch.float32)
        return _randn((T, m), device, seed, dtype=cfg.dtype, scale=0.1, col_scale=torch.exp(z))
    raise ValueError(cfg.dy_law)


def make_X(cfg: Config, layer: int, step: int, device, T=None, n=None):
    """X (T x n): the layer's input activations."""
    T = cfg.T if T is None else T
    n = cfg.layers[layer].n if n is None else n
    seed = tensor_seed(cfg.cid, layer, step, 1)
    if cfg.x_law == "normal":
        return _randn((T, n), device, seed, dtype=cfg.dtype)
    if cfg.x_law == "student_t3":
        # t_3 = z / sqrt(chi2_3 / 3) has variance 3; divide by sqrt(3) for unit variance
        g = _gen(device, seed)
        out = torch.empty((T, n), dtype=cfg.dtype, device=device)
        for r0 in range(0, T, 8192):
            r1 = min(T, r0 + 8192)
            z = torch.randn((r1 - r0, n), generator=g, device=device)
            c = torch.randn((3, r1 - r0, n), generator=g, device=device).square_().sum(0)
            out[r0:r1] = (z / torch.sqrt(c / 3.0) / (3.0 ** 0.5)).to(cfg.dtype)
        return out
    raise ValueError(cfg.x_law)


def make_W(cfg: Config, layer: int, device, m=None, n=None):
    """W (m x n) ~ N(0, 0.02^2), the usual transformer initialisation."""
    m = cfg.layers[layer].m if m is None else m
    n = cfg.layers[layer].n if n is None else n
    return _randn((m, n), device, tensor_seed(cfg.cid, layer, 0, 2), dtype=cfg.dtype, scale=0.02)


# ------------------------------------------------------------------------------ whole blocks
# The seven linear layers of one LLaMA block (the paper trains all of them with GRASS), and
# which of them read the same activations.  Tensors use layer codes 50 + position so that
# they never collide with the per-layer configurations above.
def llama_block(hidden: int, inter: int):
    shapes = {"q": (hidden, hidden), "k": (hidden, hidden), "v": (hidden, hidden),
              "o": (hidden, hidden), "gate": (inter, hidden), "up": (inter, hidden),
              "down": (hidden, inter)}
    groups = [("q", "k", "v"), ("o",), ("gate", "up"), ("down",)]
    return shapes, groups


BLOCKS = {"7b": (4096, 11008), "13b": (5120, 13824), "1b": (2048, 5461), "350m": (1024, 2736),
          "60m": (512, 1376)}


def make_block_inputs(cfg: Config, shapes, groups, device, T=None, step=0):
    """dY per layer, X per group and W per layer for one block, drawn like cfg's layers
    (dY ~ N(0, 0.1^2), X ~ N(0, 1), W ~ N(0, 0.02^2))."""
    T = cfg.T if T is None else T
    names = list(shapes)
    dY = {name: _randn((T, shapes[name][0]), device, tensor_seed(cfg.cid, 50 + i, step, 0),
                       dtype=cfg.dtype, scale=0.1) for i, name in enumerate(names)}
    X = {tuple(g): _randn((T, shapes[g[0]][1]), device, tensor_seed(cfg.cid, 50 + i, step, 1),
                          dtype=cfg.dtype) for i, g in enumerate(groups)}
    W = {name: _randn(shapes[name], device, tensor_seed(cfg.cid, 50 + i, 0, 2), dtype=cfg.dtype,
                      scale=0.02) for i, name in enumerate(names)}
    return dY, X, W
