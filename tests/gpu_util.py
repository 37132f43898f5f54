"""Helpers shared by the GPU parity tests: tensor <-> oracle conversions and error norms."""
import numpy as np
import torch

from oracle import ref
from paper_2406_17660_amd import grass

DEV = "cuda"
TOL_F32 = 1e-5   # relative Frobenius error, fp32 inputs
TOL_BF16 = 1e-2  # relative Frobenius error, bf16 inputs


def to_np(t: torch.Tensor) -> np.ndarray:
    """Host copy holding the same bits (bf16 becomes a uint16 array of bit patterns)."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def rel_fro(got, want) -> float:
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    denom = np.linalg.norm(want)
    err = np.linalg.norm(got - want)
    return float(err / denom) if denom > 0 else float(err)


def tol_for(dtype) -> float:
    return TOL_F32 if dtype == torch.float32 else TOL_BF16


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bf16 numbers around |x| (8 significand bits)."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


def gpu_select(sumsq, r, method, replacement, scale=grass.SCALE_PAPER, seed=0, refresh_id=0):
    m = sumsq.shape[0]
    idx = torch.full((r,), -1, dtype=torch.int32, device=DEV)
    rho = torch.full((r,), float("nan"), dtype=torch.float32, device=DEV)
    ws = grass.workspace(grass.select_workspace(m, r, method, replacement))
    grass.select_rows(sumsq, r, method, replacement, scale, seed, refresh_id, idx, rho, ws)
    return idx, rho, grass.select_status(ws)


def gpu_cgrad(dY, X, idx, rho, layout=grass.DY_TxM):
    T, n = X.shape
    m = dY.shape[1] if layout == grass.DY_TxM else dY.shape[0]
    r = idx.shape[0]
    GC = torch.full((r, n), float("nan"), dtype=torch.float32, device=DEV)
    dt = grass.F32 if X.dtype == torch.float32 else grass.BF16
    ws = grass.workspace(grass.cgrad_workspace(T, m, n, r, dt, layout))
    grass.compressed_grad(dY, X, idx, rho, GC, ws, layout)
    return GC


def gpu_dense(dY, X, gdtype, layout=grass.DY_TxM):
    T, n = X.shape
    m = dY.shape[1] if layout == grass.DY_TxM else dY.shape[0]
    G = torch.full((m, n), float("nan"), dtype=gdtype, device=DEV)
    dt = grass.F32 if X.dtype == torch.float32 else grass.BF16
    ws = grass.workspace(grass.dense_workspace(T, m, n, dt, layout))
    grass.dense_grad(dY, X, G, ws, layout)
    return G


def check_own_selection(idx, ref_ss, r, method, replacement):
    """What must hold for rows the GPU selected from its OWN statistic, which equals the oracle's
    `ref_ss` only up to fp32 rounding (so a near-tie may legitimately be decided differently):
    r rows, ascending, in range, distinct unless drawn with replacement, and for Top-r no
    unselected row clearly above a selected one."""
    idx = np.asarray(idx)
    m = len(ref_ss)
    assert idx.shape == (r,) and (np.diff(idx) >= 0).all()
    assert r == 0 or (idx.min() >= 0 and idx.max() < m)
    if method == grass.SEL_TOPR or not replacement:
        assert len(np.unique(idx)) == r
    if method == grass.SEL_TOPR and 0 < r < m:
        rest = np.setdiff1d(np.arange(m), idx)
        assert ref_ss[idx].min() >= ref_ss[rest].max() * (1 - 1e-5)
