"""numpy-facing wrapper of the CPU oracle (oracle/grass_ref.c).  TEST INFRASTRUCTURE ONLY.

Arrays are numpy; bf16 data is passed as its raw bits in a uint16 array (the same
bits the GPU consumes).  Results are float64 unless stated.  No arithmetic of the
method lives in this file: it only marshals arguments.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

TOPR, UNIFORM, MULTI_NORM, MULTI_NORM2 = 0, 1, 2, 3
SCALE_PAPER, SCALE_ONE, SCALE_INV_SQRT_RQ = 0, 1, 2
DY_TxM, DY_MxT = 0, 1
OK, ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_NONFINITE = 0, 1, 2, 3, 5

_lib = None


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle returned status {code}")
        self.code = code


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        L = C.CDLL(path)
        i64, vp, i32 = C.c_int64, C.c_void_p, C.c_int
        L.grass_ref_full_grad.argtypes = [vp, i32, i64, vp, i64, i32, i64, i64, i64, vp]
        L.grass_ref_row_stats.argtypes = [vp, i32, i64, i64, i64, vp]
        L.grass_ref_compressed_grad.argtypes = [vp, i32, i64, vp, i64, i32, i64, i64, i64, i64,
                                                vp, vp, vp]
        L.grass_ref_adam_rows.argtypes = [vp, i64, vp, vp, i64, i64, C.c_double, C.c_double,
                                          C.c_double, C.c_double, i64, vp]
        L.grass_ref_adam_rows_bf16state.argtypes = L.grass_ref_adam_rows.argtypes
        L.grass_ref_round_bf16.argtypes = [C.c_double]
        L.grass_ref_round_bf16.restype = C.c_double
        L.grass_ref_scatter_update.argtypes = [vp, i64, i64, i64, vp, vp, C.c_double, vp, i64]
        L.grass_ref_scatter_update_cols.argtypes = [vp, i64, i64, i64, vp, vp, C.c_double, vp, i64]
        L.grass_ref_philox4x32_10.argtypes = [vp, vp, vp]
        L.grass_ref_philox4x32_10.restype = None
        L.grass_ref_draw_word.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
        L.grass_ref_draw_word.restype = C.c_uint64
        L.grass_ref_mulhi64.argtypes = [C.c_uint64, C.c_uint64]
        L.grass_ref_mulhi64.restype = C.c_uint64
        L.grass_ref_sampling_weights.argtypes = [vp, i64, i32, vp]
        L.grass_ref_select_rows.argtypes = [vp, i64, i64, i32, i32, i32, C.c_uint64, C.c_uint64,
                                            vp, vp, vp]
        _lib = L
    return _lib


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    if a.dtype == np.float64:
        return 2
    raise TypeError(f"unsupported dtype {a.dtype}")


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _chk(code):
    if code != OK:
        raise OracleError(code)


def _mat(a):
    a = np.asarray(a)
    assert a.ndim == 2
    if a.size == 0 or a.shape[0] == 1:
        return np.ascontiguousarray(a), a.shape[1]
    assert a.strides[1] == a.itemsize, "row-major 2-D array expected"
    return a, a.strides[0] // a.itemsize


def full_grad(dY, X, layout=DY_TxM):
    dY, ldy = _mat(dY)
    X, ldx = _mat(X)
    assert _dt(dY) == _dt(X)
    T, n = X.shape
    m = dY.shape[1] if layout == DY_TxM else dY.shape[0]
    G = np.empty((m, n), np.float64)
    _chk(lib().grass_ref_full_grad(_p(dY), layout, ldy, _p(X), ldx, _dt(X), T, m, n, _p(G)))
    return G


def row_stats(G):
    G, ldg = _mat(G)
    m, n = G.shape
    out = np.empty(m, np.float64)
    _chk(lib().grass_ref_row_stats(_p(G), _dt(G), m, n, ldg, _p(out)))
    return out


def compressed_grad(dY, X, idx, rho, layout=DY_TxM):
    dY, ldy = _mat(dY)
    X, ldx = _mat(X)
    assert _dt(dY) == _dt(X)
    T, n = X.shape
    m = dY.shape[1] if layout == DY_TxM else dY.shape[0]
    idx = np.ascontiguousarray(idx, np.int32)
    rho = np.ascontiguousarray(rho, np.float32)
    r = idx.shape[0]
    GC = np.empty((r, n), np.float64)
    _chk(lib().grass_ref_compressed_grad(_p(dY), layout, ldy, _p(X), ldx, _dt(X), T, m, n, r,
                                         _p(idx), _p(rho), _p(GC)))
    return GC


def round_bf16(x):
    """Nearest bf16 value (ties to even) of every element, as float64."""
    x = np.ascontiguousarray(x, np.float64)
    f = lib().grass_ref_round_bf16
    return np.array([f(float(v)) for v in x.ravel()], np.float64).reshape(x.shape)


def adam_rows(GC, M, V, lr, beta1, beta2, eps, t, state_bf16=False):
    """Updates M and V (float64, C-contiguous) in place and returns U.  With state_bf16 the
    moments are rounded to bf16 before they are stored and used."""
    GC, ldgc = _mat(np.asarray(GC, np.float64))
    r, n = GC.shape
    assert M.dtype == np.float64 and V.dtype == np.float64
    assert M.shape == (r, n) and V.shape == (r, n)
    assert M.flags.c_contiguous and V.flags.c_contiguous
    U = np.empty((r, n), np.float64)
    fn = lib().grass_ref_adam_rows_bf16state if state_bf16 else lib().grass_ref_adam_rows
    _chk(fn(_p(GC), ldgc, _p(M), _p(V), r, n, float(lr), float(beta1), float(beta2), float(eps),
            int(t), _p(U)))
    return U


def scatter_update(W, idx, rho, alpha, U):
    """Updates W (float64) in place."""
    assert W.dtype == np.float64
    W, ldw = _mat(W)
    m, n = W.shape
    idx = np.ascontiguousarray(idx, np.int32)
    rho = np.ascontiguousarray(rho, np.float32)
    U = np.ascontiguousarray(U, np.float64)
    r = idx.shape[0]
    assert U.shape == (r, n)
    _chk(lib().grass_ref_scatter_update(_p(W), m, n, ldw, _p(idx), _p(rho), float(alpha), _p(U),
                                        r))
    return W


def scatter_update_cols(W, idx, rho, alpha, U):
    """Updates W (float64, m x n) in place: W[:, idx[j]] += alpha * rho[j] * U[j, :] (U is r x m)."""
    assert W.dtype == np.float64
    W, ldw = _mat(W)
    m, n = W.shape
    idx = np.ascontiguousarray(idx, np.int32)
    rho = np.ascontiguousarray(rho, np.float32)
    U = np.ascontiguousarray(U, np.float64)
    r = idx.shape[0]
    assert U.shape == (r, m)
    _chk(lib().grass_ref_scatter_update_cols(_p(W), m, n, ldw, _p(idx), _p(rho), float(alpha),
                                             _p(U), r))
    return W


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, np.uint32)
    key = np.ascontiguousarray(key, np.uint32)
    out = np.empty(4, np.uint32)
    lib().grass_ref_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def draw_word(seed, refresh_id, j):
    return int(lib().grass_ref_draw_word(seed, refresh_id, j))


def mulhi64(a, b):
    return int(lib().grass_ref_mulhi64(a, b))


def sampling_weights(sumsq, method):
    sumsq = np.ascontiguousarray(sumsq, np.float32)
    wq = np.empty(sumsq.shape[0], np.uint64)
    _chk(lib().grass_ref_sampling_weights(_p(sumsq), sumsq.shape[0], method, _p(wq)))
    return wq


def select_rows(sumsq, r, method, replacement=True, scale=SCALE_PAPER, seed=0, refresh_id=0):
    """Returns (idx int32[r], rho float32[r], rho_d float64[r])."""
    sumsq = np.ascontiguousarray(sumsq, np.float32)
    m = sumsq.shape[0]
    idx = np.empty(max(r, 0), np.int32)
    rho = np.empty(max(r, 0), np.float32)
    rho_d = np.empty(max(r, 0), np.float64)
    _chk(lib().grass_ref_select_rows(_p(sumsq), m, r, method, int(bool(replacement)), scale, seed,
                                     refresh_id, _p(idx), _p(rho), _p(rho_d)))
    return idx, rho, rho_d
