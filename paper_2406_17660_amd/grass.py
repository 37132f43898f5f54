"""ctypes binding of libgrass.so (the C ABI of include/grass.h).

Argument marshalling only: every step of the method runs in the HIP kernels.  Tensors
are torch CUDA tensors (torch is used for device memory and streams, nothing else); each
function takes the same arguments as the C call of the same name, with pointers and
leading dimensions taken from the tensors and the stream taken from torch's current
stream.  A missing library is an error: there is no fallback path.
"""
import ctypes as C
import os

import torch  # imported before the library is loaded so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgrass.so")

OK, ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_WORKSPACE, ERR_NONFINITE, ERR_DEVICE = range(7)
F32, BF16 = 0, 1
SEL_TOPR, SEL_UNIFORM, SEL_MULTI_NORM, SEL_MULTI_NORM2 = 0, 1, 2, 3
SCALE_PAPER, SCALE_ONE, SCALE_INV_SQRT_RQ = 0, 1, 2
DY_TxM, DY_MxT = 0, 1
TEST_GEMM_TILE, TEST_FUSED_STATS, TEST_PACK_MXT, TEST_NO_PAIRS, TEST_MAX_K_SLICES = 0, 1, 2, 3, 4
TEST_NO_NARROW_GATHER = 5

EXPORTS = [
    "grass_status_string", "grass_row_stats", "grass_select_workspace", "grass_select_rows",
    "grass_cgrad_workspace", "grass_compressed_grad", "grass_compressed_grad_timed",
    "grass_adam_rows", "grass_scatter_update",
    "grass_adam_scatter", "grass_dense_workspace", "grass_dense_grad", "grass_gather_rows",
    "grass_grad_row_stats_workspace", "grass_grad_row_stats", "grass_scatter_update_cols",
    "grass_cgrad_group_workspace", "grass_compressed_grad_group",
    "grass_adam_rows_state", "grass_adam_scatter_state", "grass_cgrad_plan",
    "grass_set_test_option", "grass_select_static_capacity", "grass_select_rows_static",
    "grass_adam_step_scalars", "grass_adam_scatter_replayable",
    "grass_step_group_workspace", "grass_step_group", "grass_step_group_timed",
    "grass_step_cols_workspace", "grass_step_cols",
]

_lib = None


class StepLayer(C.Structure):
    """grass_step_layer of include/grass.h."""
    _fields_ = [("dY", C.c_void_p), ("ldy", C.c_int64), ("m", C.c_int64), ("r", C.c_int64),
                ("idx", C.c_void_p), ("rho", C.c_void_p), ("GC", C.c_void_p), ("ldgc", C.c_int64),
                ("M", C.c_void_p), ("V", C.c_void_p), ("W", C.c_void_p), ("ldw", C.c_int64)]


class GrassError(RuntimeError):
    def __init__(self, code, where):
        super().__init__(f"{where}: {status_string(code)} (status {code})")
        self.code = code


def lib():
    """Load libgrass.so (built by paper_2406_17660_amd/build.py); raise if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2406_17660_amd.build` "
            "(hipcc, gfx950).  There is no fallback implementation.")
    L = C.CDLL(LIB_PATH)
    i64, vp, i32, f32, u64, sz = C.c_int64, C.c_void_p, C.c_int, C.c_float, C.c_uint64, C.c_size_t
    L.grass_status_string.argtypes = [i32]
    L.grass_status_string.restype = C.c_char_p
    L.grass_row_stats.argtypes = [vp, i32, i64, i64, i64, vp, vp]
    L.grass_select_workspace.argtypes = [i64, i64, i32, i32]
    L.grass_select_workspace.restype = sz
    L.grass_select_rows.argtypes = [vp, i64, i64, i32, i32, i32, u64, u64, vp, vp, vp, sz, vp]
    L.grass_select_static_capacity.argtypes = []
    L.grass_select_static_capacity.restype = sz
    L.grass_select_rows_static.argtypes = [vp, i64, i64, i32, i32, i32, u64, u64, vp, vp, vp, vp]
    L.grass_cgrad_workspace.argtypes = [i64, i64, i64, i64, i32, i32]
    L.grass_cgrad_workspace.restype = sz
    L.grass_compressed_grad.argtypes = [vp, i32, i64, vp, i64, i32, i64, i64, i64, i64, vp, vp,
                                        vp, i64, vp, sz, vp]
    L.grass_compressed_grad_timed.argtypes = L.grass_compressed_grad.argtypes + [vp, vp]
    L.grass_adam_rows.argtypes = [vp, i64, vp, vp, i64, i64, f32, f32, f32, f32, i64, vp, vp]
    L.grass_scatter_update.argtypes = [vp, i32, i64, i64, i64, vp, vp, f32, vp, i64, vp]
    L.grass_scatter_update_cols.argtypes = L.grass_scatter_update.argtypes
    L.grass_adam_scatter.argtypes = [vp, i64, vp, vp, i64, i64, f32, f32, f32, f32, i64, vp, i32,
                                     i64, i64, vp, vp, f32, vp]
    L.grass_adam_rows_state.argtypes = [vp, i64, vp, vp, i32, i64, i64, f32, f32, f32, f32, i64, vp,
                                        vp]
    L.grass_adam_scatter_state.argtypes = [vp, i64, vp, vp, i32, i64, i64, f32, f32, f32, f32, i64,
                                           vp, i32, i64, i64, vp, vp, f32, vp]
    L.grass_adam_step_scalars.argtypes = [f32, f32, f32, i64, C.POINTER(C.c_float)]
    L.grass_adam_scatter_replayable.argtypes = [vp, i64, vp, vp, i32, i64, i64, f32, f32, f32, vp,
                                                vp, i32, i64, i64, vp, vp, f32, vp]
    L.grass_step_group_workspace.argtypes = [i64, i64, i32, vp, i32, i32]
    L.grass_step_group_workspace.restype = sz
    L.grass_step_group.argtypes = [i32, vp, i32, vp, i64, i32, i64, i64, i32, i32, f32, f32, f32,
                                   f32, i64, vp, f32, vp, sz, vp, vp, vp]
    L.grass_step_group_timed.argtypes = L.grass_step_group.argtypes + [vp, vp]
    L.grass_step_cols_workspace.argtypes = [i64, i64, i64, i64, i32]
    L.grass_step_cols_workspace.restype = sz
    L.grass_step_cols.argtypes = [vp, i64, vp, i64, i32, i64, i64, i64, i64, vp, vp, vp, i64, vp, vp,
                                  i32, vp, vp, i32, i64, f32, f32, f32, f32, i64, f32, vp, sz, vp,
                                  vp, vp]
    L.grass_dense_workspace.argtypes = [i64, i64, i64, i32, i32]
    L.grass_dense_workspace.restype = sz
    L.grass_dense_grad.argtypes = [vp, i32, i64, vp, i64, i32, i64, i64, i64, vp, i32, i64, vp,
                                   sz, vp]
    L.grass_gather_rows.argtypes = [vp, i32, i64, i64, i64, vp, vp, i64, vp, i64, vp]
    L.grass_grad_row_stats_workspace.argtypes = [i64, i64, i64, i32, i32, i64, i64]
    L.grass_grad_row_stats_workspace.restype = sz
    L.grass_grad_row_stats.argtypes = [vp, i32, i64, vp, i64, i32, i64, i64, i64, vp, vp, sz, vp]
    L.grass_cgrad_plan.argtypes = [i64, i64, i64, i64, i32, i32, i32, C.POINTER(C.c_int), C.POINTER(C.c_int)]
    L.grass_set_test_option.argtypes = [i32, i32]
    L.grass_cgrad_group_workspace.argtypes = [i64, i64, i32, vp, i32, i32]
    L.grass_cgrad_group_workspace.restype = sz
    L.grass_compressed_grad_group.argtypes = [i32, vp, i32, vp, vp, i64, i32, i64, vp, i64, vp,
                                              vp, vp, vp, vp, vp, sz, vp]
    for name in EXPORTS:
        if name not in ("grass_status_string", "grass_select_workspace", "grass_cgrad_workspace",
                        "grass_select_static_capacity",
                        "grass_dense_workspace", "grass_grad_row_stats_workspace",
                        "grass_cgrad_group_workspace", "grass_step_group_workspace",
                        "grass_step_cols_workspace"):
            getattr(L, name).restype = i32
    _lib = L
    return L


def status_string(code: int) -> str:
    return lib().grass_status_string(int(code)).decode()


def _check(code, where):
    if code != OK:
        raise GrassError(code, where)


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream():
    """Handle of torch's current stream on the current device (every call is issued there)."""
    if _raw_stream is not None:  # the same handle without building a Stream object per call
        return C.c_void_p(_raw_stream(torch.cuda.current_device()))
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _mat(t: torch.Tensor):
    """(pointer, rows, cols, leading dimension) of a row-major 2-D device tensor."""
    assert t.is_cuda and t.dim() == 2, "2-D CUDA tensor expected"
    rows, cols = t.shape
    if rows > 1 and cols > 0:
        assert cols == 1 or t.stride(1) == 1, "rows must be contiguous"
        ld = t.stride(0)
    else:
        ld = max(cols, 1) if t.stride(0) < cols else t.stride(0)
    return C.c_void_p(t.data_ptr()), rows, cols, ld


def _vec(t: torch.Tensor, dtype):
    assert t.is_cuda and t.dim() == 1 and t.dtype == dtype and t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def _ws(ws):
    if ws is None:
        return None, 0
    assert ws.is_cuda and ws.is_contiguous()
    return C.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def row_stats(G: torch.Tensor, sumsq: torch.Tensor):
    p, m, n, ld = _mat(G)
    assert sumsq.shape == (m,)
    _check(lib().grass_row_stats(p, _dtype(G), m, n, ld, _vec(sumsq, torch.float32), _stream()),
           "grass_row_stats")
    return sumsq


def select_workspace(m, r, method, replacement) -> int:
    return int(lib().grass_select_workspace(m, r, method, int(bool(replacement))))


def select_rows(sumsq, r, method, replacement, scale, seed, refresh_id, idx, rho, ws):
    m = sumsq.shape[0]
    assert idx.shape == (r,) and rho.shape == (r,)
    wp, wb = _ws(ws)
    _check(lib().grass_select_rows(_vec(sumsq, torch.float32), m, r, method,
                                   int(bool(replacement)), scale, seed, refresh_id,
                                   _vec(idx, torch.int32), _vec(rho, torch.float32), wp, wb,
                                   _stream()), "grass_select_rows")
    return idx, rho


def select_static_capacity() -> int:
    return int(lib().grass_select_static_capacity())


def select_rows_static(sumsq, r, method, replacement, scale, seed, refresh_id, idx, rho, status=None):
    """grass_select_rows with the library's built-in scratch (no workspace, no allocation);
    status: optional int32 device tensor of one element that receives the status word."""
    m = sumsq.shape[0]
    assert idx.shape == (r,) and rho.shape == (r,)
    sp = None
    if status is not None:
        assert status.is_cuda and status.dtype == torch.int32 and status.numel() == 1
        sp = C.c_void_p(status.data_ptr())
    _check(lib().grass_select_rows_static(_vec(sumsq, torch.float32), m, r, method,
                                          int(bool(replacement)), scale, seed, refresh_id,
                                          _vec(idx, torch.int32), _vec(rho, torch.float32), sp,
                                          _stream()), "grass_select_rows_static")
    return idx, rho


def select_status(ws) -> int:
    """Device status word of the last grass_select_rows that used `ws` (synchronises)."""
    return int(ws.view(torch.uint8)[:4].view(torch.int32).item())


def cgrad_workspace(T, m, n, r, dtype, layout=DY_TxM) -> int:
    return int(lib().grass_cgrad_workspace(T, m, n, r, dtype, layout))


def cgrad_plan(T, n, rows, dtype, layout=DY_TxM, m=0, count=1):
    """(tile edge, number of K slices) the library plans for `count` gathered sets of `rows` rows
    in all; m: row length of dY (0: not given).  Tile 0: the gather runs inside the GEMM."""
    tile, slices = C.c_int(0), C.c_int(0)
    _check(lib().grass_cgrad_plan(T, m, n, rows, count, dtype, layout, C.byref(tile), C.byref(slices)),
           "grass_cgrad_plan")
    return tile.value, slices.value


def set_test_option(option: int, value: int):
    """Test hook: force one of the launcher's choices (0 gives it back to the library)."""
    _check(lib().grass_set_test_option(option, value), "grass_set_test_option")


def compressed_grad(dY, X, idx, rho, GC, ws, layout=DY_TxM, gemm_events=None):
    """gemm_events: optional (start, stop) torch.cuda.Event pair, already recorded once so
    that their handles exist; the library re-records them around the GEMM kernel."""
    pY, ry, cy, ldy = _mat(dY)
    pX, T, n, ldx = _mat(X)
    m = cy if layout == DY_TxM else ry
    assert (ry if layout == DY_TxM else cy) == T and dY.dtype == X.dtype
    r = idx.shape[0]
    pG, gr, gc, ldgc = _mat(GC)
    assert (gr, gc) == (r, n) and GC.dtype == torch.float32
    wp, wb = _ws(ws)
    args = (pY, layout, ldy, pX, ldx, _dtype(X), T, m, n, r, _vec(idx, torch.int32),
            _vec(rho, torch.float32), pG, ldgc, wp, wb, _stream())
    if gemm_events is None:
        _check(lib().grass_compressed_grad(*args), "grass_compressed_grad")
    else:
        e0, e1 = (C.c_void_p(e.cuda_event) for e in gemm_events)
        _check(lib().grass_compressed_grad_timed(*args, e0, e1), "grass_compressed_grad_timed")
    return GC


def _i64_array(values):
    return (C.c_int64 * len(values))(*[int(v) for v in values])


def _ptr_array(pointers):
    return (C.c_void_p * len(pointers))(*[p.value if isinstance(p, C.c_void_p) else p
                                          for p in pointers])


def cgrad_group_workspace(T, n, rs, dtype, layout=DY_TxM) -> int:
    return int(lib().grass_cgrad_group_workspace(T, n, len(rs), _i64_array(rs), dtype, layout))


def compressed_grad_group(dYs, X, idxs, rhos, GCs, ws, layout=DY_TxM):
    """Compressed gradients of several matrices that share the activations X, in one call."""
    count = len(dYs)
    assert count == len(idxs) == len(rhos) == len(GCs) and count >= 1
    pX, T, n, ldx = _mat(X)
    pYs, ldys, ms, rs, pIs, pRs, pGs, ldgcs = [], [], [], [], [], [], [], []
    for dY, idx, rho, GC in zip(dYs, idxs, rhos, GCs):
        pY, ry, cy, ldy = _mat(dY)
        assert (ry if layout == DY_TxM else cy) == T and dY.dtype == X.dtype
        r = idx.shape[0]
        pG, gr, gc, ldgc = _mat(GC)
        assert (gr, gc) == (r, n) and GC.dtype == torch.float32
        pYs.append(pY); ldys.append(ldy); ms.append(cy if layout == DY_TxM else ry); rs.append(r)
        pIs.append(_vec(idx, torch.int32)); pRs.append(_vec(rho, torch.float32))
        pGs.append(pG); ldgcs.append(ldgc)
    wp, wb = _ws(ws)
    _check(lib().grass_compressed_grad_group(
        count, _ptr_array(pYs), layout, _i64_array(ldys), pX, ldx, _dtype(X), T, _i64_array(ms), n,
        _i64_array(rs), _ptr_array(pIs), _ptr_array(pRs), _ptr_array(pGs), _i64_array(ldgcs),
        wp, wb, _stream()), "grass_compressed_grad_group")
    return GCs


def _moments(M, V, r, n):
    """Pointers and dtype code of the Adam moments (fp32, or bf16 for the 2-byte state)."""
    for a in (M, V):
        assert a.shape == (r, n) and a.is_contiguous() and a.is_cuda and a.dtype == M.dtype
    return C.c_void_p(M.data_ptr()), C.c_void_p(V.data_ptr()), _dtype(M)


def step_group_workspace(T, n, rs, dtype, layout=DY_TxM) -> int:
    return int(lib().grass_step_group_workspace(T, n, len(rs), _i64_array(rs), dtype, layout))


def step_group(dYs, X, idxs, rhos, Ms, Vs, Ws, lr, beta1, beta2, eps, t, alpha, ws, layout=DY_TxM,
               GCs=None, step_scalars=None, gemm_events=None, tail_events=None):
    """The regular step (compressed gradient, Adam, row update) of several layers sharing X in
    one call; GCs: optional list with a tensor (G_C is stored there) or None per layer;
    gemm_events / tail_events: optional (start, stop) torch.cuda.Event pairs (recorded once, so
    that their handles exist) for the matrix-multiply kernel and for the fused tail."""
    count = len(dYs)
    pX, T, n, ldx = _mat(X)
    arr = (StepLayer * count)()
    sdt = wdt = None
    for i in range(count):
        pY, ry, cy, ldy = _mat(dYs[i])
        assert (ry if layout == DY_TxM else cy) == T and dYs[i].dtype == X.dtype
        m = cy if layout == DY_TxM else ry
        r = idxs[i].shape[0]
        pW, mw, nw, ldw = _mat(Ws[i])
        assert (mw, nw) == (m, n)
        pM, pV, sd = _moments(Ms[i], Vs[i], r, n)
        assert sdt in (None, sd) and wdt in (None, _dtype(Ws[i]))
        sdt, wdt = sd, _dtype(Ws[i])
        gc = GCs[i] if GCs is not None else None
        if gc is not None:
            pG, gr, gcols, ldgc = _mat(gc)
            assert (gr, gcols) == (r, n) and gc.dtype == torch.float32
        arr[i] = StepLayer(pY.value, ldy, m, r, _vec(idxs[i], torch.int32).value,
                           _vec(rhos[i], torch.float32).value, pG.value if gc is not None else None,
                           ldgc if gc is not None else 0, pM.value, pV.value, pW.value, ldw)
    wp, wb = _ws(ws)
    sc = C.c_void_p(step_scalars.data_ptr()) if step_scalars is not None else None
    e0, e1 = ((C.c_void_p(e.cuda_event) for e in gemm_events) if gemm_events is not None
              else (None, None))
    if tail_events is None:
        _check(lib().grass_step_group(count, arr, layout, pX, ldx, _dtype(X), T, n, sdt, wdt, lr,
                                      beta1, beta2, eps, t, sc, alpha, wp, wb, _stream(), e0, e1),
               "grass_step_group")
    else:
        t0, t1 = (C.c_void_p(e.cuda_event) for e in tail_events)
        _check(lib().grass_step_group_timed(count, arr, layout, pX, ldx, _dtype(X), T, n, sdt, wdt,
                                            lr, beta1, beta2, eps, t, sc, alpha, wp, wb, _stream(),
                                            e0, e1, t0, t1), "grass_step_group_timed")


def step_cols_workspace(T, m, n, r, dtype) -> int:
    return int(lib().grass_step_cols_workspace(T, m, n, r, dtype))


def step_cols(dY, X, idx, rho, M, V, U, W, lr, beta1, beta2, eps, t, alpha, ws, GC=None,
              gemm_events=None):
    """The regular step with r of the n COLUMNS of W selected (dY T x m, X T x n, state r x m)
    in one call; GC: optional r x m tensor that receives the compressed gradient."""
    pY, T, m, ldy = _mat(dY)
    pX, Tx, n, ldx = _mat(X)
    assert Tx == T and dY.dtype == X.dtype
    r = idx.shape[0]
    pW, mw, nw, ldw = _mat(W)
    assert (mw, nw) == (m, n)
    pM, pV, sdt = _moments(M, V, r, m)
    assert U.shape == (r, m) and U.is_contiguous() and U.dtype == torch.float32 and U.is_cuda
    pG, ldgc = None, 0
    if GC is not None:
        pG, gr, gcols, ldgc = _mat(GC)
        assert (gr, gcols) == (r, m) and GC.dtype == torch.float32
    wp, wb = _ws(ws)
    e0, e1 = ((C.c_void_p(e.cuda_event) for e in gemm_events) if gemm_events is not None
              else (None, None))
    _check(lib().grass_step_cols(pY, ldy, pX, ldx, _dtype(X), T, m, n, r, _vec(idx, torch.int32),
                                 _vec(rho, torch.float32), pG, ldgc, pM, pV, sdt,
                                 C.c_void_p(U.data_ptr()), pW, _dtype(W), ldw, lr, beta1, beta2, eps,
                                 t, alpha, wp, wb, _stream(), e0, e1), "grass_step_cols")


def adam_rows(GC, M, V, lr, beta1, beta2, eps, t, U):
    pG, r, n, ldgc = _mat(GC)
    pM, pV, sdt = _moments(M, V, r, n)
    assert U.shape == (r, n) and U.is_contiguous() and U.dtype == torch.float32 and U.is_cuda
    pU = C.c_void_p(U.data_ptr())
    if sdt == F32:
        _check(lib().grass_adam_rows(pG, ldgc, pM, pV, r, n, lr, beta1, beta2, eps, t, pU,
                                     _stream()), "grass_adam_rows")
    else:
        _check(lib().grass_adam_rows_state(pG, ldgc, pM, pV, sdt, r, n, lr, beta1, beta2, eps, t,
                                           pU, _stream()), "grass_adam_rows_state")
    return U


def scatter_update(W, idx, rho, alpha, U):
    pW, m, n, ldw = _mat(W)
    r = idx.shape[0]
    assert U.shape == (r, n) and U.is_contiguous() and U.dtype == torch.float32
    _check(lib().grass_scatter_update(pW, _dtype(W), m, n, ldw, _vec(idx, torch.int32),
                                      _vec(rho, torch.float32), alpha, C.c_void_p(U.data_ptr()), r,
                                      _stream()), "grass_scatter_update")
    return W


def scatter_update_cols(W, idx, rho, alpha, U):
    pW, m, n, ldw = _mat(W)
    r = idx.shape[0]
    assert U.shape == (r, m) and U.is_contiguous() and U.dtype == torch.float32
    _check(lib().grass_scatter_update_cols(pW, _dtype(W), m, n, ldw, _vec(idx, torch.int32),
                                           _vec(rho, torch.float32), alpha,
                                           C.c_void_p(U.data_ptr()), r, _stream()),
           "grass_scatter_update_cols")
    return W


def adam_scatter(GC, M, V, lr, beta1, beta2, eps, t, W, idx, rho, alpha):
    pG, r, n, ldgc = _mat(GC)
    pW, m, nw, ldw = _mat(W)
    assert nw == n and idx.shape == (r,)
    pM, pV, sdt = _moments(M, V, r, n)
    tail = (pW, _dtype(W), m, ldw, _vec(idx, torch.int32), _vec(rho, torch.float32), alpha,
            _stream())
    if sdt == F32:
        _check(lib().grass_adam_scatter(pG, ldgc, pM, pV, r, n, lr, beta1, beta2, eps, t, *tail),
               "grass_adam_scatter")
    else:
        _check(lib().grass_adam_scatter_state(pG, ldgc, pM, pV, sdt, r, n, lr, beta1, beta2, eps,
                                              t, *tail), "grass_adam_scatter_state")
    return W


def adam_step_scalars(lr, beta1, beta2, t):
    """(lr, 1/(1-beta1^t), 1/(1-beta2^t)) as the float32 values the Adam kernels use."""
    out = (C.c_float * 3)()
    _check(lib().grass_adam_step_scalars(lr, beta1, beta2, t, out), "grass_adam_step_scalars")
    return [out[0], out[1], out[2]]


def adam_scatter_replayable(GC, M, V, beta1, beta2, eps, step_scalars, W, idx, rho, alpha):
    """grass_adam_scatter with lr and the bias corrections read from the device array
    `step_scalars` (3 floats), for steps that are captured into a graph and replayed."""
    pG, r, n, ldgc = _mat(GC)
    pW, m, nw, ldw = _mat(W)
    assert nw == n and idx.shape == (r,)
    pM, pV, sdt = _moments(M, V, r, n)
    assert step_scalars.is_cuda and step_scalars.dtype == torch.float32 and step_scalars.numel() >= 3
    _check(lib().grass_adam_scatter_replayable(
        pG, ldgc, pM, pV, sdt, r, n, beta1, beta2, eps, C.c_void_p(step_scalars.data_ptr()), pW,
        _dtype(W), m, ldw, _vec(idx, torch.int32), _vec(rho, torch.float32), alpha, _stream()),
        "grass_adam_scatter_replayable")
    return W


def dense_workspace(T, m, n, dtype, layout=DY_TxM) -> int:
    return int(lib().grass_dense_workspace(T, m, n, dtype, layout))


def dense_grad(dY, X, G, ws, layout=DY_TxM):
    pY, ry, cy, ldy = _mat(dY)
    pX, T, n, ldx = _mat(X)
    m = cy if layout == DY_TxM else ry
    pG, gr, gc, ldg = _mat(G)
    assert (gr, gc) == (m, n) and dY.dtype == X.dtype
    wp, wb = _ws(ws)
    _check(lib().grass_dense_grad(pY, layout, ldy, pX, ldx, _dtype(X), T, m, n, pG, _dtype(G),
                                  ldg, wp, wb, _stream()), "grass_dense_grad")
    return G


def grad_row_stats_workspace(T, m, n, dtype, layout=DY_TxM, ldy=None, ldx=None) -> int:
    ldy = (m if layout == DY_TxM else T) if ldy is None else ldy
    ldx = n if ldx is None else ldx
    return int(lib().grass_grad_row_stats_workspace(T, m, n, dtype, layout, ldy, ldx))


def grad_row_stats(dY, X, sumsq, ws, layout=DY_TxM):
    pY, ry, cy, ldy = _mat(dY)
    pX, T, n, ldx = _mat(X)
    m = cy if layout == DY_TxM else ry
    assert sumsq.shape == (m,) and dY.dtype == X.dtype
    wp, wb = _ws(ws)
    _check(lib().grass_grad_row_stats(pY, layout, ldy, pX, ldx, _dtype(X), T, m, n,
                                      _vec(sumsq, torch.float32), wp, wb, _stream()),
           "grass_grad_row_stats")
    return sumsq


def gather_rows(G, idx, rho, out):
    pG, m, n, ldg = _mat(G)
    r = idx.shape[0]
    pO, orr, oc, ldo = _mat(out)
    assert (orr, oc) == (r, n) and out.dtype == torch.float32
    _check(lib().grass_gather_rows(pG, _dtype(G), m, n, ldg, _vec(idx, torch.int32),
                                   _vec(rho, torch.float32), r, pO, ldo, _stream()),
           "grass_gather_rows")
    return out


def workspace(nbytes: int, device="cuda"):
    """A device byte buffer of at least `nbytes` (torch owns the memory)."""
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)
