"""GPU parity of the matrix product whose gather runs inside the kernel (narrow layers: bf16,
dY stored T x m with m <= 512, at most 128 selected rows per set, n <= 512, T a multiple of 16).

The kernel is compared element by element with the fp64 oracle, over every pipeline length,
ragged row counts and widths, repeated rows, padded leading dimensions and groups of sets that
share X, and its result with the packed route's (same products, another summation order)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2406_17660_amd import grass
from gpu_util import DEV, gpu_cgrad, rel_fro, to_f64, to_np
from test_gpu_parity import make_idx, randn, run_step_group

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def narrow_cgrad(T, m, n, r, dup, pad_y=0, pad_x=0, seed=1, max_slices=0):
    """G_C by the library's own choice of route (asserted to be the narrow kernel), the same by
    the packed route, and the oracle's."""
    dY = randn((T, m), BF, seed, scale=0.1, ld=m + pad_y)
    X = randn((T, n), BF, seed + 1, ld=n + pad_x)
    idx, rho = make_idx(m, r, seed + 2, dup)
    d_idx, d_rho = torch.from_numpy(idx).to(DEV), torch.from_numpy(rho).to(DEV)
    if max_slices:
        grass.set_test_option(grass.TEST_MAX_K_SLICES, max_slices)
    tile, slices = grass.cgrad_plan(T, n, r, grass.BF16, m=m)
    assert tile == 0, "this shape is meant to take the kernel that gathers by itself"
    got = to_f64(gpu_cgrad(dY, X, d_idx, d_rho))
    grass.set_test_option(grass.TEST_NO_NARROW_GATHER, 1)
    assert grass.cgrad_plan(T, n, r, grass.BF16, m=m)[0] in (128, 256)
    packed = to_f64(gpu_cgrad(dY, X, d_idx, d_rho))
    grass.set_test_option(grass.TEST_NO_NARROW_GATHER, 0)
    want = ref.compressed_grad(to_np(dY), to_np(X), idx, rho)
    return got, packed, want, slices


def check(got, packed, want):
    assert got.shape == want.shape and np.isfinite(got).all()
    assert rel_fro(got, want) <= 2e-5
    assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()
    assert rel_fro(got, packed) <= 2e-6  # fp32 sums of the same exact products


@pytest.mark.parametrize("T", [16, 32, 48, 64, 80, 96, 112, 128, 144, 1040])
def test_every_pipeline_length(T):
    """One K slice (the hook caps the slices): 1 to 9 K tiles and 65 in a workgroup, through the
    ring's fill, steady state and drain."""
    check(*narrow_cgrad(T, 256, 264, 100, True, max_slices=1)[:3])


@pytest.mark.parametrize("T,m,n,r,dup,pad_y,pad_x", [
    (1024, 512, 512, 128, True, 0, 0),     # the 60M attention shape, repeated rows
    (2048, 512, 512, 128, False, 8, 16),   # padded leading dimensions
    (512, 8, 8, 1, False, 0, 0),           # the smallest everything
    (512, 8, 8, 8, False, 0, 0),           # r = m
    (640, 64, 24, 64, True, 0, 0),
    (1024, 504, 328, 127, True, 0, 8),     # widths that end inside a tile, one row short of a tile
    (4096, 256, 392, 37, True, 0, 0),      # n over two column tiles with a ragged second one
    (8192, 512, 256, 128, False, 0, 0),    # many slices, one column tile
    (65536, 512, 512, 128, True, 0, 0),    # the stated token batch: 128 slices
])
def test_shapes_against_the_oracle_and_the_packed_route(T, m, n, r, dup, pad_y, pad_x):
    got, packed, want, slices = narrow_cgrad(T, m, n, r, dup, pad_y, pad_x, seed=10 + r)
    if T == 65536:
        assert slices == 128
    check(got, packed, want)


@pytest.mark.parametrize("slices", [1, 2, 3, 7, 9, 33])
def test_slice_counts(slices):
    """A ragged last slice, and slice counts on both sides of the many-slice reduction."""
    got, packed, want, planned = narrow_cgrad(2000 * 16, 128, 72, 40, True, max_slices=slices)
    assert planned <= slices and (slices > 3 or planned == slices)
    check(got, packed, want)


@pytest.mark.parametrize("T,n,ms,rs", [
    (1024, 512, (512, 512, 512), (128, 128, 128)),  # q, k, v
    (2048, 264, (512, 64, 256), (100, 3, 128)),     # sets of different row lengths and sizes
    (512, 72, (256, 256, 256, 256, 256, 256, 256, 256), (9, 17, 33, 64, 65, 127, 128, 1)),  # eight sets
])
def test_groups_sharing_activations(T, n, ms, rs):
    X = randn((T, n), BF, 40)
    dYs, idxs, rhos, host = [], [], [], []
    for i, (m, r) in enumerate(zip(ms, rs)):
        dY = randn((T, m), BF, 41 + i, scale=0.1)
        idx, rho = make_idx(m, r, 60 + i, duplicates=(i % 2 == 1))
        host.append((dY, idx, rho))
        dYs.append(dY); idxs.append(torch.from_numpy(idx).to(DEV)); rhos.append(torch.from_numpy(rho).to(DEV))
    outs = []
    for packed in (False, True):
        grass.set_test_option(grass.TEST_NO_NARROW_GATHER, int(packed))
        GCs = [torch.full((r, n), float("nan"), dtype=torch.float32, device=DEV) for r in rs]
        ws = grass.workspace(grass.cgrad_group_workspace(T, n, rs, grass.BF16))
        grass.compressed_grad_group(dYs, X, idxs, rhos, GCs, ws)
        outs.append([to_f64(g) for g in GCs])
    grass.set_test_option(grass.TEST_NO_NARROW_GATHER, 0)
    for (dY, idx, rho), got, packed in zip(host, *outs):
        check(got, packed, ref.compressed_grad(to_np(dY), to_np(X), idx, rho))


def _sweep(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for k in range(count):
        sets = int(rng.choice([1, 1, 2, 3, 8]))
        ms = tuple(int(rng.integers(1, 65)) * 8 for _ in range(sets))
        rs = tuple(int(rng.integers(1, min(128, 4 * m) + 1)) for m in ms)
        cases.append((k, int(rng.integers(1, 129)) * 16, int(rng.integers(1, 65)) * 8, ms, rs,
                      int(rng.choice([0, 8, 24])), int(rng.choice([0, 8]))))
    return cases


@pytest.mark.parametrize("k,T,n,ms,rs,pad_y,pad_x", _sweep(32, 17660))
def test_seeded_shape_sweep(k, T, n, ms, rs, pad_y, pad_x):
    """Seeded random shapes inside the kernel's limits (T a multiple of 16 up to 2048, widths and
    row lengths multiples of 8 up to 512, up to 128 unsorted rows per set with repeats, one to
    eight sets, padded leading dimensions) against the oracle."""
    rng = np.random.default_rng(1000 + k)
    X = randn((T, n), BF, 200 + k, ld=n + pad_x)
    dYs = [randn((T, m), BF, 300 + 10 * k + i, scale=0.1, ld=m + pad_y) for i, m in enumerate(ms)]
    idxs = [rng.integers(0, m, r).astype(np.int32) for m, r in zip(ms, rs)]
    rhos = [rng.uniform(0.5, 2.0, r).astype(np.float32) for r in rs]
    total = sum((r + 7) // 8 * 8 for r in rs)
    assert grass.cgrad_plan(T, n, total if len(ms) > 1 else rs[0], grass.BF16, m=max(ms), count=len(ms))[0] == 0
    GCs = [torch.full((r, n), float("nan"), dtype=torch.float32, device=DEV) for r in rs]
    d_idx = [torch.from_numpy(a).to(DEV) for a in idxs]
    d_rho = [torch.from_numpy(a).to(DEV) for a in rhos]
    if len(ms) == 1:
        ws = grass.workspace(grass.cgrad_workspace(T, ms[0], n, rs[0], grass.BF16))
        grass.compressed_grad(dYs[0], X, d_idx[0], d_rho[0], GCs[0], ws)
    else:
        ws = grass.workspace(grass.cgrad_group_workspace(T, n, rs, grass.BF16))
        grass.compressed_grad_group(dYs, X, d_idx, d_rho, GCs, ws)
    for dY, idx, rho, GC in zip(dYs, idxs, rhos, GCs):
        want = ref.compressed_grad(to_np(dY), to_np(X), idx, rho)
        got = to_f64(GC)
        assert np.isfinite(got).all() and rel_fro(got, want) <= 2e-5
        assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()


def test_rows_in_any_order():
    """The selected rows need not come sorted (the selection kernels emit them sorted; a caller's
    own list may not be): a shuffled list with repeats."""
    T, m, n, r = 2048, 512, 256, 128
    dY = randn((T, m), BF, 90, scale=0.1)
    X = randn((T, n), BF, 91)
    rng = np.random.default_rng(92)
    idx = rng.integers(0, m, r).astype(np.int32)
    idx[5] = idx[100] = idx[0]
    rho = rng.uniform(0.5, 2.0, r).astype(np.float32)
    assert grass.cgrad_plan(T, n, r, grass.BF16, m=m)[0] == 0
    got = to_f64(gpu_cgrad(dY, X, torch.from_numpy(idx).to(DEV), torch.from_numpy(rho).to(DEV)))
    want = ref.compressed_grad(to_np(dY), to_np(X), idx, rho)
    assert rel_fro(got, want) <= 2e-5 and np.abs(got - want).max() <= 1e-4 * np.abs(want).max()
    assert np.array_equal(got[5] / rho[5], got[0] / rho[0]) or rel_fro(got[5] / rho[5], got[0] / rho[0]) < 1e-6


def test_what_does_not_fit_takes_the_packed_route():
    """Eligibility is decided per call: rows of dY that are too long, too many rows in a set, a
    third column tile, a ragged token count, m x T storage and misaligned operands all give the
    same numbers through the other kernels."""
    for T, m, n, r in [(1024, 520, 512, 128), (1024, 512, 512, 136), (1024, 512, 520, 128),
                       (1000, 512, 512, 128), (1024, 508, 512, 64)]:
        assert grass.cgrad_plan(T, n, r, grass.BF16, m=m)[0] != 0
        dY = randn((T, m), BF, 70, scale=0.1)
        X = randn((T, n), BF, 71)
        idx, rho = make_idx(m, r, 72, True)
        got = to_f64(gpu_cgrad(dY, X, torch.from_numpy(idx).to(DEV), torch.from_numpy(rho).to(DEV)))
        assert rel_fro(got, ref.compressed_grad(to_np(dY), to_np(X), idx, rho)) <= 2e-5
    # an eligible shape whose activations start 2 bytes off a 16-byte boundary
    T, m, n, r = 1024, 256, 256, 64
    assert grass.cgrad_plan(T, n, r, grass.BF16, m=m)[0] == 0
    dY = randn((T, m), BF, 73, scale=0.1)
    Xw = randn((T, n + 8), BF, 74)
    X = Xw[:, 1:n + 1]
    idx, rho = make_idx(m, r, 75, False)
    got = to_f64(gpu_cgrad(dY, X, torch.from_numpy(idx).to(DEV), torch.from_numpy(rho).to(DEV)))
    assert rel_fro(got, ref.compressed_grad(to_np(dY), to_np(X), idx, rho)) <= 2e-5


@pytest.mark.parametrize("wdtype,sdtype", [(BF, torch.float32), (torch.float32, BF)])
@pytest.mark.parametrize("T,n,ms,rs,want_gc", [
    (1024, 512, (512,), (128,), True),              # few slices: the fused tail for up to eight
    (16384, 256, (512,), (100,), False),            # many slices, G_C not stored
    (8192, 264, (256, 512, 64), (128, 40, 33), True),  # a group, many slices
])
def test_regular_step_through_the_narrow_kernel(wdtype, sdtype, T, n, ms, rs, want_gc):
    """grass_step_group on narrow layers: the fused tail reads this kernel's partial tiles."""
    total = sum((r + 7) // 8 * 8 for r in rs)
    assert grass.cgrad_plan(T, n, total, grass.BF16, m=max(ms), count=len(ms))[0] == 0
    run_step_group(BF, wdtype, sdtype, T, n, ms, rs, want_gc, None)
