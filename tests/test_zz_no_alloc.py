"""grass_select_rows_static, the entry point that allocates nothing: through the C ABI, its
idx, rho and status word against grass_select_rows on the same inputs, bit for bit, on calls
in a row that share the library's static scratch (the later ones with smaller inputs)."""
import numpy as np
import pytest
import torch

from paper_2406_17660_amd import grass

pytestmark = pytest.mark.gpu
DEV = "cuda"


def statistic(m, seed, bad=None):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    ss = torch.randn(m, generator=g, device=DEV).square_() * 3.0
    if bad is not None:
        ss[m // 3] = bad
    return ss


def both(ss, r, method, replacement, scale, seed, refresh_id):
    m = ss.shape[0]
    out = []
    for static in (False, True):
        idx = torch.full((r,), -7, dtype=torch.int32, device=DEV)
        rho = torch.full((r,), float("nan"), dtype=torch.float32, device=DEV)
        if static:
            status = torch.full((1,), -1, dtype=torch.int32, device=DEV)
            before = torch.cuda.memory_allocated()
            grass.select_rows_static(ss, r, method, replacement, scale, seed, refresh_id, idx, rho, status)
            assert torch.cuda.memory_allocated() == before
            code = int(status.item())
        else:
            ws = grass.workspace(grass.select_workspace(m, r, method, replacement))
            grass.select_rows(ss, r, method, replacement, scale, seed, refresh_id, idx, rho, ws)
            code = grass.select_status(ws)
        out.append((idx.cpu().numpy(), rho.cpu().numpy(), code))
    return out


# a large problem first, then smaller ones: what the first call leaves in the scratch must not show
CASES = [
    (grass.SEL_MULTI_NORM, True, [(60000, 2000), (4096, 1024), (777, 100), (1, 1)]),
    (grass.SEL_MULTI_NORM, False, [(60000, 1500), (13824, 1024), (4096, 1024), (70, 70)]),
    (grass.SEL_MULTI_NORM2, False, [(20000, 900), (512, 128)]),
    (grass.SEL_UNIFORM, True, [(5461, 512), (100, 300)]),
    (grass.SEL_UNIFORM, False, [(2736, 256), (64, 3)]),
    (grass.SEL_TOPR, False, [(65536, 1024), (1024, 256), (5, 0)]),
]


@pytest.mark.parametrize("method,replacement,sizes", CASES)
def test_static_scratch_selection_equals_the_workspace_form(method, replacement, sizes):
    for call, (m, r) in enumerate(sizes):
        for scale in (grass.SCALE_PAPER,) + (() if method == grass.SEL_TOPR else (grass.SCALE_INV_SQRT_RQ,)):
            ss = statistic(m, 900 + call)
            (i0, r0, c0), (i1, r1, c1) = both(ss, r, method, replacement, scale, 41 + call, call)
            assert c0 == c1 == grass.OK
            assert np.array_equal(i0, i1) and np.array_equal(r0, r1), (m, r, scale)
            assert r == 0 or (i1.min() >= 0 and i1.max() < m)


def test_static_scratch_mixed_rules_back_to_back():
    """Different rules reuse the same bytes for different things (prefix sums, tree, counters)."""
    order = [(grass.SEL_MULTI_NORM, False, 30000, 700), (grass.SEL_MULTI_NORM, True, 9000, 4000),
             (grass.SEL_TOPR, False, 9000, 100), (grass.SEL_UNIFORM, False, 300, 299),
             (grass.SEL_MULTI_NORM2, True, 50, 20)]
    for k, (method, replacement, m, r) in enumerate(order):
        ss = statistic(m, 950 + k)
        (i0, r0, c0), (i1, r1, c1) = both(ss, r, method, replacement, grass.SCALE_PAPER, 7, k)
        assert c0 == c1 == grass.OK and np.array_equal(i0, i1) and np.array_equal(r0, r1)


@pytest.mark.parametrize("bad", [float("nan"), -1.0])
def test_static_scratch_reports_nonfinite_statistics_like_the_workspace_form(bad):
    ss = statistic(3000, 960, bad)
    (i0, r0, c0), (i1, r1, c1) = both(ss, 40, grass.SEL_MULTI_NORM, True, grass.SCALE_PAPER, 3, 0)
    assert c0 == c1 == grass.ERR_NONFINITE
    assert np.array_equal(i0, i1) and np.array_equal(r0, r1)
    # and without a status word of the caller's
    idx = torch.zeros(40, dtype=torch.int32, device=DEV)
    rho = torch.zeros(40, dtype=torch.float32, device=DEV)
    grass.select_rows_static(ss, 40, grass.SEL_MULTI_NORM, True, grass.SCALE_PAPER, 3, 0, idx, rho)
    assert np.array_equal(idx.cpu().numpy(), i0)


def test_static_scratch_refuses_sizes_beyond_its_capacity():
    cap = grass.select_static_capacity()
    assert cap == 1 << 20
    m = 100000
    assert grass.select_workspace(m, 10, grass.SEL_MULTI_NORM, True) > cap
    ss = statistic(m, 970)
    idx = torch.full((10,), -7, dtype=torch.int32, device=DEV)
    rho = torch.zeros(10, dtype=torch.float32, device=DEV)
    with pytest.raises(grass.GrassError) as e:
        grass.select_rows_static(ss, 10, grass.SEL_MULTI_NORM, True, grass.SCALE_PAPER, 1, 0, idx, rho)
    assert e.value.code == grass.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert (idx == -7).all()  # nothing was launched
    # Top-r needs only the status word, whatever m is
    idx2 = torch.zeros(10, dtype=torch.int32, device=DEV)
    grass.select_rows_static(ss, 10, grass.SEL_TOPR, False, grass.SCALE_PAPER, 1, 0, idx2, rho)
    ws = grass.workspace(grass.select_workspace(m, 10, grass.SEL_TOPR, False))
    idx3 = torch.zeros(10, dtype=torch.int32, device=DEV)
    grass.select_rows(ss, 10, grass.SEL_TOPR, False, grass.SCALE_PAPER, 1, 0, idx3, rho, ws)
    assert torch.equal(idx2, idx3)
