"""The regular step under HIP graph capture: the library allocates nothing, synchronises
nothing and records no memset, so a step (compressed gradient + fused Adam/scatter) can be
captured once and replayed.  Every replay is compared with the eager result."""
import pytest
import torch

from paper_2406_17660_amd import grass
from paper_2406_17660_amd.layer import AdamHyper, GrassLayer
from gpu_util import DEV

pytestmark = pytest.mark.gpu


def draw(shape, seed, scale=1.0):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return (torch.randn(shape, generator=g, device=DEV) * scale).to(torch.bfloat16)


@pytest.mark.parametrize("layout", [grass.DY_TxM, grass.DY_MxT])
@pytest.mark.parametrize("T,m,n,r", [(1024, 512, 384, 96), (2048, 1024, 1024, 512)])
def test_step_replayed_from_a_graph_equals_eager_step(layout, T, m, n, r):
    dY, X = draw((T, m), 1, 0.1), draw((T, n), 2)
    dYin = dY if layout == grass.DY_TxM else dY.t().contiguous()
    W0 = draw((m, n), 3, 0.02)
    st = GrassLayer(m, n, r, T, torch.bfloat16, "multi_norm", True, alpha=0.25,
                    adam=AdamHyper(lr=1e-3), seed=5, layout=layout)
    st.refresh(dYin, X)
    M0 = torch.randn_like(st.M).mul_(0.01)
    V0 = torch.rand_like(st.V).mul_(1e-4)

    def reset(W):
        W.copy_(W0); st.M.copy_(M0); st.V.copy_(V0); st.adam_t = 4

    # eager reference (also the warm-up that creates every lazily initialised handle)
    W = W0.clone()
    reset(W)
    st.step(dYin, X, W)
    torch.cuda.synchronize()
    want = (W.clone(), st.M.clone(), st.V.clone(), st.GC.clone())

    reset(W)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st.step(dYin, X, W)          # Adam's t = 5 and lr are host values fixed at capture
    for replay in range(3):
        reset(W)                     # eager work and a synchronisation between replays
        st.GC.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (W, st.M, st.V, st.GC)
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {replay} differs from the eager step"


def test_matrix_core_probe_reports_plausible_rates():
    """The measurement aid runs with each operand source and lands between a tenth of and just
    above the datasheet peak; random operands cannot be faster than constants by much."""
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    operands = torch.randn(32768, generator=g, device="cuda").to(torch.bfloat16)
    from paper_2406_17660_amd import probe
    rates = [probe.mfma_rate(2000, source, operands)
             for source in (probe.CONSTANTS, probe.REGISTERS, probe.LDS)]
    assert all(250.0 < r < 2600.0 for r in rates), rates
    assert rates[1] < 1.1 * rates[0] and rates[2] < 1.1 * rates[0], rates
