"""The seeded input generators (CPU only): deterministic, shaped and distributed as stated."""
import numpy as np
import torch

from paper_2406_17660_amd import workloads


def test_seeds_are_distinct_per_tensor_and_reproducible():
    seeds = {workloads.tensor_seed(c, l, s, k) for c in (1, 2, 5) for l in (0, 1, 2)
             for s in (0, 1, 7) for k in (0, 1, 2, 3)}
    assert len(seeds) == 3 * 3 * 3 * 4
    cfg = workloads.CONFIGS[2]
    a = workloads.make_dY(cfg, 0, 3, "cpu", T=64)
    b = workloads.make_dY(cfg, 0, 3, "cpu", T=64)
    c = workloads.make_dY(cfg, 0, 4, "cpu", T=64)
    assert torch.equal(a, b) and not torch.equal(a, c)
    assert a.dtype == torch.bfloat16 and tuple(a.shape) == (64, cfg.layers[0].m)


def test_shapes_follow_the_model_table():
    """Hidden and MLP widths of the LLaMA sizes the paper trains (its table of model dimensions)."""
    want = {2: (512, 1376), 3: (1024, 2736), 4: (2048, 5461)}
    for cid, (hidden, inter) in want.items():
        names = {l.name: (l.m, l.n) for l in workloads.CONFIGS[cid].layers}
        assert names["attn_qkvo"] == (hidden, hidden)
        assert names["mlp_gate_up"] == (inter, hidden) and names["mlp_down"] == (hidden, inter)
    c5 = {(l.m, l.n) for l in workloads.CONFIGS[5].layers}
    assert c5 == {(4096, 4096), (11008, 4096), (5120, 5120), (13824, 5120)}
    assert workloads.CONFIGS[5].T == 131072 and workloads.CONFIGS[5].r == 1024
    shapes, groups = workloads.llama_block(*workloads.BLOCKS["7b"])
    assert shapes["gate"] == (11008, 4096) and shapes["down"] == (4096, 11008)
    assert ("q", "k", "v") in groups and ("gate", "up") in groups


def test_distributions_have_the_stated_moments():
    cfg = workloads.CONFIGS[2]  # dY ~ N(0, 1e-2), X ~ N(0, 1), W ~ N(0, 0.02^2)
    dY = workloads.make_dY(cfg, 0, 0, "cpu", T=4096).float().numpy()
    X = workloads.make_X(cfg, 0, 0, "cpu", T=4096).float().numpy()
    W = workloads.make_W(cfg, 0, "cpu").float().numpy()
    assert abs(dY.std() - 0.1) < 2e-3 and abs(dY.mean()) < 1e-3
    assert abs(X.std() - 1.0) < 1e-2 and abs(W.std() - 0.02) < 5e-4
    t3 = workloads.make_X(workloads.CONFIGS[3], 0, 0, "cpu", T=8192).float().numpy()
    assert abs(np.median(np.abs(t3)) - 0.7649 / np.sqrt(3)) < 0.02  # median |t_3| = 0.7649
    assert np.abs(t3).max() > 8  # heavy tails
    logn = workloads.make_dY(workloads.CONFIGS[4], 0, 0, "cpu", T=2048).float().numpy()
    col_std = logn.std(axis=0)
    assert np.log(col_std / 0.1).std() > 0.7  # per-feature scales spread log-normally (sigma = 1)
