"""Host-side schedule of Algorithm 1's outer loop (CPU only): hand-computed values."""
import math

import pytest

from paper_2406_17660_amd.block import RewarmSchedule


def test_refresh_steps_are_multiples_of_K():
    s = RewarmSchedule(K=200)
    assert [t for t in range(601) if s.is_refresh(t)] == [0, 200, 400, 600]
    assert not RewarmSchedule(K=0).is_refresh(0)


def test_global_part_warmup_then_cosine_to_ten_percent():
    s = RewarmSchedule(base_lr=1e-2, warmup=1000, total=10000, min_ratio=0.1, K=200, rewarm=0)
    assert s.lr(0) == pytest.approx(1e-2 / 1000)
    assert s.lr(499) == pytest.approx(1e-2 * 0.5)
    assert s.lr(999) == pytest.approx(1e-2)
    assert s.lr(1000) == pytest.approx(1e-2)          # cosine starts at its maximum
    assert s.lr(5500) == pytest.approx(1e-2 * 0.55)   # half way: (1 + 0.1) / 2
    assert s.lr(10000) == pytest.approx(1e-3)
    assert s.lr(20000) == pytest.approx(1e-3)         # stays at the floor
    vals = [s.lr(t) for t in range(1000, 10001, 100)]
    assert all(a >= b for a, b in zip(vals, vals[1:]))


def test_rewarm_after_each_projection_update():
    s = RewarmSchedule(base_lr=1.0, warmup=0, total=10**9, min_ratio=1.0, K=200, rewarm=200)
    assert s.lr(0) == pytest.approx(1 / 200)
    assert s.lr(99) == pytest.approx(0.5)
    assert s.lr(199) == pytest.approx(1.0)
    assert s.lr(200) == pytest.approx(1 / 200)        # the ramp restarts with the new projection
    assert s.lr(399) == pytest.approx(1.0)
    short = RewarmSchedule(base_lr=1.0, warmup=0, total=10**9, min_ratio=1.0, K=200, rewarm=50)
    assert short.lr(249) == pytest.approx(1.0) and short.lr(250) == pytest.approx(1.0)
    assert short.lr(224) == pytest.approx(0.5)


def test_both_parts_multiply():
    s = RewarmSchedule(base_lr=4e-3, warmup=10, total=110, min_ratio=0.1, K=20, rewarm=4)
    t = 61  # 51 steps into the cosine span of 100; 1 step after the update at t = 60
    want = 4e-3 * (0.1 + 0.9 * 0.5 * (1 + math.cos(math.pi * 0.51))) * (2 / 4)
    assert s.lr(t) == pytest.approx(want)
