"""Pins for the oracle's Alg. 3 (PLR-aware ratio-guided scheduler)."""
import numpy as np
import pytest

from oracle import ref
from tests.util import read_golden


def _runs(prio_dev, n_dev):
    return {dev: [p + 1 for p in range(len(prio_dev)) if prio_dev[p] == dev] for dev in range(n_dev)}


def test_paper_worked_example():
    g = read_golden("alg3_example.txt")
    pd = ref.schedule(g["n_groups"][0], g["plr"], g["ratios"])
    assert _runs(pd, 3) == g["device"]


def test_group_count_example():
    # Sec. II-A: an MLP of dimension 6144 with group size 256 has 24 neuron groups;
    # the schedule must cover exactly those 24 priority indices.
    n = 6144 // 256
    assert n == 24
    pd = ref.schedule(n, [0.0, 0.1], None)
    assert len(pd) == 24 and sorted(np.bincount(pd).tolist()) == [12, 12]


def test_uniform_chunk_sizes_of_the_workloads():
    # homogeneous ratios; sizes listed from the most stable device to the lossiest
    pd = ref.schedule(43, [0.0, 0.05, 0.1, 0.2])
    assert np.bincount(pd).tolist() == [11, 11, 10, 11]
    pd = ref.schedule(112, [0, 0, .05, .05, .1, .1, .2, .3])
    assert np.bincount(pd).tolist() == [14] * 8
    pd = ref.schedule(4, [0.0, 0.0, 0.1, 0.3])
    assert pd.tolist() == [0, 1, 2, 3]


@pytest.mark.parametrize("seed", range(20))
def test_properties_random(seed):
    rng = np.random.default_rng(seed)
    n_dev = int(rng.integers(1, 9))
    n = int(rng.integers(0, 300))
    plr = rng.choice([0.0, 0.01, 0.05, 0.1, 0.3], size=n_dev)
    r = rng.random(n_dev) + 0.05
    r /= r.sum()
    pd = ref.schedule(n, plr, r)
    assert len(pd) == n and ((pd >= 0) & (pd < n_dev)).all()
    # contiguous runs, and devices appear in ascending-PLR order (ties: lower device first)
    seen = [int(pd[0])] if n else []
    for p in range(1, n):
        if pd[p] != pd[p - 1]:
            assert int(pd[p]) not in seen
            seen.append(int(pd[p]))
    keys = [(plr[dv], dv) for dv in seen]
    assert keys == sorted(keys)
    # the device with the highest PLR holds the least prioritised indices it was given
    if n and len(seen) == n_dev:
        worst = max(range(n_dev), key=lambda dv: (plr[dv], dv))
        assert pd[-1] == worst
    # run lengths within one of n*ratio (round-half-up on cumulative sums)
    counts = np.bincount(pd, minlength=n_dev) if n else np.zeros(n_dev, int)
    assert np.all(np.abs(counts - n * r) <= 1.0 + 1e-9)


def test_stable_device_never_last_and_errors():
    pd = ref.schedule(10, [0.3, 0.0, 0.3])
    # cut points round(10/3)=3, round(20/3)=7, 10; equal PLRs keep device order 0 before 2
    assert pd.tolist() == [1, 1, 1, 0, 0, 0, 0, 2, 2, 2]
    with pytest.raises(ValueError):
        ref.schedule(4, [0.1, float("nan")])
    with pytest.raises(ValueError):
        ref.schedule(4, [0.1, 0.2], [-0.5, 1.5])
    with pytest.raises(ValueError):
        ref.schedule(-1, [0.1])
