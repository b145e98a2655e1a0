"""Pins for the oracle's ranking / assignment / drop step (Sec. III-B.3)."""
import numpy as np
import pytest

import halo_synth as hs
from oracle import ref
from tests.util import read_golden


def test_hand_worked_example():
    g = read_golden("mask_example.txt")
    out = ref.build_group_mask(np.array([g["scores"]], np.float32), g["k_keep"][0],
                               g["prio_dev"], 2, np.array([g["drop"]], np.uint8))
    for k in ("order", "group_dev", "mask", "surv_idx"):
        assert out[k][0].tolist() == g[k], k
    assert out["n_surv"].tolist() == g["n_surv"]


def _brute_order(s):
    """Sort (value desc, index asc), NaN after every number: plain Python sort on tuples."""
    def key(g):
        v = float(s[g])
        return (1, 0.0, g) if np.isnan(v) else (0, -v, g)
    return sorted(range(len(s)), key=key)


@pytest.mark.parametrize("seed", range(30))
def test_ranking_matches_brute_force_sort_tiny(seed):
    rng = np.random.default_rng(seed)
    G = int(rng.integers(1, 9))
    pool = np.array([0.0, -0.0, 1.0, 1.0, -2.5, 3.25, np.inf, -np.inf, np.nan, 1e-30], np.float32)
    s = rng.choice(pool, size=(3, G)).astype(np.float32)
    K = int(rng.integers(0, G + 1))
    out = ref.build_group_mask(s, K, np.zeros(K, np.int8), 1)
    for t in range(3):
        assert out["order"][t].tolist() == _brute_order(s[t])


@pytest.mark.parametrize("G", [8, 86, 108, 224])
def test_ranking_matches_library_stable_argsort(G):
    rng = np.random.default_rng(G)
    s = rng.standard_normal((16, G)).astype(np.float32)
    s[:, ::5] = np.round(s[:, ::5])          # many exact ties
    out = ref.build_group_mask(s, G // 2, np.zeros(G // 2, np.int8), 1)
    lib = np.argsort(-s, axis=1, kind="stable")
    assert np.array_equal(out["order"], lib)


@pytest.mark.parametrize("seed", range(10))
def test_assignment_and_drop_properties(seed):
    rng = np.random.default_rng(100 + seed)
    T, G, n_dev = 7, int(rng.integers(4, 60)), int(rng.integers(1, 7))
    K = int(rng.integers(1, G + 1))
    s = rng.standard_normal((T, G)).astype(np.float32)
    prio_dev = np.sort(rng.integers(0, n_dev, size=K)).astype(np.int8)
    drop = (rng.random((T, n_dev)) < 0.4).astype(np.uint8)
    out = ref.build_group_mask(s, K, prio_dev, n_dev, drop)
    for t in range(T):
        order, gd, m = out["order"][t], out["group_dev"][t], out["mask"][t]
        assert sorted(order.tolist()) == list(range(G))
        sel = set(order[:K].tolist())
        for p, g in enumerate(order):
            if p < K:
                assert gd[g] == prio_dev[p]
                assert m[g] == (0 if drop[t, prio_dev[p]] else 1)
            else:
                assert gd[g] == -1 and m[g] == 0
        surv = [g for g in range(G) if m[g]]
        assert out["n_surv"][t] == len(surv)
        assert out["surv_idx"][t, :len(surv)].tolist() == surv
        assert (out["surv_idx"][t, len(surv):] == -1).all()
        assert set(surv) <= sel
        # every selected group scores at least as high as every unselected one
        if K < G:
            assert s[t, list(sel)].min() >= np.delete(s[t], list(sel)).max()
    # no drops given == all-zero drops
    a = ref.build_group_mask(s, K, prio_dev, n_dev, None)
    b = ref.build_group_mask(s, K, prio_dev, n_dev, np.zeros((T, n_dev), np.uint8))
    assert all(np.array_equal(a[k], b[k]) for k in a)
    assert (a["n_surv"] == K).all()


def test_all_devices_lost_and_stable_master():
    s = np.arange(12, dtype=np.float32).reshape(2, 6)
    pd = ref.schedule(4, [0.0, 0.5])
    drop = np.array([[1, 1], [0, 1]], np.uint8)
    out = ref.build_group_mask(s, 4, pd, 2, drop)
    assert out["n_surv"].tolist() == [0, 2]
    assert (out["mask"][0] == 0).all() and (out["surv_idx"][0] == -1).all()
    # token 1: the two most significant groups (5, 4) sit on the lossless device 0
    assert out["surv_idx"][1].tolist() == [4, 5, -1, -1]


def test_expected_survivors_llama7b_decode_statistic():
    # E[n_surv] = sum_i chunk_i (1 - plr_i) = 11 + 11*.95 + 10*.9 + 11*.8 = 39.25
    w = hs.LLAMA7B_DECODE
    K = w.k_keep()
    pd = ref.schedule(K, w.device_plr())
    n = []
    rng = np.random.default_rng(0)
    s = rng.standard_normal((1, w.n_groups)).astype(np.float32)
    for step in range(1024):
        drop = hs.drop_outcomes(w, 0, step)
        n.append(int(ref.build_group_mask(s, K, pd, w.n_dev, drop)["n_surv"][0]))
    # sd per step = sqrt(121*.05*.95 + 100*.1*.9 + 121*.2*.8) ~ 5.8 -> se of the mean ~ 0.18
    assert abs(np.mean(n) - 39.25) < 0.75
