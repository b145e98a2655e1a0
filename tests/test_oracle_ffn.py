"""Pins for the oracle's group-sparse SwiGLU FFN (Sec. II-A neuron groups, merge = plain sum)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import halo_synth as hs
from oracle import ref
from tests.util import rel_l2


def _rand(seed, T=3, d=40, G=5, gs=6):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg, Wu, WdT = (rng.standard_normal((G * gs, d)).astype(np.float32) * 0.3 for _ in range(3))
    return x, Wg, Wu, WdT


def _dense_library(x, Wg, Wu, WdT):
    xt, g, u, dn = (torch.from_numpy(np.asarray(v)).double() for v in (x, Wg, Wu, WdT))
    return ((F.silu(xt @ g.T) * (xt @ u.T)) @ dn).numpy()    # WdT is [ffn][d] = Wd^T


@pytest.mark.parametrize("seed", range(4))
def test_keep_all_no_drops_equals_dense_swiglu(seed):
    x, Wg, Wu, WdT = _rand(seed, T=4, d=33, G=7, gs=5)
    y = ref.group_sparse_ffn(x, Wg, Wu, WdT, 5, None)
    np.testing.assert_allclose(y, _dense_library(x, Wg, Wu, WdT), rtol=1e-12, atol=1e-13)
    ones = np.ones((4, 7), np.uint8)
    assert np.array_equal(ref.group_sparse_ffn(x, Wg, Wu, WdT, 5, ones), y)


def test_tiny_workload_dense_equivalence_through_the_whole_pass():
    w = hs.TINY
    x = hs.hidden_states(w).numpy()
    Wg, Wu, WdT = (t.numpy() for t in hs.ffn_weights(w))
    At, Bt = (t.numpy() for t in hs.predictor_weights(w))
    G = w.n_groups
    pd = ref.schedule(G, w.device_plr())
    out = ref.ffn_forward(x, At, Bt, Wg, Wu, WdT, w.group_size, G, pd, w.n_dev, None)
    assert (out["mask"] == 1).all() and (out["n_surv"] == G).all()
    assert rel_l2(out["y"], _dense_library(x, Wg, Wu, WdT)) < 1e-13


def test_sum_of_partials_is_dense_and_masked_partials_are_exact_zero():
    x, Wg, Wu, WdT = _rand(11)
    T, G, gs = 3, 5, 6
    p = ref.group_partials(x, Wg, Wu, WdT, gs)
    np.testing.assert_allclose(p.sum(axis=1), _dense_library(x, Wg, Wu, WdT), rtol=1e-12, atol=1e-13)
    # each partial alone equals the dense block restricted to that group's neurons
    for g in range(G):
        sl = slice(g * gs, (g + 1) * gs)
        np.testing.assert_allclose(p[:, g], _dense_library(x, Wg[sl], Wu[sl], WdT[sl]),
                                   rtol=1e-12, atol=1e-13)
    mask = np.array([[1, 0, 1, 0, 0], [0, 0, 0, 0, 0], [1, 1, 1, 1, 0]], np.uint8)
    pm = ref.group_partials(x, Wg, Wu, WdT, gs, mask)
    y = ref.group_sparse_ffn(x, Wg, Wu, WdT, gs, mask)
    for t in range(T):
        for g in range(G):
            if mask[t, g]:
                assert np.array_equal(pm[t, g], p[t, g])
            else:
                assert not pm[t, g].any()          # exactly zero, bit for bit
    np.testing.assert_allclose(y, pm.sum(axis=1), rtol=1e-13, atol=1e-14)
    assert not y[1].any()                           # a token with no survivor gives exactly 0


def test_unselected_groups_weights_are_never_touched():
    x, Wg, Wu, WdT = _rand(12)
    mask = np.array([[1, 0, 1, 0, 1]] * 3, np.uint8)
    y = ref.group_sparse_ffn(x, Wg, Wu, WdT, 6, mask)
    Wg2, Wu2, Wd2 = Wg.copy(), Wu.copy(), WdT.copy()
    for g in (1, 3):
        for W in (Wg2, Wu2, Wd2):
            W[g * 6:(g + 1) * 6] = np.nan
    y2 = ref.group_sparse_ffn(x, Wg2, Wu2, Wd2, 6, mask)
    assert np.isfinite(y2).all() and np.array_equal(y, y2)


def test_silu_identities():
    # SiLU(z) - SiLU(-z) = z: two neurons with gates +z and -z, ups u and -u, same down row
    z, u = 1.75, 0.5
    x = np.array([[1.0, 0.0]], np.float32)
    Wg = np.array([[z, 0], [-z, 0]], np.float32)
    Wu = np.array([[u, 0], [-u, 0]], np.float32)
    WdT = np.array([[2.0, -1.0], [2.0, -1.0]], np.float32)
    y = ref.group_sparse_ffn(x, Wg, Wu, WdT, 2)
    np.testing.assert_allclose(y, [[z * u * 2.0, -z * u]], rtol=1e-15)
    # SiLU(0) = 0 whatever the up projection is; saturation: SiLU(40) ~ 40, SiLU(-40) ~ 0
    Wg = np.array([[0.0, 0], [40.0, 0]], np.float32)
    Wu = np.array([[123.0, 0], [1.0, 0]], np.float32)
    WdT = np.array([[1.0, 0.0], [0.0, 1.0]], np.float32)
    y = ref.group_sparse_ffn(x, Wg, Wu, WdT, 1)
    assert y[0, 0] == 0.0 and abs(y[0, 1] - 40.0) < 1e-12
    y = ref.group_sparse_ffn(-x, Wg, Wu, WdT, 1)
    assert y[0, 0] == 0.0 and 0.0 < y[0, 1] < 1e-14     # (-40)(-1) e^-40


def test_group_permutation_and_down_scaling():
    x, Wg, Wu, WdT = _rand(13)
    gs, G = 6, 5
    mask = np.array([[1, 1, 0, 1, 0], [0, 1, 1, 0, 0], [1, 0, 0, 0, 1]], np.uint8)
    y = ref.group_sparse_ffn(x, Wg, Wu, WdT, gs, mask)
    perm = np.array([3, 0, 4, 2, 1])
    rows = np.concatenate([np.arange(g * gs, (g + 1) * gs) for g in perm])
    y2 = ref.group_sparse_ffn(x, Wg[rows], Wu[rows], WdT[rows], gs, mask[:, perm])
    np.testing.assert_allclose(y2, y, rtol=1e-12, atol=1e-13)
    assert np.array_equal(ref.group_sparse_ffn(x, Wg, Wu, 2 * WdT, gs, mask), 2 * y)
