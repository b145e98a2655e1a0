"""Pins for the oracle's Alg. 1 (computation-greedy) and Alg. 2 (min-max) ratio schedulers, and
agreement of the library's host functions with them."""
import numpy as np
import pytest

import paper_2601_11676_amd as H
from oracle import ref


def test_comp_greedy_hand_worked():
    # fastest first: device 0 (c=3) takes its 4, device 2 (c=2) takes the remaining 2, device 1 nothing
    r = ref.ratios_comp_greedy([4, 4, 4], [3, 1, 2], 6)
    np.testing.assert_allclose(r, [2 / 3, 0, 1 / 3], rtol=1e-15)
    # demand equal to the total budget: everybody is full, ratios = m / sum(m)
    r = ref.ratios_comp_greedy([1, 2, 5], [1, 9, 3], 8)
    np.testing.assert_allclose(r, [1 / 8, 2 / 8, 5 / 8], rtol=1e-15)
    # equal computing power: lower index first
    r = ref.ratios_comp_greedy([3, 3], [1, 1], 3)
    np.testing.assert_allclose(r, [1.0, 0.0])
    with pytest.raises(ValueError):
        ref.ratios_comp_greedy([1, 1], [1, 1], 3)          # budget below demand


def test_min_max_closed_forms():
    # nobody memory-bound: sum T c_i = M_t  =>  ratios proportional to computing power
    c = np.array([1.0, 2.0, 5.0])
    r = ref.ratios_min_max([100, 100, 100], c, 16, 1e-6)
    np.testing.assert_allclose(r, c / c.sum(), rtol=1e-6)
    # one device memory-bound: min(1,T) + min(10,T) = 6  =>  T = 5, u = (1, 5)
    r = ref.ratios_min_max([1, 10], [1, 1], 6, 1e-9)
    np.testing.assert_allclose(r, [1 / 6, 5 / 6], rtol=1e-8)
    # demand equal to the budget: everybody full
    r = ref.ratios_min_max([2, 6], [5, 1], 8, 1e-6)
    np.testing.assert_allclose(r, [0.25, 0.75], rtol=1e-5)
    # with the paper's eps = 1e-3 the threshold is within eps above the exact one
    r = ref.ratios_min_max([1, 10], [1, 1], 6)
    assert abs(r[1] * 6 - 5) < 2e-3 and abs(r.sum() - 1) < 1e-15


def exact_min_max(m, c, Mt):
    """The quantity Alg. 2's bisection approximates, solved exactly: the smallest T with
    sum_i min(m_i, T c_i) = M_t.  The sum is piecewise linear in T with breakpoints m_i / c_i (device i
    reaches its budget there); walk the breakpoints in ascending order and solve the linear piece that
    crosses M_t.  Returns (T, ratios)."""
    m, c = np.asarray(m, float), np.asarray(c, float)
    order = np.argsort(m / c, kind="stable")
    full, speed = 0.0, c.sum()                 # budget of the saturated devices, speed of the others
    T = None
    for i in order:
        t_break = m[i] / c[i]
        if full + t_break * speed >= Mt:       # the crossing lies before device i saturates
            T = (Mt - full) / speed
            break
        full += m[i]
        speed -= c[i]
    assert T is not None
    u = np.minimum(m, T * c)
    return T, u / u.sum()


@pytest.mark.parametrize("seed", range(40))
def test_min_max_within_eps_of_the_exact_threshold(seed):
    # oracle and library each against the exact solution, within what the stopping rule allows:
    # the threshold returned lies in [T*, T* + eps], so each allocation is at most eps*c_i above the
    # exact one and the ratios move by at most 2 eps sum(c) / M_t
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 9))
    m = rng.integers(3, 64, size=n) * 100.0
    c = rng.integers(6, 19, size=n) / 10.0
    Mt = float(rng.uniform(0.05, 1.0) * m.sum())
    T, r_exact = exact_min_max(m, c, Mt)
    assert abs(np.minimum(m, T * c).sum() - Mt) <= 1e-9 * Mt
    for eps in (1e-3, 1e-6, 0.5):
        bound = 2 * eps * c.sum() / Mt + 1e-12
        for fn in (ref.ratios_min_max, H.halo_ratios_min_max):
            r = fn(m, c, Mt, eps)
            assert np.abs(r - r_exact).max() <= bound, (fn.__module__, eps)
            # never below the exact threshold: the allocation covers the demand
            assert (np.minimum(m, (T + eps) * c) * (1 + 1e-12) >= r * Mt).all()


@pytest.mark.parametrize("seed", range(25))
def test_properties_and_library_agreement(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 9))
    m = rng.integers(3, 64, size=n) * 100.0                 # MB, like the paper's 300..6300 budgets
    c = rng.integers(6, 19, size=n) / 10.0                  # GHz, 0.6..1.8
    Mt = float(rng.uniform(0.2, 1.0) * m.sum())
    for name, oracle_fn, lib_fn in (("greedy", ref.ratios_comp_greedy, H.halo_ratios_comp_greedy),
                                    ("minmax", ref.ratios_min_max, H.halo_ratios_min_max)):
        r = oracle_fn(m, c, Mt)
        assert (r >= 0).all() and abs(r.sum() - 1) < 1e-12, name
        assert (r * Mt <= m * (1 + 2e-3) + 1e-9).all(), name      # nobody above its memory budget
        # the two are written differently but halve the same bracket: same threshold, same ratios
        np.testing.assert_allclose(lib_fn(m, c, Mt), r, rtol=1e-13, atol=1e-15)
    # min-max: the largest per-device time max_i r_i M_t / c_i is not above the greedy one
    tg = np.max(ref.ratios_comp_greedy(m, c, Mt) * Mt / c)
    tm = np.max(ref.ratios_min_max(m, c, Mt, 1e-9) * Mt / c)
    assert tm <= tg * (1 + 1e-6)
    # brute force on a grid for two devices: no split of M_t within the budgets has a smaller maximum
    if n == 2:
        best = min(max(a / c[0], (Mt - a) / c[1]) for a in np.linspace(max(0, Mt - m[1]), min(m[0], Mt), 4001))
        assert tm <= best * (1 + 1e-3)


def test_library_errors_and_schedule_from_ratios():
    with pytest.raises(H.HaloError):
        H.halo_ratios_min_max([1, 1], [1, 1], 3)
    with pytest.raises(H.HaloError):
        H.halo_ratios_comp_greedy([1, 1], [0, 1], 1)
    # heterogeneous devices: ratios -> Alg. 3 -> run lengths follow the ratios
    m, c, plr = [300, 6300, 2100, 900], [1.8, 0.6, 1.2, 1.5], [0.0, 0.05, 0.1, 0.2]
    r = H.halo_ratios_min_max(m, c, 4500)
    pd = H.halo_build_schedule(43, plr, r)
    assert np.array_equal(pd, ref.schedule(43, plr, ref.ratios_min_max(m, c, 4500)))
    counts = np.bincount(pd, minlength=4)
    assert np.all(np.abs(counts - 43 * r) <= 1.0)
