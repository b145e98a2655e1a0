"""Pins for the oracle's predictor (Sec. III-B.2): hand-worked values, a float64 library
matmul, and cases that separate the fixed float32 summation order from any other."""
import numpy as np
import torch

from oracle import ref


def test_hand_worked_integers():
    # A (d x r) = [[1,-1],[0,3]], B (r x G) = [[2,1],[-1,1]]; stored transposed.
    At = np.array([[1, 0], [-1, 3]], dtype=np.float32)
    Bt = np.array([[2, -1], [1, 1]], dtype=np.float32)
    # x=[1,2]: xA=[1,5] -> h=[1,5] -> s=[2-5, 1+5]
    # x=[1,-2]: xA=[1,-7] -> h=[1,0] -> s=[2, 1]    (without the ReLU it would be [9,-6])
    x = np.array([[1, 2], [1, -2]], dtype=np.float32)
    s, s64 = ref.predict_scores(x, At, Bt, want64=True)
    assert s.tolist() == [[-3.0, 6.0], [2.0, 1.0]]
    assert s64.tolist() == [[-3.0, 6.0], [2.0, 1.0]]


def test_against_float64_library_matmul():
    rng = np.random.default_rng(5)
    T, d, r, G = 5, 520, 72, 11          # ragged: d, r not multiples of 512
    x = rng.standard_normal((T, d)).astype(np.float32)
    At = (0.02 * rng.standard_normal((r, d))).astype(np.float32)
    Bt = (0.02 * rng.standard_normal((G, r))).astype(np.float32)
    s, s64 = ref.predict_scores(x, At, Bt, want64=True)
    xt, a, b = (torch.from_numpy(v).double() for v in (x, At, Bt))
    lib = (torch.relu(xt @ a.T) @ b.T).numpy()
    np.testing.assert_allclose(s64, lib, rtol=1e-12, atol=1e-15)
    # float32 in the fixed order stays within a forward error bound of the exact value:
    # |err| <= (n1 + n2) * 2^-24 * sum|terms|   (loose)
    bound = (d + r) * 2.0 ** -24 * (xt.abs() @ a.abs().T @ b.abs().T).numpy()
    assert np.all(np.abs(s.astype(np.float64) - lib) <= bound)
    assert np.max(np.abs(s - lib)) <= 1e-5 * np.max(np.abs(lib)) + 1e-7


def _one_dot(a, b):
    """dot(a,b) through the first predictor layer, read back through an identity second layer."""
    n = len(a)
    At = np.asarray(b, dtype=np.float32).reshape(1, n)
    Bt = np.ones((1, 1), dtype=np.float32)
    return float(ref.predict_scores(np.asarray(a, np.float32).reshape(1, n), At, Bt)[0, 0])


def test_partial_sums_are_interleaved_by_blocks_of_8():
    # elements 0 and 512 fall in the same partial sum (slot 0); 8 and 16 in slots 1 and 2
    n = 1024
    a = np.zeros(n, np.float32)
    b = np.ones(n, np.float32)
    a[0], a[512], a[8], a[16] = 2.0 ** 24, -(2.0 ** 24), 1.0, 1.0
    assert _one_dot(a, b) == 2.0          # a left-to-right float32 sum gives 0
    # elements 0..7 share one slot: 2^24 then eight ones are each absorbed
    a = np.zeros(n, np.float32)
    a[0] = 2.0 ** 24
    a[1:8] = 1.0
    a[8] = 1.0                            # slot 1: survives until the combination
    assert _one_dot(a, b) == 2.0 ** 24    # 2^24 + 1 ties to even -> 2^24


def test_combination_starts_at_distance_32():
    n = 512
    a = np.zeros(n, np.float32)
    b = np.ones(n, np.float32)
    a[0] = 2.0 ** 24          # slot 0
    a[256] = -(2.0 ** 24)     # slot 32: cancels slot 0 in the first round
    a[8] = 1.0                # slot 1
    assert _one_dot(a, b) == 1.0   # distance-1-first would lose the 1
    # and distance 16 before 8: slots 0,16 cancel in round two, slot 8 then survives
    a = np.zeros(n, np.float32)
    a[0], a[16 * 8], a[8 * 8] = 2.0 ** 24, -(2.0 ** 24), 1.0
    assert _one_dot(a, b) == 1.0


def test_multiply_add_is_fused():
    n = 1024
    a = np.zeros(n, np.float32)
    b = np.zeros(n, np.float32)
    a[0], b[0] = -(1 + 2.0 ** -11), 1.0
    a[512] = b[512] = 1 + 2.0 ** -12      # exact square = 1 + 2^-11 + 2^-24
    # the value is positive, so it passes the ReLU
    assert _one_dot(a, b) == 2.0 ** -24   # an unfused multiply rounds the square first -> 0


def test_relu_sits_between_the_layers_and_tokens_are_independent():
    rng = np.random.default_rng(9)
    T, d, r, G = 6, 64, 16, 8
    x = rng.standard_normal((T, d)).astype(np.float32)
    At = rng.standard_normal((r, d)).astype(np.float32)
    Bt = rng.standard_normal((G, r)).astype(np.float32)
    s = ref.predict_scores(x, At, Bt)
    perm = rng.permutation(T)
    assert np.array_equal(ref.predict_scores(x[perm], At, Bt), s[perm])
    # negating x changes which hidden units pass: s(x)+s(-x) = |xA| B, not 0
    s2 = ref.predict_scores(-x, At, Bt)
    lib = np.abs(x.astype(np.float64) @ At.T.astype(np.float64)) @ Bt.T.astype(np.float64)
    np.testing.assert_allclose(s.astype(np.float64) + s2, lib, rtol=1e-4, atol=1e-4)
