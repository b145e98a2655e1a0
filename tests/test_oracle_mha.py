"""Pins for the oracle's head-sparse attention decode step (paper Sec. II-A: one head and its
output-projection slice are one neuron group, merge = sum; Sec. III-B.3: full KV cache)."""
import dataclasses
import math

import numpy as np
import torch
import torch.nn.functional as F

import halo_synth as hs
from oracle import ref


def _case(seed, d=48, H=3, dh=8, max_len=9):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(d).astype(np.float32)
    Wq, Wk, Wv, WoT = (rng.standard_normal((H * dh, d)).astype(np.float32) * 0.3 for _ in range(4))
    kc = rng.standard_normal((H, max_len, dh)).astype(np.float32)
    vc = rng.standard_normal((H, max_len, dh)).astype(np.float32)
    return x, Wq, Wk, Wv, WoT, kc, vc


def test_all_heads_equal_library_scaled_dot_product_attention():
    for seed, pos in ((0, 0), (1, 4), (2, 8)):
        x, Wq, Wk, Wv, WoT, kc, vc = _case(seed)
        H, max_len, dh = kc.shape
        k0, v0 = kc.copy(), vc.copy()
        y = ref.mha_decode(x, Wq, Wk, Wv, WoT, kc, vc, pos, None, cache_is_bf16=False)
        # the library's view: float64, caches with the new row appended by a float64 matmul
        xd = torch.from_numpy(x).double()
        q = (torch.from_numpy(Wq).double() @ xd).view(H, 1, dh)
        K = torch.from_numpy(k0).double()[:, :pos + 1].clone()
        V = torch.from_numpy(v0).double()[:, :pos + 1].clone()
        K[:, pos] = (torch.from_numpy(Wk).double() @ xd).view(H, dh).float().double()
        V[:, pos] = (torch.from_numpy(Wv).double() @ xd).view(H, dh).float().double()
        o = F.scaled_dot_product_attention(q, K, V)                    # [H][1][dh], scale 1/sqrt(dh)
        want = o.reshape(-1) @ torch.from_numpy(WoT).double()
        np.testing.assert_allclose(y, want.numpy(), rtol=1e-9, atol=1e-12)
        # cache: row pos rewritten, everything else untouched
        assert np.array_equal(np.delete(kc, pos, axis=1), np.delete(k0, pos, axis=1))
        assert np.array_equal(np.delete(vc, pos, axis=1), np.delete(v0, pos, axis=1))
        np.testing.assert_allclose(kc[:, pos].reshape(-1), Wk.astype(np.float64) @ x, rtol=1e-6)


def test_first_position_is_linear_in_v():
    # one cached position: softmax over a single score is 1, so y = WoT^T (Wv x) for every head
    x, Wq, Wk, Wv, WoT, kc, vc = _case(3)
    y = ref.mha_decode(x, Wq, Wk, Wv, WoT, kc, vc, 0, None, cache_is_bf16=False)
    v = (Wv.astype(np.float64) @ x).astype(np.float32).astype(np.float64)
    np.testing.assert_allclose(y, v @ WoT.astype(np.float64), rtol=1e-12, atol=1e-14)


def test_zero_query_gives_the_mean_of_the_values():
    x, Wq, Wk, Wv, WoT, kc, vc = _case(4)
    H, max_len, dh = kc.shape
    pos = 5
    y = ref.mha_decode(x, np.zeros_like(Wq), Wk, Wv, WoT, kc, vc, pos, None, cache_is_bf16=False)
    o = vc[:, :pos + 1].astype(np.float64).mean(axis=1).reshape(-1)          # vc already holds the new row
    np.testing.assert_allclose(y, o @ WoT.astype(np.float64), rtol=1e-12, atol=1e-14)


def test_scale_is_one_over_sqrt_head_dim_hand_case():
    # one head of dimension 4, two positions: q = (2,0,0,0); k_0 = (1,0,0,0), new k_1 = (3,0,0,0);
    # scores 2/2 and 6/2 -> p_1 = 1/(1+exp(-2)); v_0 = e_0, v_1 = e_1; WoT = identity on 4 outputs
    d = dh = 4
    x = np.array([1, 0, 0, 0], np.float32)
    Wq = np.zeros((4, 4), np.float32); Wq[0, 0] = 2
    Wk = np.zeros((4, 4), np.float32); Wk[0, 0] = 3
    Wv = np.zeros((4, 4), np.float32); Wv[1, 0] = 1
    WoT = np.eye(4, dtype=np.float32)
    kc = np.zeros((1, 2, 4), np.float32); kc[0, 0, 0] = 1
    vc = np.zeros((1, 2, 4), np.float32); vc[0, 0, 0] = 1
    y = ref.mha_decode(x, Wq, Wk, Wv, WoT, kc, vc, 1, None, cache_is_bf16=False)
    p1 = 1.0 / (1.0 + math.exp(-2.0))
    np.testing.assert_allclose(y, [1 - p1, p1, 0, 0], rtol=1e-14, atol=1e-16)


def test_heads_are_independent_groups_and_masked_heads_add_exact_zero():
    x, Wq, Wk, Wv, WoT, kc, vc = _case(5, H=4)
    pos = 6
    full = ref.mha_decode(x, Wq, Wk, Wv, WoT, kc.copy(), vc.copy(), pos, None, cache_is_bf16=False)
    parts = []
    for h in range(4):
        m = np.zeros(4, np.uint8); m[h] = 1
        k2, v2 = kc.copy(), vc.copy()
        parts.append(ref.mha_decode(x, Wq, Wk, Wv, WoT, k2, v2, pos, m, cache_is_bf16=False))
        # keys and values are produced for every head, whatever the mask (full KV cache)
        k3, v3 = kc.copy(), vc.copy()
        ref.mha_decode(x, Wq, Wk, Wv, WoT, k3, v3, pos, None, cache_is_bf16=False)
        assert np.array_equal(k2, k3) and np.array_equal(v2, v3)
    np.testing.assert_allclose(sum(parts), full, rtol=1e-12, atol=1e-14)
    none = ref.mha_decode(x, Wq, Wk, Wv, WoT, kc.copy(), vc.copy(), pos, np.zeros(4, np.uint8), cache_is_bf16=False)
    assert not none.any()
    # a masked head's query and output weights are never used
    Wq2, Wo2 = Wq.copy(), WoT.copy()
    Wq2[8:16] = np.nan; Wo2[8:16] = np.nan
    m = np.array([1, 0, 1, 1], np.uint8)
    a = ref.mha_decode(x, Wq, Wk, Wv, WoT, kc.copy(), vc.copy(), pos, m, cache_is_bf16=False)
    b = ref.mha_decode(x, Wq2, Wk, Wv, Wo2, kc.copy(), vc.copy(), pos, m, cache_is_bf16=False)
    assert np.array_equal(a, b)


def test_new_cache_rows_are_rounded_to_bf16_nearest_even():
    x, Wq, Wk, Wv, WoT, kc, vc = _case(6)
    pos = 3
    ref.mha_decode(x, Wq, Wk, Wv, WoT, kc, vc, pos, None, cache_is_bf16=True)
    exact = (Wk.astype(np.float64) @ x)
    lib = torch.from_numpy(exact.astype(np.float32)).to(torch.bfloat16).float().numpy()   # library rounding
    assert np.array_equal(kc[:, pos].reshape(-1), lib)


def test_softmax_is_shift_invariant_for_large_scores():
    # scores around +-2000 must not overflow: the maximum is subtracted before exponentiation
    x, Wq, Wk, Wv, WoT, kc, vc = _case(7)
    y = ref.mha_decode(x, Wq * 400, Wk, Wv, WoT, kc * 10, vc, 8, None, cache_is_bf16=False)
    assert np.isfinite(y).all()


def test_workload_generator_shapes():
    w = dataclasses.replace(hs.LLAMA7B_MHA_DECODE, d=128, n_heads=4, head_dim=16, max_len=12, ctx=7, rank=16)
    Wq, Wk, Wv, WoT = hs.mha_weights(w)
    kc, vc = hs.kv_cache(w)
    assert Wq.shape == (64, 128) and kc.shape == (4, 12, 16) and vc.dtype == torch.bfloat16
    assert hs.LLAMA7B_MHA_DECODE.k_keep() == 16
    assert not torch.equal(Wq, Wk) and not torch.equal(kc, vc)
