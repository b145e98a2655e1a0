"""The seeded input generator: determinism, distribution, workload shapes."""
import numpy as np
import torch

import halo_synth as hs


def test_reproducible_and_chunk_independent():
    k = hs.stream_key(7, hs.TID_WG, 3)
    a = hs.normal((1000, 37), 0.02, torch.bfloat16, k)
    b = hs.normal((1000, 37), 0.02, torch.bfloat16, k, chunk=4099)
    assert torch.equal(a, b)
    c = hs.normal((1000, 37), 0.02, torch.bfloat16, hs.stream_key(7, hs.TID_WU, 3))
    assert not torch.equal(a, c)


def test_distribution():
    z = hs.normal((1 << 20,), 1.0, torch.float32, hs.stream_key(1, hs.TID_X)).double()
    assert abs(z.mean()) < 5e-3 and abs(z.std() - 1.0) < 5e-3
    assert abs((z.abs() < 1.0).double().mean() - 0.6827) < 3e-3
    w = hs.normal((1 << 18,), 0.02, torch.bfloat16, hs.stream_key(1, hs.TID_WG)).double()
    assert abs(w.std() - 0.02) < 3e-4
    u = hs.uniform01(1 << 18, hs.stream_key(1, hs.TID_DROP))
    assert u.min() >= 0 and u.max() < 1 and abs(u.mean() - 0.5) < 5e-3


def test_workload_shapes_match_the_configs():
    assert [w.n_groups for w in hs.WORKLOADS] == [8, 86, 108, 86, 224]
    assert hs.TINY.k_keep() == 4 and hs.LLAMA7B_DECODE.k_keep() == 43
    assert [hs.LLAMA13B_STACK.k_keep(k) for k in (0.3, 0.5, 0.7)] == [32, 54, 76]
    assert hs.LLAMA70B_STACK.k_keep() == 112
    plr = hs.LLAMA13B_STACK.device_plr()
    assert plr.shape == (6,) and (plr >= 0).all() and (plr <= 0.3).all()
    x = hs.hidden_states(hs.TINY)
    assert x.shape == (16, 256) and x.dtype == torch.float32
    d = hs.drop_outcomes(hs.LLAMA7B_DECODE, 0, 0, T=4000)
    assert np.all(np.abs(d.mean(0) - [0, .05, .1, .2]) < 0.02) and d[:, 0].sum() == 0
