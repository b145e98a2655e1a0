"""The allocation-free entry point halo_ffn_forward_static (scratch = a fixed array inside the
library) against halo_ffn_forward with a caller workspace: same kernels, so every output must be
identical bit for bit.  Two calls in a row share the array, the second with a smaller input."""
import dataclasses

import numpy as np
import pytest
import torch

import halo_synth as hs
import paper_2601_11676_amd as H
from tests import harness as hz

pytestmark = pytest.mark.gpu

OUTS = ("y", "scores", "order", "group_dev", "mask", "surv_idx", "n_surv")


def _static_forward(w, layer, x, K, prio_dev_np, drop_np):
    s = hz.shape_of(w)
    T, G = x.shape[0], w.n_groups
    pd = torch.from_numpy(np.ascontiguousarray(prio_dev_np)).to(hz.DEV)
    dr = torch.from_numpy(np.ascontiguousarray(drop_np)).to(hz.DEV)
    y = torch.full((T, w.d), float("nan"), dtype=w.torch_dtype, device=hz.DEV)
    scores = torch.empty((T, G), dtype=torch.float32, device=hz.DEV)
    order = torch.empty((T, G), dtype=torch.int32, device=hz.DEV)
    group_dev = torch.empty((T, G), dtype=torch.int8, device=hz.DEV)
    mask = torch.empty((T, G), dtype=torch.uint8, device=hz.DEV)
    surv_idx = torch.empty((T, K), dtype=torch.int32, device=hz.DEV)
    n_surv = torch.empty((T,), dtype=torch.int32, device=hz.DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    H.halo_ffn_forward_static(s, x, layer.At, layer.Bt, layer.Wg, layer.Wu, layer.Wd, K, pd, w.n_dev, dr, y,
                              scores=scores, order=order, group_dev=group_dev, mask=mask, surv_idx=surv_idx,
                              n_surv=n_surv)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return dict(y=hz.to_np32(y).astype(np.float64), scores=scores.cpu().numpy(), order=order.cpu().numpy(),
                group_dev=group_dev.cpu().numpy(), mask=mask.cpu().numpy(), surv_idx=surv_idx.cpu().numpy(),
                n_surv=n_surv.cpu().numpy())


def test_static_scratch_entry_point_equals_the_workspace_one_on_two_calls_in_a_row():
    cases = [
        dataclasses.replace(hs.LLAMA70B_STACK, name="case", ffn=24 * 128, layers=1, T=8, seed=51),   # matrix cores
        dataclasses.replace(hs.LLAMA7B_DECODE, name="case", ffn=20 * 128, T=1, seed=52),             # smaller: one token
        dataclasses.replace(hs.LLAMA7B_PREFILL, name="case", d=512, ffn=7 * 128, rank=64, T=40, seed=53),
        dataclasses.replace(hs.TINY, name="case", T=5, seed=54),                                     # float32, generic
    ]
    for w in cases:
        print(f"[case] static scratch: d={w.d} G={w.n_groups} T={w.T} {w.dtype}", flush=True)
        L = hz.Layer(w)
        x = hs.hidden_states(w, 0, hz.DEV)
        K = max(1, w.n_groups // 2)
        pd = H.halo_build_schedule(K, w.device_plr())
        drop = hs.drop_outcomes(w, T=w.T)
        a = _static_forward(w, L, x, K, pd, drop)
        b = hz.gpu_forward(w, L, x, K, pd, drop)
        for k in OUTS:
            assert np.array_equal(a[k], b[k]), (w.d, w.T, k)
        assert a["mask"].any()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    w = hs.LLAMA7B_PREFILL
    s = hz.shape_of(w)
    assert H.halo_workspace_bytes(s, w.T, w.k_keep()) > H.halo_static_scratch_bytes()
    L = hz.Layer(dataclasses.replace(w, ffn=2 * 128))          # pointers only: the call is refused before any use
    x = hs.hidden_states(w, 0, hz.DEV)
    y = torch.full((w.T, w.d), 7.0, dtype=torch.bfloat16, device=hz.DEV)
    pd = torch.from_numpy(H.halo_build_schedule(w.k_keep(), w.device_plr())).to(hz.DEV)
    with pytest.raises(H.HaloError) as e:
        H.halo_ffn_forward_static(s, x, L.At, L.Bt, L.Wg, L.Wu, L.Wd, w.k_keep(), pd, w.n_dev, None, y)
    assert e.value.code == -5
    torch.cuda.synchronize()
    assert (y == 7.0).all()
