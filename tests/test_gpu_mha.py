"""GPU parity of the head-sparse attention decode step (paper Sec. II-A: one head + its
output-projection slice = one neuron group) against the CPU oracle.  Scores / ranking / mask
over the heads bit-exact; the new cache rows within one bf16 rounding step of the oracle's
(both sides round a float accumulation of the same products; at a rounding boundary they may
land on neighbouring values); y within relative L2 2e-2."""
import dataclasses

import numpy as np
import pytest
import torch

import halo_synth as hs
import paper_2601_11676_amd as H
from oracle import ref
from tests import harness as hz

pytestmark = pytest.mark.gpu
TOL = 2e-2


def _say(msg):
    print("[case] " + msg, flush=True)


class MhaLayer:
    def __init__(self, w):
        self.w = w
        self.Wq, self.Wk, self.Wv, self.WoT = hs.mha_weights(w, 0, hz.DEV)
        self.Wo = H.pack_down_proj(self.WoT, w.head_dim)
        self.At, self.Bt = hs.mha_predictor_weights(w, 0, hz.DEV)
        self.shape = H.MhaShape(w.d, w.n_heads, w.head_dim, w.rank, w.dtype)
        self.host = tuple(hz.to_np32(t) for t in (self.Wq, self.Wk, self.Wv, self.WoT, self.At, self.Bt))


def _one_bf16_step(a, b):
    """|a - b| <= one bf16 spacing at that magnitude."""
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(b64), 1e-30))) - 7)
    return np.all(np.abs(a64 - b64) <= ulp + 1e-30)


def _check_step(L, x, kc, vc, pos, K, pd, drop):
    """One halo_mha_forward call on device caches kc / vc (updated in place) against the oracle
    fed the same caches as they were before the call."""
    w = L.w
    Hh = w.n_heads
    Wq, Wk, Wv, WoT, At, Bt = L.host
    k_ref, v_ref = hz.to_np32(kc).copy(), hz.to_np32(vc).copy()
    ws = torch.empty(H.halo_mha_workspace_bytes(L.shape, kc.shape[1]), dtype=torch.uint8, device=hz.DEV)
    pdd = torch.from_numpy(np.ascontiguousarray(pd)).to(hz.DEV)
    dr = None if drop is None else torch.from_numpy(np.ascontiguousarray(drop)).to(hz.DEV)
    y = torch.full((1, w.d), float("nan"), dtype=torch.bfloat16, device=hz.DEV)
    scores = torch.empty((1, Hh), dtype=torch.float32, device=hz.DEV)
    order = torch.empty((1, Hh), dtype=torch.int32, device=hz.DEV)
    mask = torch.empty((1, Hh), dtype=torch.uint8, device=hz.DEV)
    n_surv = torch.empty((1,), dtype=torch.int32, device=hz.DEV)
    H.halo_mha_forward(L.shape, x, L.At, L.Bt, L.Wq, L.Wk, L.Wv, L.Wo, kc, vc, pos, K, pdd, w.n_dev, dr, y, ws,
                       scores=scores, order=order, mask=mask, n_surv=n_surv)
    torch.cuda.synchronize()
    xn = hz.to_np32(x)
    sc = ref.predict_scores(xn, At, Bt)
    m = ref.build_group_mask(sc, K, pd, w.n_dev, drop)
    assert np.array_equal(scores.cpu().numpy().view(np.uint32), sc.view(np.uint32)), "scores"
    assert np.array_equal(order.cpu().numpy(), m["order"]) and np.array_equal(mask.cpu().numpy(), m["mask"])
    assert np.array_equal(n_surv.cpu().numpy(), m["n_surv"])
    yc = ref.mha_decode(xn, Wq, Wk, Wv, WoT, k_ref, v_ref, pos, m["mask"][0])
    kg, vg = hz.to_np32(kc), hz.to_np32(vc)
    # untouched rows identical, the new row within a rounding step
    assert np.array_equal(np.delete(kg, pos, axis=1), np.delete(k_ref, pos, axis=1))
    assert np.array_equal(np.delete(vg, pos, axis=1), np.delete(v_ref, pos, axis=1))
    assert _one_bf16_step(kg[:, pos], k_ref[:, pos]) and _one_bf16_step(vg[:, pos], v_ref[:, pos])
    yg = hz.to_np32(y)[0].astype(np.float64)
    assert np.isfinite(yg).all()
    if m["n_surv"][0] == 0:
        assert not yg.any()
    else:
        err = np.linalg.norm(yg - yc) / np.linalg.norm(yc)
        assert err <= TOL, f"rel L2 {err:.3e}"
    return m


@pytest.mark.parametrize("d,Hh,ctx,max_len", [
    (512, 4, 5, 16),        # plain path (row length not one of the streaming ones), one chunk
    (1024, 7, 200, 300),    # plain path, two chunks, odd head count
    (4096, 6, 0, 8),        # streaming path, first position
    (4096, 9, 127, 129),    # chunk boundary: 128 cached rows + the new one
    (4096, 9, 128, 129),
    (5120, 5, 300, 512),
    (8192, 4, 77, 128),
    (4096, 4, 4500, 4608),   # 36 chunks: more than one batch of value sums in the merge
    (4096, 2, 17000, 17024), # 133 chunks: more chunks than threads in the merge
])
def test_mha_decode_step_whole_pass(d, Hh, ctx, max_len):
    w = dataclasses.replace(hs.LLAMA7B_MHA_DECODE, name="case", d=d, n_heads=Hh, rank=64, ctx=ctx,
                            max_len=max_len, seed=31)
    _say(f"mha d={d} H={Hh} pos={ctx} max_len={max_len}")
    L = MhaLayer(w)
    kc, vc = hs.kv_cache(w, 0, hz.DEV)
    K = max(1, Hh // 2)
    pd = H.halo_build_schedule(K, w.device_plr())
    for step in range(2):
        x = hs.mha_hidden(w, step, hz.DEV)
        _check_step(L, x, kc, vc, ctx + step if ctx + step < max_len else ctx, K, pd, hs.mha_drop_outcomes(w, 0, step))


def test_mha_llama7b_shape_several_positions():
    w = hs.LLAMA7B_MHA_DECODE
    _say("mha llama7b shape")
    L = MhaLayer(w)
    kc, vc = hs.kv_cache(w, 0, hz.DEV)
    K = w.k_keep()
    pd = H.halo_build_schedule(K, w.device_plr())
    seen = set()
    for step, pos in enumerate((w.ctx, w.ctx + 1, 3, 1000)):
        x = hs.mha_hidden(w, step, hz.DEV)
        m = _check_step(L, x, kc, vc, pos, K, pd, hs.mha_drop_outcomes(w, 0, step))
        seen.add(int(m["n_surv"][0]))
    assert max(seen) <= K


def test_mha_entry_point_with_handmade_masks_and_errors():
    w = dataclasses.replace(hs.LLAMA7B_MHA_DECODE, name="case", n_heads=8, rank=64, ctx=40, max_len=64, seed=33)
    _say("mha entry point, handmade masks")
    L = MhaLayer(w)
    Wq, Wk, Wv, WoT, _, _ = L.host
    ws = torch.empty(H.halo_mha_workspace_bytes(L.shape, w.max_len), dtype=torch.uint8, device=hz.DEV)
    x = hs.mha_hidden(w, 2, hz.DEV)
    for bits in ([0] * 8, [1] * 8, [1, 0, 0, 0, 0, 0, 0, 1], [0, 0, 0, 1, 0, 0, 0, 0]):
        kc, vc = hs.kv_cache(w, 0, hz.DEV)
        k_ref, v_ref = hz.to_np32(kc).copy(), hz.to_np32(vc).copy()
        mask_np = np.array(bits, np.uint8)
        y = torch.full((1, w.d), float("nan"), dtype=torch.bfloat16, device=hz.DEV)
        H.halo_head_sparse_mha(L.shape, x, L.Wq, L.Wk, L.Wv, L.Wo, kc, vc, w.ctx,
                               torch.from_numpy(mask_np).to(hz.DEV), y, ws)
        torch.cuda.synchronize()
        yc = ref.mha_decode(hz.to_np32(x), Wq, Wk, Wv, WoT, k_ref, v_ref, w.ctx, mask_np)
        yg = hz.to_np32(y)[0].astype(np.float64)
        # keys and values are written for every head whatever the mask
        assert _one_bf16_step(hz.to_np32(kc)[:, w.ctx], k_ref[:, w.ctx])
        if not any(bits):
            assert not yg.any()
        else:
            assert np.linalg.norm(yg - yc) / np.linalg.norm(yc) <= TOL
    kc, vc = hs.kv_cache(w, 0, hz.DEV)
    y = torch.zeros((1, w.d), dtype=torch.bfloat16, device=hz.DEV)
    mk = torch.ones(8, dtype=torch.uint8, device=hz.DEV)
    with pytest.raises(H.HaloError):        # position outside the cache
        H.halo_head_sparse_mha(L.shape, x, L.Wq, L.Wk, L.Wv, L.Wo, kc, vc, w.max_len, mk, y, ws)
    with pytest.raises(H.HaloError):        # head dimension other than 128
        H.halo_head_sparse_mha(H.MhaShape(w.d, 16, 64, 64), x, L.Wq, L.Wk, L.Wv, L.Wo, kc, vc, 0, mk, y, ws)
    with pytest.raises(H.HaloError):        # workspace too small
        H.halo_head_sparse_mha(L.shape, x, L.Wq, L.Wk, L.Wv, L.Wo, kc, vc, 0, mk, y, ws[:64])


def test_mha_many_steps_free_running_cache_and_graph_replay():
    # 6 consecutive positions on the GPU's own growing cache; the oracle is teacher-forced with the
    # GPU's cache before each step.  Then the same 6 steps captured in a graph and replayed.
    w = dataclasses.replace(hs.LLAMA7B_MHA_DECODE, name="case", n_heads=12, rank=64, ctx=250, max_len=512, seed=34)
    _say("mha free-running steps + graph")
    L = MhaLayer(w)
    K = 6
    pd = H.halo_build_schedule(K, w.device_plr())
    kc, vc = hs.kv_cache(w, 0, hz.DEV)
    k0, v0 = kc.clone(), vc.clone()
    for step in range(6):
        _check_step(L, hs.mha_hidden(w, step, hz.DEV), kc, vc, w.ctx + step, K, pd, hs.mha_drop_outcomes(w, 0, step))
    # graph: y per step, caches restored first
    xs = [hs.mha_hidden(w, s, hz.DEV) for s in range(6)]
    drops = [torch.from_numpy(hs.mha_drop_outcomes(w, 0, s)).to(hz.DEV) for s in range(6)]
    pdd = torch.from_numpy(pd).to(hz.DEV)
    ws = torch.empty(H.halo_mha_workspace_bytes(L.shape, w.max_len), dtype=torch.uint8, device=hz.DEV)

    def run(ys, kc_, vc_):
        for s in range(6):
            H.halo_mha_forward(L.shape, xs[s], L.At, L.Bt, L.Wq, L.Wk, L.Wv, L.Wo, kc_, vc_, w.ctx + s, K, pdd,
                               w.n_dev, drops[s], ys[s], ws)

    ya = torch.zeros((6, 1, w.d), dtype=torch.bfloat16, device=hz.DEV)
    ka, va = k0.clone(), v0.clone()
    run(ya, ka, va)
    torch.cuda.synchronize()
    assert torch.equal(ka, kc) and torch.equal(va, vc)          # run-to-run identical
    yb = torch.zeros_like(ya)
    kb, vb = k0.clone(), v0.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(yb, kb, vb)
    for _ in range(2):
        kb.copy_(k0); vb.copy_(v0); yb.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(yb, ya) and torch.equal(kb, ka) and torch.equal(vb, va)


@pytest.mark.parametrize("d", [4096, 1024])
def test_mha_one_step_ahead_overlap_equals_the_serial_pass(d):
    # attention of step s with the mask predicted one step earlier, predictor + mask of step s+1 beside
    # it (d = 4096: in spare workgroups; d = 1024: enqueued afterwards): same bits as the serial form
    w = dataclasses.replace(hs.LLAMA7B_MHA_DECODE, name="case", d=d, n_heads=10, rank=64, ctx=130, max_len=256, seed=35)
    _say(f"halo_mha_forward_ahead vs halo_mha_forward d={d}")
    L = MhaLayer(w)
    Hh, K, n = w.n_heads, 5, 5
    pd = torch.from_numpy(H.halo_build_schedule(K, w.device_plr())).to(hz.DEV)
    xs = [hs.mha_hidden(w, i, hz.DEV) for i in range(n + 1)]
    dd = [torch.from_numpy(hs.mha_drop_outcomes(w, 0, i)).to(hz.DEV) for i in range(n + 1)]
    ws = torch.empty(H.halo_mha_workspace_bytes(L.shape, w.max_len), dtype=torch.uint8, device=hz.DEV)
    k0, v0 = hs.kv_cache(w, 0, hz.DEV)
    # serial reference on the GPU
    ka, va = k0.clone(), v0.clone()
    ya = torch.zeros((n, 1, w.d), dtype=torch.bfloat16, device=hz.DEV)
    ma = torch.zeros((n + 1, 1, Hh), dtype=torch.uint8, device=hz.DEV)
    for i in range(n):
        H.halo_mha_forward(L.shape, xs[i], L.At, L.Bt, L.Wq, L.Wk, L.Wv, L.Wo, ka, va, w.ctx + i, K, pd, w.n_dev,
                           dd[i], ya[i], ws, mask=ma[i])
    torch.cuda.synchronize()
    # overlapped form
    ffn_shape = H.Shape(w.d, Hh * 128, 128, w.rank, "bf16")
    sc = torch.empty((1, Hh), dtype=torch.float32, device=hz.DEV)
    ws2 = torch.empty(H.halo_workspace_bytes(ffn_shape, 1, K), dtype=torch.uint8, device=hz.DEV)

    def run(yb, mb, kb, vb):
        for i in range(n):
            H.halo_mha_forward_ahead(L.shape, xs[i], L.Wq, L.Wk, L.Wv, L.Wo, kb, vb, w.ctx + i, mb[i], yb[i],
                                     xs[i + 1], L.At, L.Bt, K, pd, w.n_dev, dd[i + 1], mb[i + 1], ws)

    kb, vb = k0.clone(), v0.clone()
    yb = torch.zeros_like(ya)
    mb = torch.zeros_like(ma)
    H.halo_predict_scores(ffn_shape, xs[0], L.At, L.Bt, sc, ws2)
    H.halo_build_group_mask(sc, K, pd, w.n_dev, dd[0], mb[0])
    run(yb, mb, kb, vb)
    torch.cuda.synchronize()
    assert torch.equal(mb[:n], ma[:n]) and torch.equal(yb, ya) and torch.equal(kb, ka) and torch.equal(vb, va)
    # captured and replayed twice
    kc, vc = k0.clone(), v0.clone()
    yc = torch.zeros_like(ya)
    mc = mb.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(yc, mc, kc, vc)
    for _ in range(2):
        kc.copy_(k0); vc.copy_(v0); yc.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(yc, ya) and torch.equal(mc, mb) and torch.equal(kc, ka)


def test_mha_long_context_many_chunks():
    # 8191 cached rows = 64 chunks of 128 per surviving head
    w = dataclasses.replace(hs.LLAMA7B_MHA_DECODE, name="case", n_heads=6, rank=64, ctx=8191, max_len=8192, seed=36)
    _say("mha long context")
    L = MhaLayer(w)
    kc, vc = hs.kv_cache(w, 0, hz.DEV)
    pd = H.halo_build_schedule(3, w.device_plr())
    _check_step(L, hs.mha_hidden(w, 0, hz.DEV), kc, vc, w.ctx, 3, pd, None)
    _check_step(L, hs.mha_hidden(w, 1, hz.DEV), kc, vc, 4095, 6, H.halo_build_schedule(6, w.device_plr()), None)
