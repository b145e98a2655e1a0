"""GPU parity of the FFN over 4-bit block-quantised weights (paper Sec. V-A) against the CPU
oracle, whose view of such weights is the dequantised matrices.  Same bars as the other
parity tests: bit-exact scores / ranking / masks, relative L2 <= 1e-5 (f32) or 2e-2 (bf16)."""
import dataclasses

import numpy as np
import pytest
import torch

import halo_synth as hs
import paper_2601_11676_amd as H
from oracle import ref
from tests import harness as hz

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def _say(msg):
    print("[case] " + msg, flush=True)


def test_q4_generator_bits_identical_on_cpu_and_gpu():
    _say("q4 generator cpu/gpu")
    w = hs.small_variant(hs.LLAMA7B_DECODE, 384, 3, 64)
    for a, b in zip(hs.ffn_weights_q4(w, 1, "cpu"), hs.ffn_weights_q4(w, 1, hz.DEV)):
        b = b.cpu()
        if a.dtype == torch.bfloat16:
            a, b = a.view(torch.int16), b.view(torch.int16)
        assert torch.equal(a, b)


@pytest.mark.parametrize("dtype,T,d,G,r", [
    ("f32", 16, 256, 8, 64),       # the tiny shape
    ("f32", 5, 640, 7, 72),
    ("bf16", 3, 384, 9, 40),
    ("bf16", 1, 1024, 5, 264),     # one token, but not a row length of the streaming path
    ("bf16", 7, 4096, 6, 256),
    ("bf16", 40, 512, 70, 64),     # more groups than a wave, many tokens
])
def test_q4_plain_path_whole_pass(dtype, T, d, G, r):
    w = dataclasses.replace(hs.TINY, name="case", d=d, ffn=G * 128, rank=r, T=T, dtype=dtype, seed=12)
    _say(f"q4 plain {dtype} T={T} d={d} G={G} r={r}")
    L = hz.Q4Layer(w)
    x = hs.hidden_states(w, 0, hz.DEV)
    K = max(1, G // 2)
    pd = H.halo_build_schedule(K, w.device_plr())
    drop = hs.drop_outcomes(w, T=T)
    g = hz.gpu_forward_q4(w, L, x, K, pd, drop)
    c = hz.oracle_forward(w, L, x, K, pd, drop)
    hz.assert_parity(g, c, TOL[dtype], "q4 plain")


@pytest.mark.parametrize("d,G,K", [(4096, 7, 4), (8192, 6, 6), (4096, 200, 150), (4096, 9, 1)])
def test_q4_one_token_streaming_path(d, G, K):
    w = dataclasses.replace(hs.LLAMA7B_DECODE, name="case", d=d, ffn=G * 128, rank=256, seed=22)
    _say(f"q4 one-token path d={d} G={G} K={K}")
    L = hz.Q4Layer(w)
    pd = H.halo_build_schedule(K, w.device_plr())
    for step in range(3):
        x = hs.hidden_states(w, step, hz.DEV)
        drop = hs.drop_outcomes(w, 0, step)
        g = hz.gpu_forward_q4(w, L, x, K, pd, drop)
        c = hz.oracle_forward(w, L, x, K, pd, drop)
        hz.assert_parity(g, c, TOL["bf16"], f"q4 t1 d={d} step {step}")


@pytest.mark.parametrize("T,d,G,r", [
    (2, 1024, 5, 64),
    (4, 5120, 9, 256),       # LLaMA-13B row length (ten 512-element chunks: the last code buffer is half full)
    (8, 8192, 7, 512),       # LLaMA-2-70B row length
    (16, 4096, 6, 256),
    (5, 4096, 20, 256),      # union larger than any token's set; ragged neuron runs per wave
    (3, 512, 3, 40),         # a single chunk per row
    (6, 5120, 90, 256),      # more 16-row tiles than workgroups: a workgroup walks several
    (16, 8192, 40, 256),     # x larger than its LDS space: staged a range of columns at a time, per tile
    (17, 1024, 9, 64),       # more than 16 tokens: tiles of tokens, here 15 + 2 (no tile of one token)
    (33, 2048, 12, 64),      # 16 + 15 + 2
    (100, 1024, 20, 40),     # six tiles of 16 and one of 4
])
def test_q4_few_tokens_matrix_core_path(T, d, G, r):
    w = dataclasses.replace(hs.LLAMA13B_STACK, name="case", d=d, ffn=G * 128, rank=r, T=T, layers=1, seed=18)
    _say(f"q4 few tokens T={T} d={d} G={G}")
    L = hz.Q4Layer(w)
    x = hs.hidden_states(w, 0, hz.DEV)
    for K in (max(1, G // 2), G):
        pd = H.halo_build_schedule(K, w.device_plr())
        drop = hs.drop_outcomes(w, T=T)
        if K < G:
            drop[T - 1] = 1                    # one token loses every device: exact zeros expected
        g = hz.gpu_forward_q4(w, L, x, K, pd, drop)
        c = hz.oracle_forward(w, L, x, K, pd, drop)
        hz.assert_parity(g, c, TOL["bf16"], f"q4 few tokens K={K}")


def test_q4_llama7b_decode_full_size_steps():
    w = hs.LLAMA7B_DECODE
    _say("q4 llama7b decode full size")
    L = hz.Q4Layer(w)
    K = w.k_keep()
    pd = H.halo_build_schedule(K, w.device_plr())
    for step in (0, 1, 2, 3, 7, 100, 500, 1023):
        x = hs.hidden_states(w, step, hz.DEV)
        drop = hs.drop_outcomes(w, 0, step)
        g = hz.gpu_forward_q4(w, L, x, K, pd, drop)
        c = hz.oracle_forward(w, L, x, K, pd, drop)
        hz.assert_parity(g, c, TOL["bf16"], f"q4 7b step {step}")


def test_q4_ffn_entry_point_with_handmade_masks_and_errors():
    w = dataclasses.replace(hs.LLAMA7B_DECODE, name="case", ffn=10 * 128, rank=64, seed=23)
    _say("q4 ffn entry point, handmade masks")
    L = hz.Q4Layer(w)
    s = hz.shape_of(w)
    _, _, Wg, Wu, WdT = L.host()
    ws = torch.empty(H.halo_workspace_bytes(s, 1, 0), dtype=torch.uint8, device=hz.DEV)
    x = hs.hidden_states(w, 3, hz.DEV)
    xn = hz.to_np32(x)
    for bits in ([0] * 10, [1] * 10, [1, 0, 0, 0, 0, 0, 0, 0, 0, 1], [0, 0, 0, 0, 1, 0, 0, 0, 0, 0]):
        mask_np = np.array([bits], np.uint8)
        y = torch.full((1, w.d), float("nan"), dtype=torch.bfloat16, device=hz.DEV)
        H.halo_group_sparse_ffn_q4(s, x, L.q4, torch.from_numpy(mask_np).to(hz.DEV), y, ws)
        torch.cuda.synchronize()
        yg = hz.to_np32(y).astype(np.float64)
        yc = ref.group_sparse_ffn(xn, Wg, Wu, WdT, 128, mask_np)
        if not any(bits):
            assert not yg.any()
        else:
            assert np.linalg.norm(yg - yc) / np.linalg.norm(yc) <= TOL["bf16"]
    # a group size other than the quantisation block is refused before anything is enqueued
    bad = H.Shape(w.d, 20 * 64, 64, w.rank, "bf16")
    y = torch.zeros((1, w.d), dtype=torch.bfloat16, device=hz.DEV)
    with pytest.raises(H.HaloError):
        H.halo_group_sparse_ffn_q4(bad, x, L.q4, torch.zeros((1, 20), dtype=torch.uint8, device=hz.DEV), y, ws)
    # no tokens: nothing to do
    H.halo_group_sparse_ffn_q4(s, x[:0], L.q4, torch.zeros((0, 10), dtype=torch.uint8, device=hz.DEV), y[:0], ws)
    torch.cuda.synchronize()


@pytest.mark.parametrize("T,d,G", [(2, 8192, 6), (4, 5120, 10), (16, 4096, 5), (3, 1024, 70)])
def test_q4_few_tokens_with_handmade_masks(T, d, G):
    # the matrix-core kernels on masks no schedule would give: no group at all (exact zeros), one group of one
    # token, every group of every token, a different single group per token, the last group only
    w = dataclasses.replace(hs.LLAMA13B_STACK, name="case", d=d, ffn=G * 128, rank=64, T=T, layers=1, seed=31)
    _say(f"q4 few tokens, handmade masks T={T} d={d} G={G}")
    L = hz.Q4Layer(w)
    s = hz.shape_of(w)
    _, _, Wg, Wu, WdT = L.host()
    ws = torch.empty(H.halo_workspace_bytes(s, T, G), dtype=torch.uint8, device=hz.DEV)
    x = hs.hidden_states(w, 1, hz.DEV)
    xn = hz.to_np32(x)
    masks = [np.zeros((T, G), np.uint8), np.zeros((T, G), np.uint8), np.ones((T, G), np.uint8),
             np.zeros((T, G), np.uint8), np.zeros((T, G), np.uint8)]
    masks[1][T - 1, G // 2] = 1
    for t in range(T):
        masks[3][t, (3 * t + 1) % G] = 1
    masks[4][:, G - 1] = 1
    for mask_np in masks:
        y = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device=hz.DEV)
        H.halo_group_sparse_ffn_q4(s, x, L.q4, torch.from_numpy(mask_np).to(hz.DEV), y, ws)
        torch.cuda.synchronize()
        yg = hz.to_np32(y).astype(np.float64)
        yc = ref.group_sparse_ffn(xn, Wg, Wu, WdT, 128, mask_np)
        for t in range(T):
            if not mask_np[t].any():
                assert not yg[t].any(), t
            else:
                assert np.linalg.norm(yg[t] - yc[t]) / np.linalg.norm(yc[t]) <= TOL["bf16"], t


@pytest.mark.parametrize("d,T,r,G,K", [
    (4096, 1, 256, 20, 10), (8192, 1, 256, 20, 10), (512, 3, 256, 20, 10), (5120, 4, 256, 20, 10),
    (8192, 8, 256, 20, 10), (384, 3, 256, 20, 10),
    (4096, 1, 256, 86, 43),      # enough surviving neurons for the runs to be cut by weight around the predictor rows
    (4096, 1, 512, 86, 60),      # two predictor rows per gate/up workgroup
    (4096, 1, 128, 20, 10),      # a predictor size that is not dealt evenly: workgroups of its own
    (1024, 20, 64, 12, 6),       # more than 16 tokens: tiles of tokens, the prediction enqueued after the FFN
])
def test_q4_one_step_ahead_overlap_equals_the_serial_pass(d, T, r, G, K):
    # predictor + mask of step s+1 beside (or, for shapes without spare workgroups, after) the FFN of step s
    w = dataclasses.replace(hs.LLAMA7B_DECODE, name="case", d=d, ffn=G * 128, rank=r, T=T, seed=9)
    _say(f"halo_ffn_forward_ahead_q4 vs halo_ffn_forward_q4 d={d} T={T} r={r} G={G} K={K}")
    s = hz.shape_of(w)
    L = hz.Q4Layer(w)
    n = 5
    pd = H.halo_build_schedule(K, w.device_plr())
    xs = [hs.hidden_states(w, i, hz.DEV) for i in range(n + 1)]
    drops = [hs.drop_outcomes(w, 0, i, T=T) for i in range(n + 1)]
    serial = [hz.gpu_forward_q4(w, L, xs[i], K, pd, drops[i]) for i in range(n)]
    ws = torch.empty(H.halo_workspace_bytes(s, T, K), dtype=torch.uint8, device=hz.DEV)
    pdd = torch.from_numpy(pd).to(hz.DEV)
    dd = [torch.from_numpy(x).to(hz.DEV) for x in drops]
    masks = torch.zeros((n + 1, T, G), dtype=torch.uint8, device=hz.DEV)
    ys = torch.zeros((n, T, w.d), dtype=torch.bfloat16, device=hz.DEV)
    sc = torch.empty((T, G), dtype=torch.float32, device=hz.DEV)
    H.halo_predict_scores(s, xs[0], L.At, L.Bt, sc, ws)
    H.halo_build_group_mask(sc, K, pdd, w.n_dev, dd[0], masks[0])

    def run(ys_, masks_):
        for i in range(n):
            H.halo_ffn_forward_ahead_q4(s, xs[i], L.q4, masks_[i], ys_[i], xs[i + 1], L.At, L.Bt, K, pdd,
                                        w.n_dev, dd[i + 1], masks_[i + 1], ws)

    run(ys, masks)
    torch.cuda.synchronize()
    for i in range(n):
        assert np.array_equal(masks[i].cpu().numpy(), serial[i]["mask"]), i
        assert np.array_equal(hz.to_np32(ys[i]).astype(np.float64), serial[i]["y"]), i
    g = torch.cuda.CUDAGraph()
    ys2 = torch.zeros_like(ys)
    masks2 = masks.clone()
    with torch.cuda.graph(g):
        run(ys2, masks2)
    for _ in range(2):
        ys2.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(ys2, ys) and torch.equal(masks2, masks)


@pytest.mark.parametrize("wl", [hs.LLAMA13B_STACK, hs.LLAMA70B_STACK])
def test_q4_full_size_single_layer_of_the_stacks(wl):
    # 4 / 8 tokens at the 13B / 70B layer shapes (the plain 4-bit path); y for every token
    _say(f"q4 {wl.name} one full-size layer")
    L = hz.Q4Layer(wl, layer=2)
    x = hs.hidden_states(wl, 0, hz.DEV)
    K = wl.k_keep(0.5)
    pd = H.halo_build_schedule(K, wl.device_plr())
    drop = hs.drop_outcomes(wl, 2, 0)
    g = hz.gpu_forward_q4(wl, L, x, K, pd, drop)
    c = hz.oracle_forward(wl, L, x, K, pd, drop)
    hz.assert_parity(g, c, TOL["bf16"], "q4 " + wl.name)


@pytest.mark.parametrize("big_workspace", [False, True])
def test_q4_llama7b_prefill_all_tokens(big_workspace):
    # 512 tokens over 4-bit weights: with the plain workspace the few-token kernels walk the tokens 16 at a
    # time; with room for a block's weights as bf16 they are expanded once and the bf16 kernels run
    w = hs.LLAMA7B_PREFILL
    _say(f"q4 7B prefill, 512 tokens, every token, big workspace {big_workspace}")
    s = hz.shape_of(w)
    K = w.k_keep()
    small, big = H.halo_workspace_bytes(s, w.T, K), H.halo_workspace_bytes_q4(s, w.T, K)
    assert big == small + 3 * w.ffn * w.d * 2 and H.halo_workspace_bytes_q4(s, 16, K) == H.halo_workspace_bytes(s, 16, K)
    L = hz.Q4Layer(w)
    x = hs.hidden_states(w, 0, hz.DEV)
    pd = H.halo_build_schedule(K, w.device_plr())
    drop = hs.drop_outcomes(w)
    g = hz.gpu_forward_q4(w, L, x, K, pd, drop, big_workspace=big_workspace)
    c = hz.oracle_forward(w, L, x, K, pd, drop)
    hz.assert_parity(g, c, TOL["bf16"], "q4 7B prefill")


@pytest.mark.parametrize("T,d,G", [(17, 1024, 9), (40, 2048, 12), (300, 1024, 20)])
def test_q4_many_tokens_on_expanded_weights(T, d, G):
    # small shapes through the expansion to bf16 (workspace of halo_workspace_bytes_q4)
    w = dataclasses.replace(hs.LLAMA13B_STACK, name="case", d=d, ffn=G * 128, rank=64, T=T, layers=1, seed=19)
    _say(f"q4 many tokens, expanded weights T={T} d={d} G={G}")
    L = hz.Q4Layer(w)
    x = hs.hidden_states(w, 0, hz.DEV)
    K = max(1, G // 2)
    pd = H.halo_build_schedule(K, w.device_plr())
    drop = hs.drop_outcomes(w, T=T)
    g = hz.gpu_forward_q4(w, L, x, K, pd, drop, big_workspace=True)
    c = hz.oracle_forward(w, L, x, K, pd, drop)
    hz.assert_parity(g, c, TOL["bf16"], "q4 many tokens expanded")


@pytest.mark.parametrize("wl,keep,layers", [(hs.LLAMA13B_STACK, 0.3, None), (hs.LLAMA70B_STACK, 0.5, 6)])
def test_q4_stack_teacher_forced(wl, keep, layers):
    # the free-running stack over 4-bit weights, predictor one layer ahead (layer 0 dense: every group of
    # every token, so the few-token kernels walk several tiles per workgroup); checked layers are compared
    # with the oracle fed the GPU's own layer inputs
    n = wl.layers if layers is None else layers
    check = sorted({0, 1, 2, n // 2, n - 1})
    _say(f"q4 {wl.name} stack of {n} layers, checked {check}")
    seen = []

    def on_layer(l, rec, pd_np, K):
        hz.check_stack_layer(wl, l, rec, pd_np, K, TOL["bf16"])
        seen.append(l)
        print(f"  layer {l} ok", flush=True)
    h = hz.run_stack_gpu(wl, keep, layers=layers, check_layers=check, on_layer=on_layer, q4=True)
    assert torch.isfinite(h).all() and seen == check

