#!/usr/bin/env python3
"""Benchmark of the HALO group-sparse FFN path on one MI355X.

One "step" = one whole pass (predictor -> group mask -> group-sparse SwiGLU FFN) over one
batch of synthetic input.  The default workload is the LLaMA-7B-shape single-layer decode:
d=4096, ffn=11008 as 86 groups of 128, bf16, one token per step, 43 groups kept, 4 simulated
devices with loss rates {0, 0.05, 0.1, 0.2}, fresh hidden state and loss outcomes per step.
`--workload` also accepts llama7b_prefill (512 tokens per step, matrix-core roofline),
llama13b_stack and llama70b_stack (one layer of that shape per step, 4 / 8 tokens; with
`--stack` a step is the whole stack, every layer resident, see main_stack), tiny, and
llama7b_mha_decode (the attention block as neuron groups).

Form of the pass.  By default each step calls halo_ffn_forward_ahead: the FFN of step s with
the mask predicted one step earlier, and beside it -- in spare workgroups of the same two
launches -- predictor + mask of step s+1 (the paper's Pred || Load/Comp overlap, one layer
ahead).  Every step therefore runs the predictor, the mask and the FFN once.  `--serial` uses
halo_ffn_forward (predictor, mask, FFN back to back) instead; workloads with more than 16
tokens per step always do.

Weights: the layer is replicated into --copies independent copies visited round-robin, so
that consecutive steps read different HBM (a real decode walks 32 different layers per token;
one 135 MB half-layer would otherwise sit in the 256 MB Infinity Cache).

Timing.  All inputs are resident in HBM before the clock starts.  The K steps are captured
into a HIP graph -- repeated inside the graph as often as it takes for one replay to last about
10 ms, so that the figure does not depend on K -- and --replays replays (default 5) are each
timed with a HIP event pair on the launch stream; `value` and `ms_per_step` come from the
median replay.  A second, eager pass over the same steps attaches a HIP event pair to the
dispatch of the dominant kernel (FFN gate/up) of every --time-every-th step, repeated until at
least --min-timed launches were timed, for the `roofline` object; the other launches are plain,
so the host stays ahead of the GPU.  The GPU's own ceilings (read stream, bf16 matrix
instructions) are measured in the same run with the library's benchmark aids and printed beside
the nominal peaks.  `roofline.traffic` is read from the committed rocprofv3 --pmc summary under
profiles/ (null if there is none for this kernel and workload).  The CPU oracle is then timed on
a bounded sample of the same steps (at least 8 for one-token workloads, whatever K is) and its
outputs compared with the GPU's.

Prints one JSON line.
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
TARGET_REPLAY_MS = 10.0


def read_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", f"pmc_{kernel}_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch"):
            try:
                return float(line.split()[1])
            except (IndexError, ValueError):
                return None
    return None


def timed_graph(torch, st, enqueue, k_steps, est_us_per_step, replays, use_graph=True):
    """Capture `reps` rounds of enqueue() (one round = the K steps) on stream st, replay once untimed,
    then `replays` times, each between a HIP event pair on st.  Returns (median seconds per round,
    all per-round times, reps)."""
    reps = max(1, int(math.ceil(TARGET_REPLAY_MS * 1e3 / max(est_us_per_step * k_steps, 1e-3))))
    reps = min(reps, max(1, 8192 // max(k_steps, 1)))          # bound the graph's node count
    if use_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            for _ in range(reps):
                enqueue()
        run = graph.replay
    else:
        def run():
            for _ in range(reps):
                enqueue()
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        run()                                                  # untimed: the first replay uploads the graph
    torch.cuda.synchronize()
    times = []
    for _ in range(replays):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(st):
            e0.record()
            run()
            e1.record()
        e1.synchronize()
        times.append(e0.elapsed_time(e1) * 1e-3 / reps)
    return float(np.median(times)), times, reps


def measured_ceilings(torch, H, st, window_bytes, want_mfma, second_window_bytes=None):
    """The GPU's own read-stream rate (for launches of window_bytes, and for 1 GiB launches) and,
    if asked, its bf16 matrix-instruction rate.  second_window_bytes: also time plain reads in
    launches of that size (the step's other streaming kernel)."""
    buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda:0")
    buf.fill_(0x5a)
    sink = torch.zeros(256, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    out = {}
    win = max(1 << 20, int(window_bytes))
    g, us = H.halo_peak_read_stream(buf, win, 64, sink, stream=st)
    out["read_stream_same_size"] = {"GBps": g, "us_per_launch": us, "bytes_per_launch": win // 16384 * 16384}
    if second_window_bytes:
        win2 = max(1 << 20, int(second_window_bytes))
        g, us = H.halo_peak_read_stream(buf, win2, 64, sink, stream=st)
        out["read_stream_second_size"] = {"GBps": g, "us_per_launch": us, "bytes_per_launch": win2 // 16384 * 16384}
    g, us = H.halo_peak_read_stream(buf, 1 << 30, 8, sink, stream=st)
    out["read_stream_GBps"] = g
    if want_mfma:
        out["mfma_bf16_TFLOPs"] = H.halo_peak_mfma_bf16(20000, 4, sink, stream=st)
    del buf
    return out


def timed_steps_of(k_steps, passes, every, n):
    """Steps whose dominant-kernel launch carried events: launch i of the eager passes is timed if
    i % every == 0, and launch i runs step i % K."""
    return [i % k_steps for i in range(0, k_steps * passes, every)][:n]


def main_mha(args, w):
    """Head-sparse attention decode (one head + its output-projection slice = one neuron group).
    One step = predictor -> head mask -> q/k/v rows, attention over the KV cache, output
    projection, for one new token; weights and caches rotate over --copies replicas."""
    import torch

    import halo_synth as hs
    import paper_2601_11676_amd as H

    dev = "cuda:0"
    K, W, NC = args.steps, args.warmup, min(args.copies, 8)
    Hh, d, dh = w.n_heads, w.d, w.head_dim
    k_keep = w.k_keep()
    shape = H.MhaShape(d, Hh, dh, w.rank, w.dtype)
    copies = []
    for c in range(NC):
        Wq, Wk, Wv, WoT = hs.mha_weights(w, 0, dev, copy=c)
        At, Bt = hs.mha_predictor_weights(w, 0, dev, copy=c)
        kc, vc = hs.kv_cache(w, 0, dev, copy=c)
        copies.append((At, Bt, Wq, Wk, Wv, H.pack_down_proj(WoT, dh), kc, vc))
        if c == 0:
            host0 = tuple(t.float().cpu().numpy() for t in (Wq, Wk, Wv, WoT, At, Bt))
            k0, v0 = kc.float().cpu().numpy(), vc.float().cpu().numpy()   # cache of copy 0 before any step
        del WoT
    n_all = W + K
    xs = torch.stack([hs.mha_hidden(w, s, dev) for s in range(n_all + 1)])
    drops_np = np.stack([hs.mha_drop_outcomes(w, 0, s) for s in range(n_all + 1)])
    drops = torch.from_numpy(drops_np).to(dev)
    prio_dev_np = H.halo_build_schedule(k_keep, w.device_plr())
    prio_dev = torch.from_numpy(prio_dev_np).to(dev)
    ys = torch.zeros((n_all, 1, d), dtype=w.torch_dtype, device=dev)
    masks = torch.zeros((n_all + 1, 1, Hh), dtype=torch.uint8, device=dev)
    ws = torch.empty(H.halo_mha_workspace_bytes(shape, w.max_len), dtype=torch.uint8, device=dev)
    span = w.max_len - w.ctx                       # positions a copy's cache can still take
    pos_of = lambda s: w.ctx + (s // NC) % span    # each copy's cache grows by one row per visit
    st = torch.cuda.Stream()

    def make_serial(s):
        At, Bt, Wq, Wk, Wv, Wo, kc, vc = copies[s % NC]
        H.halo_mha_forward(shape, xs[s], At, Bt, Wq, Wk, Wv, Wo, kc, vc, pos_of(s), k_keep, prio_dev, w.n_dev,
                           drops[s], ys[s], ws, mask=masks[s], stream=st)

    def make_ahead(s):
        # attention of step s with the mask predicted one step earlier; beside it, in spare workgroups
        # of the q/k/v and output-projection launches, predictor + head mask of step s+1
        _, _, Wq, Wk, Wv, Wo, kc, vc = copies[s % NC]
        At, Bt = copies[(s + 1) % NC][:2]
        H.halo_mha_forward_ahead(shape, xs[s], Wq, Wk, Wv, Wo, kc, vc, pos_of(s), masks[s], ys[s], xs[s + 1],
                                 At, Bt, k_keep, prio_dev, w.n_dev, drops[s + 1], masks[s + 1], ws, stream=st)

    calls = [H.prepared(make_serial if args.serial else make_ahead, s) for s in range(n_all)]
    torch.cuda.synchronize()
    make_serial(0)                          # also provides masks[0] for the overlapped form (row pos_of(0)
    for s in range(W):                      # of copy 0 is simply written again by step 0)
        calls[s]()
    torch.cuda.synchronize()
    use_graph = not args.no_graph

    def enqueue():
        for s in range(W, W + K):
            calls[s]()
    elapsed, times, reps = timed_graph(torch, st, enqueue, K, 36.0, args.replays, use_graph)
    y_timed = ys[W:W + K].clone()
    passes = max(1, int(math.ceil(args.min_timed * args.time_every / K)))
    H.halo_profile_begin(K * passes // args.time_every + 1, args.time_every)
    torch.cuda.synchronize()
    for _ in range(passes):
        for s in range(W, W + K):
            calls[s]()
    torch.cuda.synchronize()
    kern_ms, kern_n, kern_name = H.halo_profile_end()
    same = bool(torch.equal(y_timed, ys[W:W + K]))

    n_surv = masks[W:W + K].cpu().numpy().sum(axis=2)[:, 0]                 # [K]
    esz = 2
    row_bytes = d * esz
    qkv_bytes = (2 * Hh * dh + n_surv * dh) * row_bytes                     # per launch
    cache_bytes = np.array([n_surv[i] * 2 * (pos_of(W + i) + 1) * dh * esz for i in range(K)])
    out_bytes = n_surv * dh * row_bytes
    total_bytes = float((qkv_bytes + cache_bytes + out_bytes).sum())
    timed = qkv_bytes[timed_steps_of(K, passes, args.time_every, kern_n)]
    achieved = float(timed.sum()) / (kern_ms * 1e-3) / 1e9 if kern_ms > 0 else 0.0
    ceil = measured_ceilings(torch, H, st, float(qkv_bytes.mean()), False)
    out = {
        "metric": f"MHA tokens/s (decode), {w.name}, {w.keep} of the heads kept, {w.ctx} cached positions",
        "value": K / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "d": d, "n_heads": Hh, "head_dim": dh, "rank": w.rank, "ctx": w.ctx,
                   "max_len": w.max_len, "k_keep": k_keep, "n_dev": w.n_dev,
                   "plr": [float(v) for v in w.device_plr()], "seed": w.seed, "weight_copies": NC, "graph": use_graph,
                   "predictor": "serial" if args.serial else "one step ahead, beside the attention block"},
        "timing": {"method": "HIP events around each graph replay, median", "replays": len(times),
                   "rounds_of_K_steps_per_replay": reps, "us_per_step_each_replay": [t / K * 1e6 for t in times]},
        "whole_pass": {"mean_n_surv": float(n_surv.mean()), "bytes_per_step": total_bytes / K,
                       "GBps": total_bytes / elapsed / 1e9,
                       "frac_of_hbm_peak": total_bytes / elapsed / 1e9 / HBM_PEAK_GBPS,
                       "frac_of_measured_stream": total_bytes / elapsed / 1e9 / ceil["read_stream_GBps"],
                       "graph_equals_eager": same},
        "roofline": {"bound": "hbm", "kernel": kern_name, "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": read_traffic(kern_name, w.name),
                     "launches": int(kern_n), "avg_us": kern_ms / max(kern_n, 1) * 1e3,
                     "bytes_per_launch": float(timed.mean()) if len(timed) else 0.0,
                     "measured_peak": ceil["read_stream_GBps"],
                     "frac_of_measured": achieved / ceil["read_stream_GBps"],
                     "measured_same_size_launch": ceil["read_stream_same_size"]},
    }
    if not args.no_cpu:
        from oracle import ref
        Wq, Wk, Wv, WoT, At, Bt = host0
        # copy 0's first visit after the caches were last in their generated state is step 0; replay the
        # oracle over copy 0's visits from the start so that its cache matches the GPU's at every step
        visits = [s for s in range(W + K) if s % NC == 0]
        sample = visits[: max(1, min(args.cpu_steps, 16))]
        kc, vc = k0.copy(), v0.copy()
        x_np = xs.float().cpu().numpy()
        y_np = ys.float().cpu().numpy()
        worst, masks_ok = 0.0, True
        t0 = time.perf_counter()
        outs = []
        for s in sample:
            sc = ref.predict_scores(x_np[s], At, Bt)
            m = ref.build_group_mask(sc, k_keep, prio_dev_np, w.n_dev, drops_np[s])
            outs.append((m["mask"], ref.mha_decode(x_np[s], Wq, Wk, Wv, WoT, kc, vc, pos_of(s), m["mask"][0])))
        cpu_t = time.perf_counter() - t0
        # the eager and graph passes re-ran the timed steps on the same cache rows, so only steps before
        # the timed region (warm-up visits) are compared value by value with the GPU's stored outputs
        for s, (mk, yc) in zip(sample, outs):
            if s >= W:
                break
            masks_ok &= bool(np.array_equal(mk, masks[s].cpu().numpy()))
            den = np.linalg.norm(yc)
            if den > 0:
                worst = max(worst, float(np.linalg.norm(y_np[s, 0] - yc) / den))
        out["cpu_baseline"] = {"value": len(sample) / cpu_t, "unit": "tokens/s", "cores": ref.num_threads(),
                               "kind": "oracle",
                               "sample": f"{len(sample)} steps on weight copy 0 (whole pass each)",
                               "ms_per_step": cpu_t / len(sample) * 1e3,
                               "gpu_vs_oracle_max_rel_l2": worst, "masks_bit_exact": masks_ok}
    print(json.dumps(out), flush=True)


def main_stack(args, w):
    """The whole FFN stack as one step: every layer's weights resident in HBM, T tokens walk the L
    layers; x_l = h_l / rms(h_l), y_l = FFN_l(x_l; mask_l), h_{l+1} = h_l + y_l (float32).  Layer 0
    runs dense and lossless; the mask of layer l+1 is predicted from x_l beside layer l's FFN (the
    paper's one-layer-ahead scheme).  Three launches per layer: gate/up (+ predictor rows), down
    projection (+ mask workgroups), residual + norm."""
    import torch

    import halo_synth as hs
    import paper_2601_11676_amd as H

    dev = "cuda:0"
    K, W = args.steps, args.warmup
    T, G, d, L = w.T, w.n_groups, w.d, w.layers
    keep = w.keep[0] if args.keep is None else args.keep
    k_keep = w.k_keep(keep)
    shape = H.Shape(w.d, w.ffn, w.group_size, w.rank, w.dtype)
    esz = 2
    t_gen = time.perf_counter()
    layers = []
    for l in range(L):
        At, Bt = hs.predictor_weights(w, l, dev)
        if args.q4:                                   # (At, Bt, the six code / scale arrays)
            layers.append((At, Bt, hs.ffn_weights_q4(w, l, dev)))
        else:
            Wg, Wu, WdT = hs.ffn_weights(w, l, dev)
            layers.append((At, Bt, Wg, Wu, H.pack_down_proj(WdT, w.group_size)))
            del WdT
        if l % 10 == 9:
            print(f"[bench] generated {l + 1} of {L} layers, {torch.cuda.memory_allocated() / 1e9:.1f} GB resident",
                  file=sys.stderr, flush=True)
    t_gen = time.perf_counter() - t_gen
    n_all = W + K
    h0 = torch.stack([hs.hidden_states(w, s, dev, dtype=torch.float32) for s in range(n_all)])     # [n][T][d]
    drops_np = np.stack([np.stack([hs.drop_outcomes(w, l, s) for l in range(L)]) for s in range(n_all)])
    drops = torch.from_numpy(drops_np).to(dev)                                                      # [n][L][T][n_dev]
    prio_dev_np = H.halo_build_schedule(k_keep, w.device_plr())
    prio_dev = torch.from_numpy(prio_dev_np).to(dev)
    ws = torch.empty(H.halo_workspace_bytes(shape, T, G), dtype=torch.uint8, device=dev)
    h = torch.zeros((T, d), dtype=torch.float32, device=dev)
    xbuf = torch.zeros((L + 1, T, d), dtype=w.torch_dtype, device=dev)
    ybuf = torch.zeros((L, T, d), dtype=w.torch_dtype, device=dev)
    masks = torch.zeros((n_all, L, T, G), dtype=torch.uint8, device=dev)
    masks[:, 0] = 1                                  # layer 0: every group, nothing lost
    h_out = torch.zeros((n_all, T, d), dtype=torch.float32, device=dev)
    st = torch.cuda.Stream()

    def stack_pass(s):
        h.copy_(h0[s])
        H.halo_stack_residual_norm(h, None, xbuf[0], stream=st)
        for l in range(L):
            if args.q4:
                q4 = layers[l][2]
                if l + 1 < L:
                    At, Bt = layers[l + 1][:2]
                    H.halo_ffn_forward_ahead_q4(shape, xbuf[l], q4, masks[s, l], ybuf[l], xbuf[l], At, Bt, k_keep,
                                                prio_dev, w.n_dev, drops[s, l + 1], masks[s, l + 1], ws, stream=st)
                else:
                    H.halo_group_sparse_ffn_q4(shape, xbuf[l], q4, masks[s, l], ybuf[l], ws, stream=st)
                H.halo_stack_residual_norm(h, ybuf[l], xbuf[l + 1], stream=st)
                continue
            _, _, Wg, Wu, Wd = layers[l]
            if l + 1 < L:
                At, Bt = layers[l + 1][:2]
                H.halo_ffn_forward_ahead(shape, xbuf[l], Wg, Wu, Wd, masks[s, l], ybuf[l], xbuf[l], At, Bt, k_keep,
                                         prio_dev, w.n_dev, drops[s, l + 1], masks[s, l + 1], ws, stream=st)
            else:
                H.halo_group_sparse_ffn(shape, xbuf[l], Wg, Wu, Wd, masks[s, l], ybuf[l], ws, stream=st)
            H.halo_stack_residual_norm(h, ybuf[l], xbuf[l + 1], stream=st)
        h_out[s].copy_(h)

    with torch.cuda.stream(st):
        for s in range(W):
            stack_pass(s)
    torch.cuda.synchronize()

    def enqueue():
        for s in range(W, W + K):
            stack_pass(s)
    per_layer_est = {5120: 60.0, 8192: 235.0}.get(d, 100.0) * (0.55 if args.q4 else 1.0)
    elapsed, times, reps = timed_graph(torch, st, enqueue, K, per_layer_est * L, args.replays, not args.no_graph)
    h_timed = h_out[W:W + K].clone()

    # dominant kernel under events: one eager pass over the K steps
    every = max(1, args.time_every)
    H.halo_profile_begin(K * L // every + 1, every)
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        for s in range(W, W + K):
            stack_pass(s)
    torch.cuda.synchronize()
    kern_ms, kern_n, kern_name = H.halo_profile_end()
    same = bool(torch.equal(h_timed, h_out[W:W + K]))

    mask_np = masks[W:W + K].cpu().numpy()                      # [K][L][T][G]
    union = mask_np.any(axis=2).sum(axis=2)                     # [K][L] groups read per layer
    n_surv = mask_np.sum(axis=3)                                # [K][L][T]
    group_bytes = w.group_size * d * esz
    if args.q4:                                                 # codes + one bf16 scale per 128 elements
        group_bytes = w.group_size * (d // 2 + (d // 128) * 2)
    ffn_bytes = float(union.sum()) * 3 * group_bytes
    flat_union = union.reshape(-1)                              # launch order: step-major, layer-minor
    timed_union = flat_union[::every][:kern_n]
    gate_up_bytes = float(timed_union.sum()) * 2 * group_bytes
    achieved = gate_up_bytes / (kern_ms * 1e-3) / 1e9 if kern_ms > 0 else 0.0
    ceil = measured_ceilings(torch, H, st, float(union[:, 1:].mean()) * 2 * group_bytes, False)
    out = {
        "metric": f"FFN-stack tokens/s (decode), {w.name}: {L} layers resident, keep {keep}" + (", 4-bit weights" if args.q4 else ""),
        "value": K * T / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype + (" activations, 4-bit block-quantised FFN weights" if args.q4 else ""), "data": "synthetic",
        "config": {"workload": w.name + "_full_stack" + ("_q4" if args.q4 else ""), "d": d, "ffn": w.ffn, "n_groups": G, "group_size": w.group_size,
                   "rank": w.rank, "tokens_per_step": T, "layers": L, "keep": keep, "k_keep": k_keep,
                   "n_dev": w.n_dev, "plr": [float(v) for v in w.device_plr()], "seed": w.seed,
                   "resident_GB": torch.cuda.memory_allocated() / 1e9, "graph": not args.no_graph,
                   "predictor": "one layer ahead, beside the FFN; layer 0 dense and lossless"},
        "timing": {"method": "HIP events around each graph replay, median", "replays": len(times),
                   "rounds_of_K_steps_per_replay": reps, "ms_per_step_each_replay": [t / K * 1e3 for t in times],
                   "weights_generated_in_s": t_gen},
        "whole_pass": {"us_per_layer": elapsed / K / L * 1e6, "mean_n_surv_sparse_layers": float(n_surv[:, 1:].mean()),
                       "mean_union_sparse_layers": float(union[:, 1:].mean()),
                       "weight_GBps": ffn_bytes / elapsed / 1e9,
                       "frac_of_hbm_peak": ffn_bytes / elapsed / 1e9 / HBM_PEAK_GBPS,
                       "frac_of_measured_stream": ffn_bytes / elapsed / 1e9 / ceil["read_stream_GBps"],
                       "graph_equals_eager": same},
        "roofline": {"bound": "hbm", "kernel": kern_name, "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": read_traffic(kern_name, w.name + ("_q4" if args.q4 else "")),
                     "launches": int(kern_n), "avg_us": kern_ms / max(kern_n, 1) * 1e3,
                     "bytes_per_launch": gate_up_bytes / max(kern_n, 1),
                     "measured_peak": ceil["read_stream_GBps"],
                     "frac_of_measured": achieved / ceil["read_stream_GBps"],
                     "measured_same_size_launch": ceil["read_stream_same_size"]},
    }
    if not args.no_cpu:
        # the oracle, teacher-forced on two layers of the last timed step (it is fed the GPU's own x_l and
        # x_{l-1}); its time per layer, times L, is the stack's CPU figure
        from oracle import ref
        s = W + K - 1
        with torch.cuda.stream(st):
            stack_pass(s)
        torch.cuda.synchronize()
        x_np = xbuf.float().cpu().numpy()
        y_np = ybuf.float().cpu().numpy()
        check = sorted({1, L // 2})
        cpu_t, worst, masks_ok = 0.0, 0.0, True
        for l in check:
            if args.q4:
                At, Bt, q4 = layers[l]
                host = [At.float().cpu().numpy(), Bt.float().cpu().numpy(),
                        *ref.dequant_ffn_q4([t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()
                                             for t in q4])]
            else:
                At, Bt, Wg, Wu, Wd = layers[l]
                WdT = Wd.permute(0, 2, 1).reshape(w.ffn, d)       # back to neuron-major for the oracle
                host = [t.float().cpu().numpy() for t in (At, Bt, Wg, Wu, WdT)]
            t0 = time.perf_counter()
            sc = ref.predict_scores(x_np[l - 1], host[0], host[1])
            m = ref.build_group_mask(sc, k_keep, prio_dev_np, w.n_dev, drops_np[s, l])
            yc = ref.group_sparse_ffn(x_np[l], host[2], host[3], host[4], w.group_size, m["mask"])
            cpu_t += time.perf_counter() - t0
            masks_ok &= bool(np.array_equal(m["mask"], masks[s, l].cpu().numpy()))
            den = np.linalg.norm(yc)
            if den > 0:
                worst = max(worst, float(np.linalg.norm(y_np[l] - yc) / den))
            del host
        per_layer = cpu_t / len(check)
        out["cpu_baseline"] = {"value": T / (per_layer * L), "unit": "tokens/s", "cores": ref.num_threads(),
                               "kind": "oracle",
                               "sample": f"layers {check} of one step, teacher-forced; per-layer time x {L} layers",
                               "ms_per_layer": per_layer * 1e3,
                               "gpu_vs_oracle_max_rel_l2": worst, "masks_bit_exact": masks_ok}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="default 1024 (8 with --stack)")
    ap.add_argument("--warmup", type=int, default=None, help="default 64 (1 with --stack)")
    ap.add_argument("--copies", type=int, default=16, help="independent weight copies rotated over")
    ap.add_argument("--workload", default="llama7b_decode")
    ap.add_argument("--stack", action="store_true",
                    help="llama13b_stack / llama70b_stack: a step is the whole stack with every layer resident (bf16, or 4-bit with --q4)")
    ap.add_argument("--keep", type=float, default=None, help="keep ratio (default: the workload's first)")
    ap.add_argument("--no-graph", action="store_true", help="launch the timed steps eagerly")
    ap.add_argument("--serial", action="store_true",
                    help="predictor, mask and FFN back to back on one stream (halo_ffn_forward) instead "
                         "of the predictor running one step ahead beside the FFN (halo_ffn_forward_ahead)")
    ap.add_argument("--q4", action="store_true",
                    help="4-bit block-quantised FFN weights (halo_ffn_forward_q4 / _ahead_q4) instead of bf16")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--cpu-steps", type=int, default=64)
    ap.add_argument("--replays", type=int, default=5, help="timed graph replays (the median is reported)")
    ap.add_argument("--time-every", type=int, default=4,
                    help="attach HIP events to one dominant-kernel launch in this many (event launches are "
                         "slow on the host; timing all of them starves the GPU and slows the kernel itself)")
    ap.add_argument("--min-timed", type=int, default=128,
                    help="the eager event pass is repeated until this many launches were timed")
    ap.add_argument("--chains", type=int, default=1,
                    help="also time the K steps as this many independent chains of steps on as many streams "
                         "(each chain strictly sequential; reported beside the headline as `concurrent_chains`, "
                         "never as `value`)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the benchmark, run 8 plain device-to-device copies of 256 MiB "
                         "(a kernel of known traffic) for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (the simulated devices are a "
              "group-to-device map plus drop flags on one GPU); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.steps is None:
        args.steps = 8 if args.stack else 1024
    if args.warmup is None:
        args.warmup = 1 if args.stack else 64
    if args.steps < 1 or args.warmup < 0 or args.replays < 1:
        print("bench.py: --steps >= 1, --warmup >= 0, --replays >= 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import halo_synth as hs
    import paper_2601_11676_amd as H

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    H.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = 256 << 20
        src = torch.full((n,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(8):
            dst.copy_(src)          # one elementwise copy kernel: reads n bytes, writes n bytes
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": n, "bytes_written": n, "launches": 8}}))
        return
    if args.workload in hs.MHA_BY_NAME:
        main_mha(args, hs.MHA_BY_NAME[args.workload])
        return
    w = hs.BY_NAME[args.workload]
    if args.stack:
        if w.layers < 2 or args.serial:
            print("bench.py: --stack needs a multi-layer workload (overlapped form)", file=sys.stderr)
            sys.exit(2)
        main_stack(args, w)
        return
    K, W, NC = args.steps, args.warmup, args.copies
    T, G, d = w.T, w.n_groups, w.d
    keep = w.keep[0] if args.keep is None else args.keep
    k_keep = w.k_keep(keep)
    shape = H.Shape(w.d, w.ffn, w.group_size, w.rank, w.dtype)
    esz = 2 if w.dtype == "bf16" else 4

    # ---- resident inputs -------------------------------------------------------------
    copies = []
    for c in range(NC):
        At, Bt = hs.predictor_weights(w, 0, dev, copy=c)
        if args.q4:
            copies.append((At, Bt, hs.ffn_weights_q4(w, 0, dev, copy=c)))
            continue
        Wg, Wu, WdT = hs.ffn_weights(w, 0, dev, copy=c)
        copies.append((At, Bt, Wg, Wu, H.pack_down_proj(WdT, w.group_size)))   # library layout
        if c == 0:
            WdT0 = WdT                  # neuron-major original of copy 0, for the oracle leg
        del WdT
    n_all = W + K + 1                      # one extra input: the last step predicts one step ahead
    xs = torch.stack([hs.hidden_states(w, s, dev) for s in range(n_all)])          # [n][T][d]
    drops_np = np.stack([hs.drop_outcomes(w, 0, s) for s in range(n_all)])          # [n][T][n_dev]
    drops = torch.from_numpy(drops_np).to(dev)
    prio_dev_np = H.halo_build_schedule(k_keep, w.device_plr())
    prio_dev = torch.from_numpy(prio_dev_np).to(dev)
    ys = torch.zeros((n_all, T, d), dtype=w.torch_dtype, device=dev)
    masks = torch.zeros((n_all, T, G), dtype=torch.uint8, device=dev)
    ws_bytes = H.halo_workspace_bytes_q4(shape, T, k_keep) if args.q4 else H.halo_workspace_bytes(shape, T, k_keep)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    st = torch.cuda.Stream()               # every library call below goes to this stream (default priority)

    def step_serial_q4(s, ws=ws, st=st, ys=ys):
        At, Bt, q4 = copies[s % NC]
        H.halo_ffn_forward_q4(shape, xs[s], At, Bt, q4, k_keep, prio_dev, w.n_dev, drops[s], ys[s], ws,
                              mask=masks[s], stream=st)

    def step_ahead_q4(s, ws=ws, st=st, ys=ys):
        q4 = copies[s % NC][2]
        At, Bt = copies[(s + 1) % NC][:2]
        H.halo_ffn_forward_ahead_q4(shape, xs[s], q4, masks[s], ys[s], xs[s + 1], At, Bt, k_keep, prio_dev,
                                    w.n_dev, drops[s + 1], masks[s + 1], ws, stream=st)

    def step_serial(s, ws=ws, st=st, ys=ys):
        At, Bt, Wg, Wu, Wd = copies[s % NC]
        H.halo_ffn_forward(shape, xs[s], At, Bt, Wg, Wu, Wd, k_keep, prio_dev, w.n_dev, drops[s],
                           ys[s], ws, mask=masks[s], stream=st)

    def step_ahead(s, ws=ws, st=st, ys=ys):
        # FFN of step s with the mask predicted one step earlier; beside it, in spare workgroups
        # of the same launches, predictor + mask of step s+1 (the paper's Pred || Comp overlap)
        _, _, Wg, Wu, Wd = copies[s % NC]
        At, Bt = copies[(s + 1) % NC][:2]
        H.halo_ffn_forward_ahead(shape, xs[s], Wg, Wu, Wd, masks[s], ys[s], xs[s + 1], At, Bt, k_keep,
                                 prio_dev, w.n_dev, drops[s + 1], masks[s + 1], ws, stream=st)

    if T > 16:
        args.serial = True      # the overlap rides in spare workgroups of the one- and few-token kernels only
    # marshal every step's call once: the timed and the profiled loops then cost a few
    # microseconds of host time per step, so the GPU is never left waiting for Python
    make = step_serial if args.serial else step_ahead
    if args.q4:
        make = step_serial_q4 if args.serial else step_ahead_q4
    calls = [H.prepared(make, s) for s in range(W + K)]

    # ---- warm-up -----------------------------------------------------------------------
    torch.cuda.synchronize()
    (step_serial_q4 if args.q4 else step_serial)(0)   # also provides masks[0] for the overlapped form
    for s in range(W):
        calls[s]()
    if not args.serial:
        # masks[W] for the first timed step (the warm-up's last step wrote it already unless W == 0)
        ws_scores = torch.empty((T, G), dtype=torch.float32, device=dev)
        At, Bt = copies[W % NC][:2]
        H.halo_predict_scores(shape, xs[W], At, Bt, ws_scores, ws, stream=st)
        H.halo_build_group_mask(ws_scores, k_keep, prio_dev, w.n_dev, drops[W], masks[W], stream=st)
    torch.cuda.synchronize()

    # ---- timed: K steps, median of the replays ---------------------------------------------
    use_graph = not args.no_graph

    def enqueue():
        for s in range(W, W + K):
            calls[s]()
    est_us = {1: 26.0, 4: 60.0, 8: 230.0, 512: 190.0}.get(T, 50.0)
    elapsed, times, reps = timed_graph(torch, st, enqueue, K, est_us, args.replays, use_graph)
    y_timed = ys[W:W + K].clone()

    # ---- optional: the same K steps as several independent chains on as many streams -------
    chains = None
    if args.chains > 1 and use_graph and K >= 2 * args.chains:
        C = args.chains
        bounds = [W + K * c // C for c in range(C + 1)]
        streams = [st] + [torch.cuda.Stream() for _ in range(C - 1)]
        wss = [ws] + [torch.empty_like(ws) for _ in range(C - 1)]
        ys2 = torch.zeros_like(ys)
        ccalls = []
        for c in range(C):
            ccalls.append([H.prepared(make, s_, ws=wss[c], st=streams[c], ys=ys2) for s_ in range(bounds[c], bounds[c + 1])])
        if not args.serial:
            for c in range(1, C):                   # the mask of each chain's first step (chain 0's exists already)
                At, Bt = copies[bounds[c] % NC][:2]
                H.halo_predict_scores(shape, xs[bounds[c]], At, Bt, ws_scores, ws, stream=st)
                H.halo_build_group_mask(ws_scores, k_keep, prio_dev, w.n_dev, drops[bounds[c]], masks[bounds[c]], stream=st)
        torch.cuda.synchronize()

        def enqueue_chains():
            for c in range(1, C):
                streams[c].wait_stream(st)          # fork
            for c in range(C):
                for call in ccalls[c]:
                    call()
            for c in range(1, C):
                st.wait_stream(streams[c])          # join
        c_elapsed, c_times, c_reps = timed_graph(torch, st, enqueue_chains, K, est_us / C, args.replays, True)
        chains = {"chains": C, "us_per_step": c_elapsed / K * 1e6, "tokens_per_s": K * T / c_elapsed,
                  "rounds_of_K_steps_per_replay": c_reps,
                  "same_outputs_as_one_chain": bool(torch.equal(ys2[W:W + K], y_timed)),
                  "note": "independent chains of steps overlap each other's launch boundaries; a single sequence "
                          "cannot do this (its steps depend on each other): not the headline"}

    # ---- dominant kernel under HIP events (eager passes over the same steps) -------------
    passes = max(1, int(math.ceil(args.min_timed * args.time_every / K)))
    H.halo_profile_begin(K * passes // args.time_every + 1, args.time_every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(passes):
        for s in range(W, W + K):
            calls[s]()
    t_enq = time.perf_counter() - t0
    torch.cuda.synchronize()
    t_eager = time.perf_counter() - t0
    kern_ms, kern_n, kern_name = H.halo_profile_end()
    same = bool(torch.equal(y_timed, ys[W:W + K]))       # graph replay == eager, bit for bit

    mask_np = masks[W:W + K].cpu().numpy()
    n_surv = mask_np.sum(axis=2)                          # [K][T]
    union = mask_np.any(axis=1).sum(axis=1)               # [K] groups read per step
    group_bytes = w.group_size * d * esz                  # one projection of one group
    if args.q4:                                           # codes + one bf16 scale per 128 elements
        group_bytes = w.group_size * d // 2 + w.group_size * d // hs.Q4_BLOCK * 2
    ffn_bytes = float(union.sum()) * 3 * group_bytes      # over the K steps
    pred_bytes = K * (w.rank * d + G * w.rank) * esz
    # bytes of exactly the launches that were timed
    timed = timed_steps_of(K, passes, args.time_every, kern_n)
    gate_up_bytes = float(union[timed].sum()) * 2 * group_bytes
    achieved = gate_up_bytes / (kern_ms * 1e-3) / 1e9 if kern_ms > 0 else 0.0
    traffic = read_traffic(kern_name, w.name + ("_q4" if args.q4 else ""))
    many = "_pf" in kern_name
    ceil = measured_ceilings(torch, H, st, float(union.mean()) * 2 * group_bytes, many,
                             None if many else float(union.mean()) * group_bytes)
    whole = {
        "mean_n_surv": float(n_surv.mean()), "mean_union": float(union.mean()),
        "weight_GBps": ffn_bytes / elapsed / 1e9,
        "total_GBps": (ffn_bytes + pred_bytes) / elapsed / 1e9,
        "frac_of_hbm_peak": ffn_bytes / elapsed / 1e9 / HBM_PEAK_GBPS,
        "frac_of_measured_stream": ffn_bytes / elapsed / 1e9 / ceil["read_stream_GBps"],
        "graph_equals_eager": same,
        "event_pass_us_per_step": t_eager / (K * passes) * 1e6,
        "event_pass_host_us_per_step": t_enq / (K * passes) * 1e6,
    }
    if "read_stream_second_size" in ceil:
        # what two plain read-only launches of the step's two weight streams cost back to back: no mask,
        # no arithmetic, no dependency between them -- the floor of any two-launch form of the step
        floor_us = ceil["read_stream_same_size"]["us_per_launch"] + ceil["read_stream_second_size"]["us_per_launch"]
        whole["plain_read_two_launches_us"] = floor_us
        whole["plain_read_two_launches_frac_of_hbm_peak"] = ffn_bytes / K / (floor_us * 1e-6) / 1e9 / HBM_PEAK_GBPS
        whole["step_over_plain_read_two_launches"] = elapsed / K * 1e6 / floor_us
    if chains is not None:
        chains["weight_GBps"] = ffn_bytes / (chains["us_per_step"] * 1e-6 * K) / 1e9
        chains["frac_of_hbm_peak"] = chains["weight_GBps"] / HBM_PEAK_GBPS
        whole["concurrent_chains"] = chains
    if many:
        # many tokens: the dominant kernel is a dense contraction on the matrix cores
        flops = float(n_surv[timed].sum()) * w.group_size * d * 2 * 2      # gate and up, 2 flop per MAC
        tf = flops / (kern_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": kern_name, "achieved": tf,
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS,
                "traffic": traffic, "launches": int(kern_n), "avg_us": kern_ms / max(kern_n, 1) * 1e3,
                "flops_per_launch": flops / max(kern_n, 1),
                "hbm_GBps_of_this_kernel": achieved,
                "measured_peak": ceil["mfma_bf16_TFLOPs"], "frac_of_measured": tf / ceil["mfma_bf16_TFLOPs"]}
        step_flops = float(n_surv.sum()) / K * w.group_size * d * 2 * 3
        step_bytes = ffn_bytes / K + 2 * T * d * esz
        step_us = elapsed / K * 1e6
        whole.update({
            "flops_per_step": step_flops, "TFLOPs": step_flops / (elapsed / K) / 1e12,
            "frac_of_mfma_peak": step_flops / (elapsed / K) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "bound_mfma_us": step_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e6,
            "bound_hbm_us": step_bytes / (HBM_PEAK_GBPS * 1e9) * 1e6,
            "bound_mfma_measured_us": step_flops / (ceil["mfma_bf16_TFLOPs"] * 1e12) * 1e6,
            "bound_hbm_measured_us": step_bytes / (ceil["read_stream_GBps"] * 1e9) * 1e6,
            "step_over_max_bound": step_us / max(step_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e6,
                                                 step_bytes / (HBM_PEAK_GBPS * 1e9) * 1e6)})
    else:
        roof = {"bound": "hbm", "kernel": kern_name, "achieved": achieved, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                "launches": int(kern_n), "avg_us": kern_ms / max(kern_n, 1) * 1e3,
                "bytes_per_launch": gate_up_bytes / max(kern_n, 1),
                "measured_peak": ceil["read_stream_GBps"], "frac_of_measured": achieved / ceil["read_stream_GBps"],
                "measured_same_size_launch": ceil["read_stream_same_size"]}

    out = {
        "metric": ("FFN tokens/s (decode), LLaMA-7B shape, 50% groups kept" if w.name == "llama7b_decode" and args.keep is None
                   else f"FFN tokens/s, {w.name}, keep {keep}") + (", 4-bit weights" if args.q4 else ""),
        "value": K * T / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": elapsed / K * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype + (" activations, 4-bit block-quantised FFN weights" if args.q4 else ""),
        "data": "synthetic",
        "config": {"workload": w.name + ("_q4" if args.q4 else ""), "d": d, "ffn": w.ffn, "n_groups": G, "group_size": w.group_size,
                   "rank": w.rank, "tokens_per_step": T, "keep": keep, "k_keep": k_keep, "n_dev": w.n_dev,
                   "plr": [float(v) for v in w.device_plr()], "seed": w.seed, "weight_copies": NC,
                   "graph": use_graph, "predictor": "serial" if args.serial else "one step ahead, beside the FFN"},
        "timing": {"method": "HIP events around each graph replay, median", "replays": len(times),
                   "rounds_of_K_steps_per_replay": reps, "us_per_step_each_replay": [t / K * 1e6 for t in times]},
        "whole_pass": whole,
        "roofline": roof,
    }

    # ---- CPU oracle on a bounded sample of the same inputs (rank 0, N=1) -----------------
    if not args.no_cpu:
        from oracle import ref
        if args.q4:
            At, Bt = (t.float().cpu().numpy() for t in copies[0][:2])
            Wg, Wu, WdT = ref.dequant_ffn_q4([t.float().cpu().numpy() if t.dtype == torch.bfloat16
                                              else t.cpu().numpy() for t in copies[0][2]])
        else:
            At, Bt, Wg, Wu, WdT = (t.float().cpu().numpy() for t in (*copies[0][:4], WdT0))
        # the sample: hidden states and loss outcomes of the first timed steps, run once more on the GPU
        # against weight copy 0 (the copy the oracle holds) with the serial pass, and by the oracle
        n_chk = max(1, min(max(8, min(args.cpu_steps, K)), max(1, 64 // T)))
        idx = [W + (i % K) for i in range(n_chk)]
        y_chk = torch.zeros((n_chk, T, d), dtype=w.torch_dtype, device=dev)
        m_chk = torch.zeros((n_chk, T, G), dtype=torch.uint8, device=dev)
        for i, s in enumerate(idx):
            if args.q4:
                H.halo_ffn_forward_q4(shape, xs[s], copies[0][0], copies[0][1], copies[0][2], k_keep, prio_dev,
                                      w.n_dev, drops[s], y_chk[i], ws, mask=m_chk[i], stream=st)
            else:
                H.halo_ffn_forward(shape, xs[s], *copies[0], k_keep, prio_dev, w.n_dev, drops[s], y_chk[i], ws,
                                   mask=m_chk[i], stream=st)
        torch.cuda.synchronize()
        x_np = xs.float().cpu().numpy()
        t0 = time.perf_counter()
        outs = [ref.ffn_forward(x_np[s], At, Bt, Wg, Wu, WdT, w.group_size, k_keep, prio_dev_np,
                                w.n_dev, drops_np[s]) for s in idx]
        cpu_t = time.perf_counter() - t0
        worst, masks_ok = 0.0, True
        y_np = y_chk.float().cpu().numpy()
        m_np = m_chk.cpu().numpy()
        for i, o in enumerate(outs):
            masks_ok &= bool(np.array_equal(o["mask"], m_np[i]))
            den = np.linalg.norm(o["y"])
            if den > 0:
                worst = max(worst, float(np.linalg.norm(y_np[i] - o["y"]) / den))
        out["cpu_baseline"] = {
            "value": n_chk * T / cpu_t, "unit": "tokens/s", "cores": ref.num_threads(),
            "kind": "oracle",
            "sample": f"inputs of {n_chk} timed steps against weight copy 0, whole pass each",
            "ms_per_step": cpu_t / n_chk * 1e3,
            "gpu_vs_oracle_max_rel_l2": worst, "masks_bit_exact": masks_ok,
        }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
