#!/usr/bin/env python3
"""Benchmark of the HALO group-sparse FFN path on one MI355X.

One "step" = one whole pass (predictor -> group mask -> group-sparse SwiGLU FFN) over one
batch of synthetic input.  The default workload is the LLaMA-7B-shape single-layer decode:
d=4096, ffn=11008 as 86 groups of 128, bf16, one token per step, 43 groups kept, 4 simulated
devices with loss rates {0, 0.05, 0.1, 0.2}, fresh hidden state and loss outcomes per step.
`--workload` also accepts llama7b_prefill (512 tokens per step, matrix-core roofline),
llama13b_stack and llama70b_stack (one layer of that shape per step, 4 / 8 tokens) and tiny.

Form of the pass.  By default each step calls halo_ffn_forward_ahead: the FFN of step s with
the mask predicted one step earlier, and beside it -- in spare workgroups of the same two
launches -- predictor + mask of step s+1 (the paper's Pred || Load/Comp overlap, one layer
ahead).  Every step therefore runs the predictor, the mask and the FFN once.  `--serial` uses
halo_ffn_forward (predictor, mask, FFN back to back) instead; workloads with more than 16
tokens per step always do.

Weights: the layer is replicated into --copies independent copies visited round-robin, so
that consecutive steps read different HBM (a real decode walks 32 different layers per token;
one 135 MB half-layer would otherwise sit in the 256 MB Infinity Cache).

Timing: all inputs are resident in HBM before the clock starts.  The K timed steps are
captured once into a HIP graph (the loop is launch-bound otherwise) and one replay is timed
between two device synchronisations: `value`.  A second, eager pass over the same K steps
attaches a HIP event pair to the dispatch of the dominant kernel (FFN gate/up) of every
--time-every-th step for the `roofline` object; the other launches are plain, so the host
stays ahead of the GPU and the kernel is measured in the same back-to-back regime as the
graph.  `roofline.traffic` is read from the committed rocprofv3 --pmc summary under
profiles/ (null if there is none for this kernel and workload).  The CPU oracle is then timed
on a bounded sample of the same steps and its outputs compared with the GPU's.

Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


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
    if use_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            for s in range(W, W + K):
                calls[s]()
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(st):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(W, W + K):
            calls[s]()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    y_timed = ys[W:W + K].clone()
    H.halo_profile_begin(K, args.time_every)
    torch.cuda.synchronize()
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
    timed = qkv_bytes[::args.time_every][:kern_n]
    achieved = float(timed.sum()) / (kern_ms * 1e-3) / 1e9 if kern_ms > 0 else 0.0
    out = {
        "metric": f"MHA tokens/s (decode), {w.name}, {w.keep} of the heads kept, {w.ctx} cached positions",
        "value": K / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "d": d, "n_heads": Hh, "head_dim": dh, "rank": w.rank, "ctx": w.ctx,
                   "max_len": w.max_len, "k_keep": k_keep, "n_dev": w.n_dev,
                   "plr": [float(v) for v in w.device_plr()], "seed": w.seed, "weight_copies": NC, "graph": use_graph,
                   "predictor": "serial" if args.serial else "one step ahead, beside the attention block"},
        "whole_pass": {"mean_n_surv": float(n_surv.mean()), "bytes_per_step": total_bytes / K,
                       "GBps": total_bytes / elapsed / 1e9,
                       "frac_of_hbm_peak": total_bytes / elapsed / 1e9 / HBM_PEAK_GBPS, "graph_equals_eager": same},
        "roofline": {"bound": "hbm", "kernel": kern_name, "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": read_traffic(kern_name, w.name),
                     "launches": int(kern_n), "avg_us": kern_ms / max(kern_n, 1) * 1e3,
                     "bytes_per_launch": float(timed.mean()) if len(timed) else 0.0},
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1024)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--copies", type=int, default=16, help="independent weight copies rotated over")
    ap.add_argument("--workload", default="llama7b_decode")
    ap.add_argument("--no-graph", action="store_true", help="launch the timed steps eagerly")
    ap.add_argument("--serial", action="store_true",
                    help="predictor, mask and FFN back to back on one stream (halo_ffn_forward) instead "
                         "of the predictor running one step ahead beside the FFN (halo_ffn_forward_ahead)")
    ap.add_argument("--q4", action="store_true",
                    help="4-bit block-quantised FFN weights (halo_ffn_forward_q4 / _ahead_q4) instead of bf16")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--cpu-steps", type=int, default=64)
    ap.add_argument("--time-every", type=int, default=4,
                    help="attach HIP events to one dominant-kernel launch in this many (event launches are "
                         "slow on the host; timing all of them starves the GPU and slows the kernel itself)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the benchmark, run 8 plain device-to-device copies of 256 MiB "
                         "(a kernel of known traffic) for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (the simulated devices are a "
              "group-to-device map plus drop flags on one GPU); run with --gpus 1", file=sys.stderr)
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
    K, W, NC = args.steps, args.warmup, args.copies
    T, G, d = w.T, w.n_groups, w.d
    k_keep = w.k_keep()
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
    ws = torch.empty(H.halo_workspace_bytes(shape, T, k_keep), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    st = torch.cuda.Stream()               # every library call below goes to this stream (default priority)

    def step_serial_q4(s):
        At, Bt, q4 = copies[s % NC]
        H.halo_ffn_forward_q4(shape, xs[s], At, Bt, q4, k_keep, prio_dev, w.n_dev, drops[s], ys[s], ws,
                              mask=masks[s], stream=st)

    def step_ahead_q4(s):
        q4 = copies[s % NC][2]
        At, Bt = copies[(s + 1) % NC][:2]
        H.halo_ffn_forward_ahead_q4(shape, xs[s], q4, masks[s], ys[s], xs[s + 1], At, Bt, k_keep, prio_dev,
                                    w.n_dev, drops[s + 1], masks[s + 1], ws, stream=st)

    def step_serial(s):
        At, Bt, Wg, Wu, Wd = copies[s % NC]
        H.halo_ffn_forward(shape, xs[s], At, Bt, Wg, Wu, Wd, k_keep, prio_dev, w.n_dev, drops[s],
                           ys[s], ws, mask=masks[s], stream=st)

    def step_ahead(s):
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

    def step(s):
        calls[s]()

    # ---- warm-up -----------------------------------------------------------------------
    torch.cuda.synchronize()
    (step_serial_q4 if args.q4 else step_serial)(0)   # also provides masks[0] for the overlapped form
    for s in range(W):
        step(s)
    torch.cuda.synchronize()
    if not args.serial:
        ws_scores = torch.empty((T, G), dtype=torch.float32, device=dev)

        def prologue():                     # masks[W] for the first timed step (untimed)
            At, Bt = copies[W % NC][:2]
            H.halo_predict_scores(shape, xs[W], At, Bt, ws_scores, ws, stream=st)
            H.halo_build_group_mask(ws_scores, k_keep, prio_dev, w.n_dev, drops[W], masks[W], stream=st)
    else:
        def prologue():
            pass

    # ---- timed: K steps ------------------------------------------------------------------
    use_graph = not args.no_graph
    if use_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            for s in range(W, W + K):
                step(s)
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            graph.replay()                  # untimed: first replay uploads the graph
        prologue()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(st):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        prologue()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(W, W + K):
            step(s)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    y_timed = ys[W:W + K].clone()

    # ---- dominant kernel under HIP events (eager pass over the same steps) -------------
    prologue()
    H.halo_profile_begin(K, args.time_every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(W, W + K):
        step(s)
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
    gate_up_bytes = float(union.sum()) * 2 * group_bytes  # over the K launches
    ffn_bytes = float(union.sum()) * 3 * group_bytes
    pred_bytes = K * (w.rank * d + G * w.rank) * esz
    # bytes of exactly the launches that were timed (every args.time_every-th step)
    timed_union = union[::args.time_every][:kern_n]
    gate_up_bytes = float(timed_union.sum()) * 2 * group_bytes
    achieved = gate_up_bytes / (kern_ms * 1e-3) / 1e9 if kern_ms > 0 else 0.0
    traffic = read_traffic(kern_name, w.name + ("_q4" if args.q4 else ""))
    if "_pf" in kern_name:
        # many tokens: the dominant kernel is a dense contraction on the matrix cores
        flops = float(n_surv[::args.time_every][:kern_n].sum()) * w.group_size * d * 2 * 2   # gate and up, 2 flop per MAC
        roof = {"bound": "mfma", "kernel": kern_name, "achieved": flops / (kern_ms * 1e-3) / 1e12,
                "peak": 2500.0, "unit": "TFLOP/s", "frac": flops / (kern_ms * 1e-3) / 1e12 / 2500.0,
                "traffic": traffic, "launches": int(kern_n), "avg_us": kern_ms / max(kern_n, 1) * 1e3,
                "flops_per_launch": flops / max(kern_n, 1),
                "hbm_GBps_of_this_kernel": achieved}
    else:
        roof = {"bound": "hbm", "kernel": kern_name, "achieved": achieved, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                "launches": int(kern_n), "avg_us": kern_ms / max(kern_n, 1) * 1e3,
                "bytes_per_launch": gate_up_bytes / max(kern_n, 1)}

    out = {
        "metric": ("FFN tokens/s (decode), LLaMA-7B shape, 50% groups kept" if w.name == "llama7b_decode"
                   else f"FFN tokens/s, {w.name}, keep {w.keep[0]}") + (", 4-bit weights" if args.q4 else ""),
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
                   "rank": w.rank, "tokens_per_step": T, "k_keep": k_keep, "n_dev": w.n_dev,
                   "plr": [float(v) for v in w.device_plr()], "seed": w.seed, "weight_copies": NC,
                   "graph": use_graph, "predictor": "serial" if args.serial else "one step ahead, beside the FFN"},
        "whole_pass": {
            "mean_n_surv": float(n_surv.mean()), "mean_union": float(union.mean()),
            "weight_GBps": ffn_bytes / elapsed / 1e9,
            "total_GBps": (ffn_bytes + pred_bytes) / elapsed / 1e9,
            "frac_of_hbm_peak": ffn_bytes / elapsed / 1e9 / HBM_PEAK_GBPS,
            "graph_equals_eager": same,
            "event_pass_us_per_step": t_eager / K * 1e6, "event_pass_host_us_per_step": t_enq / K * 1e6,
        },
        "roofline": roof,
    }

    # ---- CPU oracle on a bounded sample of the same steps (rank 0, N=1) -----------------
    if not args.no_cpu:
        from oracle import ref
        if args.q4:
            At, Bt = (t.float().cpu().numpy() for t in copies[0][:2])
            Wg, Wu, WdT = ref.dequant_ffn_q4([t.float().cpu().numpy() if t.dtype == torch.bfloat16
                                              else t.cpu().numpy() for t in copies[0][2]])
        else:
            At, Bt, Wg, Wu, WdT = (t.float().cpu().numpy() for t in (*copies[0][:4], WdT0))
        sample = [s for s in range(W, W + K) if s % NC == 0][: max(1, min(args.cpu_steps, 64 // T))]
        if not sample:
            sample = [W]
        x_np = xs.float().cpu().numpy()
        t0 = time.perf_counter()
        outs = [ref.ffn_forward(x_np[s], At, Bt, Wg, Wu, WdT, w.group_size, k_keep, prio_dev_np,
                                w.n_dev, drops_np[s]) for s in sample]
        cpu_t = time.perf_counter() - t0
        worst, masks_ok = 0.0, True
        y_np = ys.float().cpu().numpy()
        for s, o in zip(sample, outs):
            masks_ok &= bool(np.array_equal(o["mask"], masks[s].cpu().numpy()))
            den = np.linalg.norm(o["y"])
            if den > 0:
                worst = max(worst, float(np.linalg.norm(y_np[s] - o["y"]) / den))
        out["cpu_baseline"] = {
            "value": len(sample) * T / cpu_t, "unit": "tokens/s", "cores": ref.num_threads(),
            "kind": "oracle",
            "sample": f"{len(sample)} of the {K} timed steps (those on weight copy 0), whole pass each",
            "ms_per_step": cpu_t / len(sample) * 1e3,
            "gpu_vs_oracle_max_rel_l2": worst, "masks_bit_exact": masks_ok,
        }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
