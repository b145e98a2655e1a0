"""Helpers shared by the tests (fixture parsing, error norms)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name):
    """Parse 'key v v v' / 'device i: v v' lines into a dict of lists of floats/ints."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("device"):
                head, vals = line.split(":")
                out.setdefault("device", {})[int(head.split()[1])] = [int(v) for v in vals.split()]
            else:
                k, *vals = line.split()
                out[k] = [float(v) if ("." in v or "e" in v) else int(v) for v in vals]
    return out


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def drop_strategy_case():
    """Inputs of the drop-strategy comparison (paper Sec. II-C): a bf16 FFN block whose groups get a
    heavy-tailed output scale (2^(g mod 5) on the down projection), so that the groups' partial-output
    norms differ the way the paper observes for real activations.  Returns the workload, K, and host
    tensors (torch, bf16): x, Wg, Wu, WdT."""
    import dataclasses

    import torch

    import halo_synth as hs

    w = dataclasses.replace(hs.LLAMA13B_STACK, name="case", d=1024, ffn=16 * 128, rank=64, T=8, layers=1, seed=41)
    Wg, Wu, WdT = hs.ffn_weights(w, 0, "cpu")
    scale = torch.tensor([2.0 ** (g % 5) for g in range(w.n_groups)]).repeat_interleave(128)
    WdT = (WdT.float() * scale[:, None]).to(torch.bfloat16)
    x = hs.hidden_states(w, 0, "cpu")
    return w, 8, x, Wg, Wu, WdT


def drop_strategy_scores(w, norms):
    """Significance values of the three strategies for [T][G] partial-output norms: the norms
    themselves (lose the low-norm groups), seeded uniforms (Random), the negated norms (lose the
    high-norm groups)."""
    import halo_synth as hs

    T, G = norms.shape
    rnd = hs.uniform01(T * G, hs.stream_key(w.seed, hs.TID_MISC)).astype(np.float32).reshape(T, G)
    return {"low_norm": np.ascontiguousarray(norms, dtype=np.float32), "random": rnd,
            "high_norm": np.ascontiguousarray(-norms, dtype=np.float32)}
