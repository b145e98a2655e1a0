"""Glue used by the GPU parity tests: run the HIP path and the oracle on the same seeded
inputs.  The oracle is only ever called from here, smoke() and bench.py's CPU leg."""
import numpy as np
import torch

import halo_synth as hs
import paper_2601_11676_amd as H
from oracle import ref

DEV = "cuda:0"


def shape_of(w: hs.Workload) -> H.Shape:
    return H.Shape(w.d, w.ffn, w.group_size, w.rank, w.dtype)


def to_np32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


class Layer:
    """Device tensors of one layer of a workload (+ lazily, host float32 copies for the oracle)."""

    def __init__(self, w: hs.Workload, layer: int = 0, copy: int = 0):
        self.w = w
        self.Wg, self.Wu, self.WdT = hs.ffn_weights(w, layer, DEV, copy)
        self.Wd = H.pack_down_proj(self.WdT, w.group_size)     # the library's group-blocked layout
        self.At, self.Bt = hs.predictor_weights(w, layer, DEV, copy)
        self._host = None

    def host(self):
        if self._host is None:
            self._host = tuple(to_np32(t) for t in (self.At, self.Bt, self.Wg, self.Wu, self.WdT))
        return self._host


class Q4Layer:
    """One layer with 4-bit block-quantised FFN weights (device tensors in the library's storage
    format); host() gives the oracle its view: the dequantised float32 matrices."""

    def __init__(self, w: hs.Workload, layer: int = 0, copy: int = 0):
        self.w = w
        self.q4 = hs.ffn_weights_q4(w, layer, DEV, copy)
        self.At, self.Bt = hs.predictor_weights(w, layer, DEV, copy)
        self._host = None

    def host(self):
        if self._host is None:
            q = [t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy() for t in self.q4]
            self._host = (to_np32(self.At), to_np32(self.Bt)) + tuple(ref.dequant_ffn_q4(q))
        return self._host


def gpu_forward_q4(w, layer: Q4Layer, x, K, prio_dev_np, drop_np, big_workspace=False):
    """halo_ffn_forward_q4 through the C boundary; returns numpy outputs.  big_workspace: sized by
    halo_workspace_bytes_q4 (many tokens then run on expanded weights)."""
    s = shape_of(w)
    T, G = x.shape[0], w.n_groups
    size = H.halo_workspace_bytes_q4(s, T, K) if big_workspace else H.halo_workspace_bytes(s, T, K)
    ws = torch.empty(size, dtype=torch.uint8, device=DEV)
    pd = torch.from_numpy(np.ascontiguousarray(prio_dev_np)).to(DEV)
    dr = None if drop_np is None else torch.from_numpy(np.ascontiguousarray(drop_np)).to(DEV)
    y = torch.full((T, w.d), float("nan"), dtype=w.torch_dtype, device=DEV)
    scores = torch.empty((T, G), dtype=torch.float32, device=DEV)
    order = torch.empty((T, G), dtype=torch.int32, device=DEV)
    group_dev = torch.empty((T, G), dtype=torch.int8, device=DEV)
    mask = torch.empty((T, G), dtype=torch.uint8, device=DEV)
    surv_idx = torch.empty((T, max(K, 1)), dtype=torch.int32, device=DEV)[:, :K].contiguous()
    n_surv = torch.empty((T,), dtype=torch.int32, device=DEV)
    H.halo_ffn_forward_q4(s, x, layer.At, layer.Bt, layer.q4, K, pd, w.n_dev, dr, y, ws, scores=scores,
                          order=order, group_dev=group_dev, mask=mask, surv_idx=surv_idx, n_surv=n_surv)
    torch.cuda.synchronize()
    return dict(y=to_np32(y).astype(np.float64), scores=scores.cpu().numpy(),
                order=order.cpu().numpy(), group_dev=group_dev.cpu().numpy(),
                mask=mask.cpu().numpy(), surv_idx=surv_idx.cpu().numpy(), n_surv=n_surv.cpu().numpy())


def gpu_forward(w, layer: Layer, x, K, prio_dev_np, drop_np, x_pred=None, ws_tokens=None):
    """halo_ffn_forward through the C boundary; returns numpy outputs.  ws_tokens: size the
    workspace for that many tokens instead of x's."""
    s = shape_of(w)
    T, G = x.shape[0], w.n_groups
    ws = torch.empty(H.halo_workspace_bytes(s, T if ws_tokens is None else ws_tokens, K), dtype=torch.uint8,
                     device=DEV)
    pd = torch.from_numpy(np.ascontiguousarray(prio_dev_np)).to(DEV)
    dr = None if drop_np is None else torch.from_numpy(np.ascontiguousarray(drop_np)).to(DEV)
    y = torch.full((T, w.d), float("nan"), dtype=w.torch_dtype, device=DEV)
    scores = torch.empty((T, G), dtype=torch.float32, device=DEV)
    order = torch.empty((T, G), dtype=torch.int32, device=DEV)
    group_dev = torch.empty((T, G), dtype=torch.int8, device=DEV)
    mask = torch.empty((T, G), dtype=torch.uint8, device=DEV)
    surv_idx = torch.empty((T, max(K, 1)), dtype=torch.int32, device=DEV)[:, :K].contiguous()
    n_surv = torch.empty((T,), dtype=torch.int32, device=DEV)
    H.halo_ffn_forward(s, x, layer.At, layer.Bt, layer.Wg, layer.Wu, layer.Wd, K, pd, w.n_dev, dr,
                       y, ws, x_pred=x_pred, scores=scores, order=order, group_dev=group_dev,
                       mask=mask, surv_idx=surv_idx, n_surv=n_surv)
    torch.cuda.synchronize()
    return dict(y=to_np32(y).astype(np.float64), scores=scores.cpu().numpy(),
                order=order.cpu().numpy(), group_dev=group_dev.cpu().numpy(),
                mask=mask.cpu().numpy(), surv_idx=surv_idx.cpu().numpy(), n_surv=n_surv.cpu().numpy())


def oracle_forward(w, layer: Layer, x, K, prio_dev_np, drop_np, x_pred=None):
    At, Bt, Wg, Wu, WdT = layer.host()
    xn = to_np32(x)
    if x_pred is None:
        return ref.ffn_forward(xn, At, Bt, Wg, Wu, WdT, w.group_size, K, prio_dev_np, w.n_dev, drop_np)
    sc = ref.predict_scores(to_np32(x_pred), At, Bt)
    out = ref.build_group_mask(sc, K, prio_dev_np, w.n_dev, drop_np)
    out["scores"] = sc
    out["y"] = ref.group_sparse_ffn(xn, Wg, Wu, WdT, w.group_size, out["mask"])
    return out


INT_KEYS = ("order", "group_dev", "mask", "surv_idx", "n_surv")

# Element-wise bar beside the relative-L2 one: no single output may be off by more than this many
# root-mean-squares of its token's reference row.  A relative L2 of 2e-2 alone would let one wholly
# wrong element of a 4096-wide row through (1/sqrt(4096) = 1.6e-2); an element that is wrong by its
# own size is about one rms off.  bf16: the output rounding is 2^-9 of the element (elements reach
# ~4.5 rms) plus the rounded activation's share -- observed <= 1.9e-2 over every parity case, bar = three times that;
# f32: accumulation order only.
ELEM_TOL = {1e-5: 5e-5, 2e-2: 6e-2}
WORST = {"l2": 0.0, "elem": 0.0}          # largest ratios seen in this process (printed by the tests)


def check_y(yg, yc, n_surv, tol, what=""):
    """y of the HIP path against the oracle's: per token relative L2 <= tol and every element within
    ELEM_TOL[tol] of the token's reference rms; tokens with no surviving group exactly zero."""
    yg = np.asarray(yg, dtype=np.float64)
    yc = np.asarray(yc, dtype=np.float64)
    assert yg.shape == yc.shape, what + " shape"
    assert np.isfinite(yg).all(), what + " y finite"
    for t in range(yc.shape[0]):
        if n_surv[t] == 0:
            assert not yg[t].any(), f"{what} token {t}: no survivor must give exact zeros"
            continue
        diff = yg[t] - yc[t]
        err = np.linalg.norm(diff) / np.linalg.norm(yc[t])
        assert err <= tol, f"{what} token {t}: rel L2 {err:.3e} > {tol}"
        rms = np.sqrt(np.mean(yc[t] ** 2))
        worst = np.abs(diff).max() / rms
        assert worst <= ELEM_TOL[tol], f"{what} token {t}: element {int(np.abs(diff).argmax())} off by {worst:.3e} rms"
        if tol > 1e-3:
            WORST["l2"] = max(WORST["l2"], err)
            WORST["elem"] = max(WORST["elem"], worst)
    den = np.linalg.norm(yc)
    if den > 0:
        assert np.linalg.norm(yg - yc) / den <= tol, what + " whole tensor"


def assert_parity(gpu, cpu, tol, what=""):
    """Bit-exact scores / ranking / masks / indices; y within `tol` (relative L2, per token and whole)
    and within the element-wise bar."""
    assert np.array_equal(gpu["scores"].view(np.uint32), cpu["scores"].view(np.uint32)), what + " scores"
    for k in INT_KEYS:
        assert np.array_equal(gpu[k], cpu[k]), f"{what} {k}"
    check_y(gpu["y"], cpu["y"], cpu["n_surv"], tol, what)


# --------------------------------------------------------------------------
# FFN stacks (the 13B x 40 and 70B x 80 workloads)
# --------------------------------------------------------------------------
def rms_norm(h: torch.Tensor) -> torch.Tensor:
    """x = h / sqrt(mean(h^2) + 1e-5) in float32 (no gain).  Harness glue between layers: the
    workloads are FFN-only stacks, so a norm keeps the residual stream bounded."""
    return h * torch.rsqrt(h.pow(2).mean(dim=-1, keepdim=True) + 1e-5)


def stack_check_layers(w, n_random):
    """Layers whose output is compared with the oracle: the first three, the middle pair, the last
    pair, and n_random more drawn from the workload's seed."""
    L = w.layers
    fixed = {0, 1, 2, L // 2 - 1, L // 2, L - 2, L - 1}
    rest = [l for l in range(L) if l not in fixed]
    u = hs.uniform01(len(rest), hs.stream_key(w.seed, hs.TID_MISC, 77))
    picked = [rest[i] for i in np.argsort(u, kind="stable")[:n_random]]
    return sorted(fixed | set(picked))


def run_stack_gpu(w, keep, layers=None, check_layers=(), on_layer=None, q4=False):
    """Free-running stack on the GPU with the predictor one layer ahead (layer l+1's mask is
    predicted from layer l's input, as in the paper); layer 0 runs dense and lossless.
    q4: the layers' FFN weights are 4-bit block-quantised and the `_q4` entry points run.
    For each layer of check_layers, on_layer(l, rec, pd_np, K) is called with
    rec = dict(x, x_prev, y, mask, drop, host) (host copies) while the run goes on -- records
    are not kept, a 70B layer is 2.8 GB as float32.  Returns the final residual stream."""
    s = shape_of(w)
    n_layers = w.layers if layers is None else layers
    T, G = w.T, w.n_groups
    K = w.k_keep(keep)
    pd_np = H.halo_build_schedule(K, w.device_plr())
    pd = torch.from_numpy(pd_np).to(DEV)
    ws = torch.empty(H.halo_workspace_bytes(s, T, G), dtype=torch.uint8, device=DEV)
    h = hs.hidden_states(w, 0, DEV, dtype=torch.float32)
    mask = torch.ones((T, G), dtype=torch.uint8, device=DEV)          # layer 0: every group, no loss
    make = Q4Layer if q4 else Layer
    cur = make(w, 0)
    x_prev = None
    for l in range(n_layers):
        nxt = make(w, l + 1) if l + 1 < n_layers else None
        x = rms_norm(h).to(w.torch_dtype)
        y = torch.empty((T, w.d), dtype=w.torch_dtype, device=DEV)
        if nxt is not None:
            drop_next = hs.drop_outcomes(w, l + 1, 0)
            mask_next = torch.empty((T, G), dtype=torch.uint8, device=DEV)
            if q4:
                H.halo_ffn_forward_ahead_q4(s, x, cur.q4, mask, y, x, nxt.At, nxt.Bt, K, pd, w.n_dev,
                                            torch.from_numpy(drop_next).to(DEV), mask_next, ws)
            else:
                H.halo_ffn_forward_ahead(s, x, cur.Wg, cur.Wu, cur.Wd, mask, y, x, nxt.At, nxt.Bt, K, pd,
                                         w.n_dev, torch.from_numpy(drop_next).to(DEV), mask_next, ws)
        elif q4:
            H.halo_group_sparse_ffn_q4(s, x, cur.q4, mask, y, ws)
        else:
            H.halo_group_sparse_ffn(s, x, cur.Wg, cur.Wu, cur.Wd, mask, y, ws)
        torch.cuda.synchronize()
        if l in check_layers and on_layer is not None:
            rec = dict(x=to_np32(x), x_prev=None if x_prev is None else to_np32(x_prev),
                       y=to_np32(y).astype(np.float64), mask=mask.cpu().numpy(),
                       host=cur.host(), drop=None if l == 0 else hs.drop_outcomes(w, l, 0))
            on_layer(l, rec, pd_np, K)
            del rec
        h = h + y.float()
        x_prev = x
        if nxt is not None:
            mask = mask_next
        cur._host = None
        cur = nxt
    return h


def check_stack_layer(w, l, rec, pd_np, K, tol):
    """Teacher-forced parity of one layer: the oracle gets the GPU's own layer inputs."""
    At, Bt, Wg, Wu, WdT = rec["host"]
    G = w.n_groups
    if l == 0:
        mask_ref = np.ones((w.T, G), np.uint8)
    else:
        sc = ref.predict_scores(rec["x_prev"], At, Bt)
        mask_ref = ref.build_group_mask(sc, K, pd_np, w.n_dev, rec["drop"])["mask"]
    assert np.array_equal(rec["mask"], mask_ref), f"layer {l}: mask"
    y_ref = ref.group_sparse_ffn(rec["x"], Wg, Wu, WdT, w.group_size, mask_ref)
    check_y(rec["y"], y_ref, mask_ref.sum(axis=1), tol, f"layer {l}")
