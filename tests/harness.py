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


def gpu_forward(w, layer: Layer, x, K, prio_dev_np, drop_np, x_pred=None):
    """halo_ffn_forward through the C boundary; returns numpy outputs."""
    s = shape_of(w)
    T, G = x.shape[0], w.n_groups
    ws = torch.empty(H.halo_workspace_bytes(s, T, K), dtype=torch.uint8, device=DEV)
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


def assert_parity(gpu, cpu, tol, what=""):
    """Bit-exact scores / ranking / masks / indices; y within relative L2 `tol`, per token and whole."""
    assert np.array_equal(gpu["scores"].view(np.uint32), cpu["scores"].view(np.uint32)), what + " scores"
    for k in INT_KEYS:
        assert np.array_equal(gpu[k], cpu[k]), f"{what} {k}"
    yg, yc = gpu["y"], cpu["y"]
    assert np.isfinite(yg).all(), what + " y finite"
    for t in range(yc.shape[0]):
        if cpu["n_surv"][t] == 0:
            assert not yg[t].any(), f"{what} token {t}: no survivor must give exact zeros"
        else:
            err = np.linalg.norm(yg[t] - yc[t]) / np.linalg.norm(yc[t])
            assert err <= tol, f"{what} token {t}: rel L2 {err:.3e} > {tol}"
    den = np.linalg.norm(yc)
    if den > 0:
        assert np.linalg.norm(yg - yc) / den <= tol, what + " whole tensor"
