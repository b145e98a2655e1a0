"""ctypes binding of libhalo.so: marshalling only (pointers, sizes, the current stream)."""
from __future__ import annotations

import ctypes as C
import os
import threading
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhalo.so")
_lib = None
_tls = threading.local()      # prepared(): the recorder standing in for the library in this thread, if any

HALO_F32, HALO_BF16 = 0, 1


class HaloError(RuntimeError):
    def __init__(self, fn: str, code: int):
        self.code = code
        msg = load_library().halo_status_string(code).decode()
        super().__init__(f"{fn} failed: {msg} ({code})")


class _CShape(C.Structure):
    _fields_ = [("d", C.c_int32), ("ffn", C.c_int32), ("group_size", C.c_int32),
                ("n_groups", C.c_int32), ("rank", C.c_int32), ("dtype", C.c_int32)]


class _CMhaShape(C.Structure):
    _fields_ = [("d", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32), ("rank", C.c_int32),
                ("dtype", C.c_int32)]


class MhaShape:
    """halo_mha_shape: d, n_heads, head_dim, rank, dtype ('bf16')."""

    def __init__(self, d: int, n_heads: int, head_dim: int, rank: int, dtype: str = "bf16"):
        self.d, self.n_heads, self.head_dim, self.rank, self.dtype = d, n_heads, head_dim, rank, dtype
        code = {"f32": HALO_F32, "bf16": HALO_BF16}.get(dtype, -1)
        self.c = _CMhaShape(d, n_heads, head_dim, rank, code)


class Shape:
    """halo_shape: d, ffn, group_size, n_groups, rank, dtype ('f32' | 'bf16')."""

    def __init__(self, d: int, ffn: int, group_size: int, rank: int, dtype: str = "bf16",
                 n_groups: Optional[int] = None):
        self.d, self.ffn, self.group_size, self.rank = d, ffn, group_size, rank
        self.n_groups = ffn // group_size if n_groups is None else n_groups
        self.dtype = dtype
        code = {"f32": HALO_F32, "bf16": HALO_BF16}.get(dtype, -1)
        self.c = _CShape(d, ffn, group_size, self.n_groups, rank, code)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libhalo.so (built in-tree by paper_2601_11676_amd.build).  There is no fallback:
    a missing library is an error."""
    global _lib
    stack = getattr(_tls, "recorders", None)
    if stack:
        return stack[-1]
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2601_11676_amd.build`")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    ps = C.POINTER(_CShape)
    lib.halo_status_string.restype = C.c_char_p
    lib.halo_status_string.argtypes = [C.c_int]
    lib.halo_build_schedule.restype = C.c_int
    lib.halo_build_schedule.argtypes = [i32, i32, vp, vp, vp]
    lib.halo_ratios_comp_greedy.restype = C.c_int
    lib.halo_ratios_comp_greedy.argtypes = [i32, vp, vp, C.c_double, vp]
    lib.halo_ratios_min_max.restype = C.c_int
    lib.halo_ratios_min_max.argtypes = [i32, vp, vp, C.c_double, C.c_double, vp]
    lib.halo_workspace_bytes.restype = sz
    lib.halo_workspace_bytes.argtypes = [ps, i32, i32]
    lib.halo_workspace_bytes_q4.restype = sz
    lib.halo_workspace_bytes_q4.argtypes = [ps, i32, i32]
    lib.halo_predict_scores.restype = C.c_int
    lib.halo_predict_scores.argtypes = [ps, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.halo_build_group_mask.restype = C.c_int
    lib.halo_build_group_mask.argtypes = [vp, i32, i32, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.halo_group_sparse_ffn.restype = C.c_int
    lib.halo_group_sparse_ffn.argtypes = [ps, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.halo_ffn_forward.restype = C.c_int
    lib.halo_ffn_forward.argtypes = [ps, vp, vp, i32, vp, vp, vp, vp, vp, i32, vp, i32, vp, vp,
                                     vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.halo_static_scratch_bytes.restype = sz
    lib.halo_static_scratch_bytes.argtypes = []
    lib.halo_ffn_forward_static.restype = C.c_int
    lib.halo_ffn_forward_static.argtypes = [ps, vp, vp, i32, vp, vp, vp, vp, vp, i32, vp, i32, vp, vp,
                                            vp, vp, vp, vp, vp, vp, vp]
    lib.halo_ffn_forward_ahead.restype = C.c_int
    lib.halo_ffn_forward_ahead.argtypes = [ps, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, i32,
                                           vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.halo_group_sparse_ffn_q4.restype = C.c_int
    lib.halo_group_sparse_ffn_q4.argtypes = [ps, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.halo_ffn_forward_q4.restype = C.c_int
    lib.halo_ffn_forward_q4.argtypes = [ps, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, i32, vp,
                                        vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.halo_ffn_forward_ahead_q4.restype = C.c_int
    lib.halo_ffn_forward_ahead_q4.argtypes = [ps, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp,
                                              i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    pm = C.POINTER(_CMhaShape)
    lib.halo_mha_workspace_bytes.restype = sz
    lib.halo_mha_workspace_bytes.argtypes = [pm, i32]
    lib.halo_head_sparse_mha.restype = C.c_int
    lib.halo_head_sparse_mha.argtypes = [pm, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, sz, vp]
    lib.halo_mha_forward.restype = C.c_int
    lib.halo_mha_forward.argtypes = [pm, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, i32, vp, vp,
                                     vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.halo_mha_forward_ahead.restype = C.c_int
    lib.halo_mha_forward_ahead.argtypes = [pm, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, i32, vp,
                                           i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.halo_profile_begin.restype = C.c_int
    lib.halo_profile_begin.argtypes = [i32, i32]
    lib.halo_profile_end.restype = C.c_int
    lib.halo_profile_end.argtypes = [vp, vp, vp, i32]
    lib.halo_stack_residual_norm.restype = C.c_int
    lib.halo_stack_residual_norm.argtypes = [vp, vp, vp, i32, i32, i32, C.c_float, vp]
    lib.halo_peak_read_stream.restype = C.c_int
    lib.halo_peak_read_stream.argtypes = [vp, sz, sz, i32, vp, vp, vp, vp]
    lib.halo_peak_mfma_bf16.restype = C.c_int
    lib.halo_peak_mfma_bf16.argtypes = [i32, i32, vp, vp, vp]
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _check(fn: str, rc: int):
    if rc != 0:
        raise HaloError(fn, rc)


def pack_down_proj(WdT: torch.Tensor, group_size: int) -> torch.Tensor:
    """Re-arrange a neuron-major down projection WdT [ffn][d] (row n = the weights leaving
    neuron n) into the library's group-blocked layout Wd [n_groups][d][group_size].
    Data movement only."""
    ffn, d = WdT.shape
    return WdT.view(ffn // group_size, group_size, d).permute(0, 2, 1).contiguous()


def halo_build_schedule(n_prio: int, plr: Sequence[float],
                        ratios: Optional[Sequence[float]] = None) -> np.ndarray:
    """Host-only (Alg. 3).  Returns prio_dev as an int8 numpy array of length n_prio."""
    plr_a = np.ascontiguousarray(np.asarray(plr, dtype=np.float64))
    rat_a = None if ratios is None else np.ascontiguousarray(np.asarray(ratios, dtype=np.float64))
    if rat_a is not None and rat_a.shape != plr_a.shape:
        raise ValueError("ratios and plr must have one entry per device")
    out = np.zeros(max(int(n_prio), 0), dtype=np.int8)
    rc = load_library().halo_build_schedule(
        int(n_prio), int(plr_a.shape[0]),
        None if rat_a is None else rat_a.ctypes.data_as(C.c_void_p),
        plr_a.ctypes.data_as(C.c_void_p), out.ctypes.data_as(C.c_void_p))
    _check("halo_build_schedule", rc)
    return out


def _host_ratios(name, mem, comp, demand, *extra) -> np.ndarray:
    m = np.ascontiguousarray(np.asarray(mem, dtype=np.float64))
    c = np.ascontiguousarray(np.asarray(comp, dtype=np.float64))
    if m.shape != c.shape or m.ndim != 1:
        raise ValueError("mem and comp must have one entry per device")
    r = np.zeros_like(m)
    rc = getattr(load_library(), name)(int(m.shape[0]), m.ctypes.data_as(C.c_void_p),
                                       c.ctypes.data_as(C.c_void_p), float(demand), *extra,
                                       r.ctypes.data_as(C.c_void_p))
    _check(name, rc)
    return r


def halo_ratios_comp_greedy(mem, comp, demand: float) -> np.ndarray:
    """Host-only (Alg. 1)."""
    return _host_ratios("halo_ratios_comp_greedy", mem, comp, demand)


def halo_ratios_min_max(mem, comp, demand: float, eps: float = 1e-3) -> np.ndarray:
    """Host-only (Alg. 2)."""
    return _host_ratios("halo_ratios_min_max", mem, comp, demand, float(eps))


def halo_workspace_bytes(shape: Shape, T: int, k_keep: int) -> int:
    return int(load_library().halo_workspace_bytes(C.byref(shape.c), int(T), int(k_keep)))


def halo_workspace_bytes_q4(shape: Shape, T: int, k_keep: int) -> int:
    return int(load_library().halo_workspace_bytes_q4(C.byref(shape.c), int(T), int(k_keep)))


def halo_predict_scores(shape: Shape, x, At, Bt, scores, workspace, stream=None) -> None:
    T = x.shape[0]
    rc = load_library().halo_predict_scores(C.byref(shape.c), _ptr(x), T, _ptr(At), _ptr(Bt),
                                            _ptr(scores), _ptr(workspace), workspace.numel(),
                                            _stream(stream))
    _check("halo_predict_scores", rc)


def halo_build_group_mask(scores, k_keep: int, prio_dev, n_dev: int, drop, mask, order=None,
                          group_dev=None, surv_idx=None, n_surv=None, stream=None) -> None:
    T, G = scores.shape
    rc = load_library().halo_build_group_mask(_ptr(scores), T, G, int(k_keep), _ptr(prio_dev),
                                              int(n_dev), _ptr(drop), _ptr(order), _ptr(group_dev),
                                              _ptr(mask), _ptr(surv_idx), _ptr(n_surv),
                                              _stream(stream))
    _check("halo_build_group_mask", rc)


def halo_group_sparse_ffn(shape: Shape, x, Wg, Wu, Wd, mask, y, workspace, stream=None) -> None:
    T = x.shape[0]
    rc = load_library().halo_group_sparse_ffn(C.byref(shape.c), _ptr(x), T, _ptr(Wg), _ptr(Wu),
                                              _ptr(Wd), _ptr(mask), _ptr(y), _ptr(workspace),
                                              workspace.numel(), _stream(stream))
    _check("halo_group_sparse_ffn", rc)


def halo_ffn_forward(shape: Shape, x, At, Bt, Wg, Wu, Wd, k_keep: int, prio_dev, n_dev: int,
                     drop, y, workspace, x_pred=None, scores=None, order=None, group_dev=None,
                     mask=None, surv_idx=None, n_surv=None, stream=None) -> None:
    T = x.shape[0]
    xp = x if x_pred is None else x_pred
    rc = load_library().halo_ffn_forward(
        C.byref(shape.c), _ptr(x), _ptr(xp), T, _ptr(At), _ptr(Bt), _ptr(Wg), _ptr(Wu), _ptr(Wd),
        int(k_keep), _ptr(prio_dev), int(n_dev), _ptr(drop), _ptr(y), _ptr(scores), _ptr(order),
        _ptr(group_dev), _ptr(mask), _ptr(surv_idx), _ptr(n_surv), _ptr(workspace),
        workspace.numel(), _stream(stream))
    _check("halo_ffn_forward", rc)


def halo_static_scratch_bytes() -> int:
    return int(load_library().halo_static_scratch_bytes())


def halo_ffn_forward_static(shape: Shape, x, At, Bt, Wg, Wu, Wd, k_keep: int, prio_dev, n_dev: int,
                            drop, y, x_pred=None, scores=None, order=None, group_dev=None,
                            mask=None, surv_idx=None, n_surv=None, stream=None) -> None:
    """halo_ffn_forward over the library's own fixed scratch array: no workspace argument."""
    T = x.shape[0]
    xp = x if x_pred is None else x_pred
    rc = load_library().halo_ffn_forward_static(
        C.byref(shape.c), _ptr(x), _ptr(xp), T, _ptr(At), _ptr(Bt), _ptr(Wg), _ptr(Wu), _ptr(Wd),
        int(k_keep), _ptr(prio_dev), int(n_dev), _ptr(drop), _ptr(y), _ptr(scores), _ptr(order),
        _ptr(group_dev), _ptr(mask), _ptr(surv_idx), _ptr(n_surv), _stream(stream))
    _check("halo_ffn_forward_static", rc)


def halo_ffn_forward_ahead(shape: Shape, x, Wg, Wu, Wd, mask_cur, y, x_pred_next, At_next, Bt_next,
                           k_keep: int, prio_dev, n_dev: int, drop_next, mask_next, workspace,
                           scores_next=None, order_next=None, group_dev_next=None,
                           surv_idx_next=None, n_surv_next=None, stream=None) -> None:
    T = x.shape[0]
    rc = load_library().halo_ffn_forward_ahead(
        C.byref(shape.c), _ptr(x), T, _ptr(Wg), _ptr(Wu), _ptr(Wd), _ptr(mask_cur), _ptr(y),
        _ptr(x_pred_next), _ptr(At_next), _ptr(Bt_next), int(k_keep), _ptr(prio_dev), int(n_dev),
        _ptr(drop_next), _ptr(scores_next), _ptr(order_next), _ptr(group_dev_next), _ptr(mask_next),
        _ptr(surv_idx_next), _ptr(n_surv_next), _ptr(workspace), workspace.numel(),
        _stream(stream))
    _check("halo_ffn_forward_ahead", rc)


def halo_group_sparse_ffn_q4(shape: Shape, x, q4, mask, y, workspace, stream=None) -> None:
    """q4 = (Wg_codes, Wg_scales, Wu_codes, Wu_scales, Wd_codes, Wd_scales), see include/halo.h."""
    T = x.shape[0]
    rc = load_library().halo_group_sparse_ffn_q4(
        C.byref(shape.c), _ptr(x), T, *[_ptr(t) for t in q4], _ptr(mask), _ptr(y), _ptr(workspace),
        workspace.numel(), _stream(stream))
    _check("halo_group_sparse_ffn_q4", rc)


def halo_ffn_forward_q4(shape: Shape, x, At, Bt, q4, k_keep: int, prio_dev, n_dev: int, drop, y, workspace,
                        x_pred=None, scores=None, order=None, group_dev=None, mask=None, surv_idx=None,
                        n_surv=None, stream=None) -> None:
    T = x.shape[0]
    xp = x if x_pred is None else x_pred
    rc = load_library().halo_ffn_forward_q4(
        C.byref(shape.c), _ptr(x), _ptr(xp), T, _ptr(At), _ptr(Bt), *[_ptr(t) for t in q4], int(k_keep),
        _ptr(prio_dev), int(n_dev), _ptr(drop), _ptr(y), _ptr(scores), _ptr(order), _ptr(group_dev),
        _ptr(mask), _ptr(surv_idx), _ptr(n_surv), _ptr(workspace), workspace.numel(), _stream(stream))
    _check("halo_ffn_forward_q4", rc)


def halo_ffn_forward_ahead_q4(shape: Shape, x, q4, mask_cur, y, x_pred_next, At_next, Bt_next, k_keep: int,
                              prio_dev, n_dev: int, drop_next, mask_next, workspace, scores_next=None,
                              order_next=None, group_dev_next=None, surv_idx_next=None, n_surv_next=None,
                              stream=None) -> None:
    T = x.shape[0]
    rc = load_library().halo_ffn_forward_ahead_q4(
        C.byref(shape.c), _ptr(x), T, *[_ptr(t) for t in q4], _ptr(mask_cur), _ptr(y), _ptr(x_pred_next),
        _ptr(At_next), _ptr(Bt_next), int(k_keep), _ptr(prio_dev), int(n_dev), _ptr(drop_next),
        _ptr(scores_next), _ptr(order_next), _ptr(group_dev_next), _ptr(mask_next), _ptr(surv_idx_next),
        _ptr(n_surv_next), _ptr(workspace), workspace.numel(), _stream(stream))
    _check("halo_ffn_forward_ahead_q4", rc)


def halo_mha_workspace_bytes(shape: MhaShape, max_len: int) -> int:
    return int(load_library().halo_mha_workspace_bytes(C.byref(shape.c), int(max_len)))


def halo_head_sparse_mha(shape: MhaShape, x, Wq, Wk, Wv, Wo, k_cache, v_cache, pos: int, mask, y, workspace,
                         stream=None) -> None:
    """k_cache / v_cache: [n_heads][max_len][head_dim]; Wo head-blocked (pack_down_proj(WoT, head_dim))."""
    rc = load_library().halo_head_sparse_mha(
        C.byref(shape.c), _ptr(x), _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(Wo), _ptr(k_cache), _ptr(v_cache),
        int(k_cache.shape[1]), int(pos), _ptr(mask), _ptr(y), _ptr(workspace), workspace.numel(), _stream(stream))
    _check("halo_head_sparse_mha", rc)


def halo_mha_forward(shape: MhaShape, x, At, Bt, Wq, Wk, Wv, Wo, k_cache, v_cache, pos: int, k_keep: int,
                     prio_dev, n_dev: int, drop, y, workspace, x_pred=None, scores=None, order=None,
                     group_dev=None, mask=None, surv_idx=None, n_surv=None, stream=None) -> None:
    xp = x if x_pred is None else x_pred
    rc = load_library().halo_mha_forward(
        C.byref(shape.c), _ptr(x), _ptr(xp), _ptr(At), _ptr(Bt), _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(Wo),
        _ptr(k_cache), _ptr(v_cache), int(k_cache.shape[1]), int(pos), int(k_keep), _ptr(prio_dev), int(n_dev),
        _ptr(drop), _ptr(y), _ptr(scores), _ptr(order), _ptr(group_dev), _ptr(mask), _ptr(surv_idx),
        _ptr(n_surv), _ptr(workspace), workspace.numel(), _stream(stream))
    _check("halo_mha_forward", rc)


def halo_mha_forward_ahead(shape: MhaShape, x, Wq, Wk, Wv, Wo, k_cache, v_cache, pos: int, mask_cur, y,
                           x_pred_next, At_next, Bt_next, k_keep: int, prio_dev, n_dev: int, drop_next, mask_next,
                           workspace, scores_next=None, order_next=None, group_dev_next=None, surv_idx_next=None,
                           n_surv_next=None, stream=None) -> None:
    rc = load_library().halo_mha_forward_ahead(
        C.byref(shape.c), _ptr(x), _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(Wo), _ptr(k_cache), _ptr(v_cache),
        int(k_cache.shape[1]), int(pos), _ptr(mask_cur), _ptr(y), _ptr(x_pred_next), _ptr(At_next), _ptr(Bt_next),
        int(k_keep), _ptr(prio_dev), int(n_dev), _ptr(drop_next), _ptr(scores_next), _ptr(order_next),
        _ptr(group_dev_next), _ptr(mask_next), _ptr(surv_idx_next), _ptr(n_surv_next), _ptr(workspace),
        workspace.numel(), _stream(stream))
    _check("halo_mha_forward_ahead", rc)


class _Recorder:
    """Stands in for the library inside prepared(): notes the one C call a wrapper makes instead of
    making it."""

    def __init__(self, lib):
        self._lib = lib
        self.calls = []

    def __getattr__(self, name):
        cfn = getattr(self._lib, name)

        def rec(*cargs):
            self.calls.append((cfn, cargs, name))
            return 0
        return rec


def prepared(fn, *args, **kwargs):
    """Marshal the arguments of one of the halo_* calls above once and return a zero-argument
    callable that repeats exactly that call (same pointers, same stream).  For launch-bound
    loops where per-call Python marshalling would dominate; the caller keeps the tensors alive.
    The recording is local to the calling thread (other threads keep calling the real library)
    and nests."""
    rec = _Recorder(load_library())
    stack = getattr(_tls, "recorders", None)
    if stack is None:
        stack = _tls.recorders = []
    stack.append(rec)
    try:
        fn(*args, **kwargs)
    finally:
        popped = stack.pop()
        assert popped is rec
    if len(rec.calls) != 1:
        raise RuntimeError("prepared() expects a function that makes exactly one library call")
    cfn, cargs, name = rec.calls[0]

    def call():
        rc = cfn(*cargs)
        if rc != 0:
            raise HaloError(name, rc)
    return call


def halo_profile_begin(max_launches: int, every: int = 1) -> None:
    _check("halo_profile_begin", load_library().halo_profile_begin(int(max_launches), int(every)))


def halo_profile_end():
    """Returns (total_ms, launches, kernel_name) of the dominant FFN kernel since begin."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    name = C.create_string_buffer(64)
    rc = load_library().halo_profile_end(C.byref(ms), C.byref(n), name, 64)
    _check("halo_profile_end", rc)
    return ms.value, n.value, name.value.decode()


def halo_peak_read_stream(buf, window_bytes: int, launches: int, sink, stream=None):
    """Returns (GB/s, microseconds per launch) of the read-stream aid over windows of `buf`."""
    g, us = C.c_double(0.0), C.c_double(0.0)
    rc = load_library().halo_peak_read_stream(_ptr(buf), buf.numel() * buf.element_size(), int(window_bytes),
                                              int(launches), _ptr(sink), _stream(stream), C.byref(g), C.byref(us))
    _check("halo_peak_read_stream", rc)
    return g.value, us.value


def halo_peak_mfma_bf16(iters: int, launches: int, sink, stream=None) -> float:
    """Returns the bf16 matrix-instruction rate of the MFMA aid in TFLOP/s."""
    t = C.c_double(0.0)
    rc = load_library().halo_peak_mfma_bf16(int(iters), int(launches), _ptr(sink), _stream(stream), C.byref(t))
    _check("halo_peak_mfma_bf16", rc)
    return t.value


def halo_stack_residual_norm(h, y, x, eps: float = 1e-5, stream=None) -> None:
    """h += y (y may be None); x = h / sqrt(mean(h^2) + eps), row by row.  h float32, x/y float32 or bf16."""
    T, d = h.shape
    if h.dtype != torch.float32:
        raise ValueError("h must be float32")
    code = HALO_F32 if x.dtype == torch.float32 else HALO_BF16
    rc = load_library().halo_stack_residual_norm(_ptr(h), _ptr(y), _ptr(x), int(T), int(d), code, float(eps),
                                                 _stream(stream))
    _check("halo_stack_residual_norm", rc)
