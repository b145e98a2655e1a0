"""ctypes front end of the CPU oracle (oracle/halo_ref.c) -- test infrastructure only.

Takes numpy arrays (float inputs as float32 holding the storage-dtype values,
widened exactly) and returns numpy arrays.  No arithmetic of the method lives
here: every function marshals arguments and calls the C oracle.
"""
from __future__ import annotations

import ctypes as C
from typing import Optional

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.ensure_built())
    return _lib


def _p(a: Optional[np.ndarray], ct):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(ct))


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def num_threads() -> int:
    return int(lib().halo_ref_num_threads())


def schedule(n_prio: int, plr, ratios=None) -> np.ndarray:
    """prio_dev[p] = device that executes priority index p (Alg. 3)."""
    plr = np.ascontiguousarray(np.asarray(plr, dtype=np.float64))
    rat = None if ratios is None else np.ascontiguousarray(np.asarray(ratios, dtype=np.float64))
    out = np.full(max(n_prio, 0), -7, dtype=np.int8)
    rc = lib().halo_ref_schedule(C.c_int32(n_prio), C.c_int32(len(plr)), _p(rat, C.c_double),
                                 _p(plr, C.c_double), _p(out, C.c_int8))
    if rc != 0:
        raise ValueError("halo_ref_schedule rejected its arguments")
    return out


def _ratios(fn_name, m, c, Mt, *extra):
    m = np.ascontiguousarray(np.asarray(m, dtype=np.float64))
    c = np.ascontiguousarray(np.asarray(c, dtype=np.float64))
    assert m.shape == c.shape
    r = np.full(m.shape, np.nan)
    rc = getattr(lib(), fn_name)(C.c_int32(len(m)), _p(m, C.c_double), _p(c, C.c_double), C.c_double(Mt),
                                 *[C.c_double(e) for e in extra], _p(r, C.c_double))
    if rc != 0:
        raise ValueError(fn_name + " rejected its arguments")
    return r


def ratios_comp_greedy(m, c, Mt) -> np.ndarray:
    """Alg. 1: workload ratios, fastest devices filled first."""
    return _ratios("halo_ref_ratios_comp_greedy", m, c, Mt)


def ratios_min_max(m, c, Mt, eps: float = 1e-3) -> np.ndarray:
    """Alg. 2: workload ratios minimising the largest per-device time."""
    return _ratios("halo_ref_ratios_min_max", m, c, Mt, eps)


def predict_scores(x, At, Bt, want64: bool = False):
    x, At, Bt = _f32(x), _f32(At), _f32(Bt)
    T, d = x.shape
    r, d2 = At.shape
    G, r2 = Bt.shape
    assert d == d2 and r == r2
    s = np.empty((T, G), dtype=np.float32)
    s64 = np.empty((T, G), dtype=np.float64) if want64 else None
    rc = lib().halo_ref_predict_scores(_p(x, C.c_float), C.c_int32(T), C.c_int32(d), C.c_int32(r),
                                       C.c_int32(G), _p(At, C.c_float), _p(Bt, C.c_float),
                                       _p(s, C.c_float), _p(s64, C.c_double))
    if rc != 0:
        raise ValueError("halo_ref_predict_scores rejected its arguments")
    return (s, s64) if want64 else s


def build_group_mask(scores, K: int, prio_dev, n_dev: int, drop=None):
    scores = _f32(scores)
    T, G = scores.shape
    prio_dev = np.ascontiguousarray(np.asarray(prio_dev, dtype=np.int8))
    assert prio_dev.shape == (K,)
    dr = None if drop is None else np.ascontiguousarray(np.asarray(drop, dtype=np.uint8))
    if dr is not None:
        assert dr.shape == (T, n_dev)
    order = np.empty((T, G), dtype=np.int32)
    group_dev = np.empty((T, G), dtype=np.int8)
    mask = np.empty((T, G), dtype=np.uint8)
    surv_idx = np.empty((T, K), dtype=np.int32)
    n_surv = np.empty((T,), dtype=np.int32)
    rc = lib().halo_ref_build_group_mask(_p(scores, C.c_float), C.c_int32(T), C.c_int32(G),
                                         C.c_int32(K), _p(prio_dev, C.c_int8), C.c_int32(n_dev),
                                         _p(dr, C.c_uint8), _p(order, C.c_int32),
                                         _p(group_dev, C.c_int8), _p(mask, C.c_uint8),
                                         _p(surv_idx, C.c_int32), _p(n_surv, C.c_int32))
    if rc != 0:
        raise ValueError("halo_ref_build_group_mask rejected its arguments")
    return dict(order=order, group_dev=group_dev, mask=mask, surv_idx=surv_idx, n_surv=n_surv)


def _ffn_args(x, Wg, Wu, WdT, gs):
    x, Wg, Wu, WdT = _f32(x), _f32(Wg), _f32(Wu), _f32(WdT)
    T, d = x.shape
    ffn, d2 = Wg.shape
    assert d == d2 and Wu.shape == Wg.shape and WdT.shape == Wg.shape and ffn % gs == 0
    return x, Wg, Wu, WdT, T, d, ffn // gs


def group_partials(x, Wg, Wu, WdT, gs: int, mask=None) -> np.ndarray:
    x, Wg, Wu, WdT, T, d, G = _ffn_args(x, Wg, Wu, WdT, gs)
    m = None if mask is None else np.ascontiguousarray(np.asarray(mask, dtype=np.uint8))
    out = np.empty((T, G, d), dtype=np.float64)
    rc = lib().halo_ref_group_partials(_p(x, C.c_float), C.c_int32(T), C.c_int32(d), C.c_int32(G),
                                       C.c_int32(gs), _p(Wg, C.c_float), _p(Wu, C.c_float),
                                       _p(WdT, C.c_float), _p(m, C.c_uint8), _p(out, C.c_double))
    if rc != 0:
        raise ValueError("halo_ref_group_partials rejected its arguments")
    return out


def group_sparse_ffn(x, Wg, Wu, WdT, gs: int, mask=None) -> np.ndarray:
    x, Wg, Wu, WdT, T, d, G = _ffn_args(x, Wg, Wu, WdT, gs)
    m = None if mask is None else np.ascontiguousarray(np.asarray(mask, dtype=np.uint8))
    if m is not None:
        assert m.shape == (T, G)
    y = np.empty((T, d), dtype=np.float64)
    rc = lib().halo_ref_group_sparse_ffn(_p(x, C.c_float), C.c_int32(T), C.c_int32(d),
                                         C.c_int32(G), C.c_int32(gs), _p(Wg, C.c_float),
                                         _p(Wu, C.c_float), _p(WdT, C.c_float), _p(m, C.c_uint8),
                                         _p(y, C.c_double))
    if rc != 0:
        raise ValueError("halo_ref_group_sparse_ffn rejected its arguments")
    return y


def ffn_forward(x, At, Bt, Wg, Wu, WdT, gs: int, K: int, prio_dev, n_dev: int, drop=None):
    """Whole pass; returns dict(y, scores, order, group_dev, mask, surv_idx, n_surv)."""
    x, Wg, Wu, WdT, T, d, G = _ffn_args(x, Wg, Wu, WdT, gs)
    At, Bt = _f32(At), _f32(Bt)
    r = At.shape[0]
    assert At.shape == (r, d) and Bt.shape == (G, r)
    prio_dev = np.ascontiguousarray(np.asarray(prio_dev, dtype=np.int8))
    assert prio_dev.shape == (K,)
    dr = None if drop is None else np.ascontiguousarray(np.asarray(drop, dtype=np.uint8))
    y = np.empty((T, d), dtype=np.float64)
    scores = np.empty((T, G), dtype=np.float32)
    order = np.empty((T, G), dtype=np.int32)
    group_dev = np.empty((T, G), dtype=np.int8)
    mask = np.empty((T, G), dtype=np.uint8)
    surv_idx = np.empty((T, K), dtype=np.int32)
    n_surv = np.empty((T,), dtype=np.int32)
    rc = lib().halo_ref_ffn_forward(
        _p(x, C.c_float), C.c_int32(T), C.c_int32(d), C.c_int32(G), C.c_int32(gs), C.c_int32(r),
        _p(At, C.c_float), _p(Bt, C.c_float), _p(Wg, C.c_float), _p(Wu, C.c_float),
        _p(WdT, C.c_float), C.c_int32(K), _p(prio_dev, C.c_int8), C.c_int32(n_dev),
        _p(dr, C.c_uint8), _p(y, C.c_double), _p(scores, C.c_float), _p(order, C.c_int32),
        _p(group_dev, C.c_int8), _p(mask, C.c_uint8), _p(surv_idx, C.c_int32),
        _p(n_surv, C.c_int32))
    if rc != 0:
        raise ValueError("halo_ref_ffn_forward rejected its arguments")
    return dict(y=y, scores=scores, order=order, group_dev=group_dev, mask=mask,
                surv_idx=surv_idx, n_surv=n_surv)


def _u32(a) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(a))
    assert a.dtype in (np.int32, np.uint32)
    return a.view(np.uint32)


def dequant_q4(codes, scales) -> np.ndarray:
    """Row-major 4-bit matrix -> float32 [rows][cols] (blocks of 128 along cols)."""
    codes, scales = _u32(codes), _f32(scales)
    rows, cols = codes.shape[0], codes.shape[1] * 8
    assert scales.shape == (rows, cols // 128)
    out = np.empty((rows, cols), dtype=np.float32)
    rc = lib().halo_ref_dequant_q4(_p(codes, C.c_uint32), _p(scales, C.c_float), C.c_int64(rows),
                                   C.c_int32(cols), _p(out, C.c_float))
    if rc != 0:
        raise ValueError("halo_ref_dequant_q4 rejected its arguments")
    return out


def dequant_down_q4(codes, scales) -> np.ndarray:
    """Group-blocked 4-bit down projection [G][d][gs/8] -> float32 WdT [G*gs][d]."""
    codes, scales = _u32(codes), _f32(scales)
    G, d, gs = codes.shape[0], codes.shape[1], codes.shape[2] * 8
    assert scales.shape == (G, d)
    out = np.empty((G * gs, d), dtype=np.float32)
    rc = lib().halo_ref_dequant_down_q4(_p(codes, C.c_uint32), _p(scales, C.c_float), C.c_int32(G),
                                        C.c_int32(d), C.c_int32(gs), _p(out, C.c_float))
    if rc != 0:
        raise ValueError("halo_ref_dequant_down_q4 rejected its arguments")
    return out


def dequant_ffn_q4(q4):
    """(Wg_codes, Wg_scales, Wu_codes, Wu_scales, Wd_codes, Wd_scales) -> (Wg, Wu, WdT) float32."""
    return dequant_q4(q4[0], q4[1]), dequant_q4(q4[2], q4[3]), dequant_down_q4(q4[4], q4[5])


def mha_decode(x, Wq, Wk, Wv, WoT, k_cache, v_cache, pos: int, mask=None, cache_is_bf16: bool = True):
    """One decode step of head-sparse attention.  k_cache / v_cache: float32 [H][max_len][dh] holding
    storage-type values; they are updated in place at position pos.  Returns y [d] float64."""
    x = _f32(x).reshape(-1)
    Wq, Wk, Wv, WoT = _f32(Wq), _f32(Wk), _f32(Wv), _f32(WoT)
    d = x.shape[0]
    assert k_cache.dtype == np.float32 and v_cache.dtype == np.float32
    assert k_cache.flags["C_CONTIGUOUS"] and v_cache.flags["C_CONTIGUOUS"] and k_cache.shape == v_cache.shape
    H, max_len, dh = k_cache.shape
    assert Wq.shape == (H * dh, d) and Wk.shape == Wq.shape and Wv.shape == Wq.shape and WoT.shape == Wq.shape
    m = None if mask is None else np.ascontiguousarray(np.asarray(mask, dtype=np.uint8).reshape(-1))
    if m is not None:
        assert m.shape == (H,)
    y = np.empty((d,), dtype=np.float64)
    rc = lib().halo_ref_mha_decode(_p(x, C.c_float), C.c_int32(d), C.c_int32(H), C.c_int32(dh),
                                   _p(Wq, C.c_float), _p(Wk, C.c_float), _p(Wv, C.c_float), _p(WoT, C.c_float),
                                   _p(k_cache, C.c_float), _p(v_cache, C.c_float), C.c_int32(max_len),
                                   C.c_int32(pos), _p(m, C.c_uint8), C.c_int32(1 if cache_is_bf16 else 0),
                                   _p(y, C.c_double))
    if rc != 0:
        raise ValueError("halo_ref_mha_decode rejected its arguments")
    return y
