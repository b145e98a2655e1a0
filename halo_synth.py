"""Seeded synthetic inputs for the HALO group-sparse FFN path.

This module only manufactures inputs (weights, hidden states, packet-loss
outcomes, workload shapes).  It contains none of the method's arithmetic:
no predictor, ranking, scheduling or FFN step lives here.  Both the CPU
oracle's tests and the HIP path's tests / benchmark draw their inputs from
these functions, so that the two sides see bit-identical data.

Generator.  Every tensor element is a pure function of
(seed, tensor id, layer, step, flat index):

    k  = fold(seed, tensor id, layer, step)        (splitmix64 finaliser chain)
    u  = splitmix64_finaliser(k + (index+1) * 0x9E3779B97F4A7C15)
    z  = Z[u >> 48]          Z = 65536 standard-normal quantiles at (i+1/2)/65536
    v  = round_to_dtype(float32(sigma) * z)

Only 64-bit integer operations and one table lookup are involved, so the
same torch code gives the same bits on the CPU and on the GPU (which lets
the 113 GB LLaMA-2-70B-shape stack be produced directly in HBM and
re-produced one layer at a time on the host).  Uniform variates for the
packet-loss outcomes are (u >> 11) * 2**-53.

The workloads stand in for what the paper ran (GSM8K-derived 128+128 token
requests on 4-bit LLaMA models, section V-A): same FFN shapes, random
weights N(0, 0.02), hidden states N(0, 1).
"""
from __future__ import annotations

import dataclasses
import functools
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

# tensor ids (stream selectors)
TID_X = 1
TID_WG = 2
TID_WU = 3
TID_WDT = 4
TID_AT = 5
TID_BT = 6
TID_DROP = 7
TID_PLR = 8
TID_MISC = 9
TID_WQ = 10
TID_WK = 11
TID_WV = 12
TID_WOT = 13
TID_KCACHE = 14
TID_VCACHE = 15
TID_Q4_CODES = 16     # + 0 gate, 1 up, 2 down
TID_Q4_SCALES = 24    # + 0 gate, 1 up, 2 down


def _mix_py(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, tensor_id: int, layer: int = 0, step: int = 0) -> int:
    k = _mix_py(seed + _GAMMA)
    k = _mix_py(k ^ (tensor_id & _M64))
    k = _mix_py(k ^ (layer & _M64))
    k = _mix_py(k ^ (step & _M64))
    return k


def _s64(v: int) -> int:
    """Two's-complement reinterpretation of an unsigned 64-bit value."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right on int64 tensors."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def raw_u64(key: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """u for flat indices start .. start+count-1, as int64 bit patterns."""
    idx = torch.arange(start + 1, start + count + 1, dtype=torch.int64, device=device)
    z = idx * _s64(_GAMMA) + _s64(key)
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


@functools.lru_cache(maxsize=1)
def _quantile_table_np() -> np.ndarray:
    from scipy.special import ndtri

    p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return ndtri(p).astype(np.float32)


_table_cache = {}


def quantile_table(device="cpu") -> torch.Tensor:
    dev = torch.device(device)
    key = (dev.type, dev.index)
    if key not in _table_cache:
        _table_cache[key] = torch.from_numpy(_quantile_table_np().copy()).to(dev)
    return _table_cache[key]


def normal(shape: Sequence[int], sigma: float, dtype: torch.dtype, key: int,
           device="cpu", chunk: int = 1 << 25) -> torch.Tensor:
    """Tensor of N(0, sigma^2) values (quantised to 65536 quantiles), rounded to dtype."""
    n = int(np.prod(shape)) if len(shape) else 1
    out = torch.empty(n, dtype=dtype, device=device)
    tab = quantile_table(device)
    sig = torch.tensor(float(sigma), dtype=torch.float32, device=device)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        u = raw_u64(key, s, c, device)
        z = tab[_lsr(u, 48)]
        out[s:s + c] = (z * sig).to(dtype)
    return out.reshape(tuple(shape))


def uniform01(count: int, key: int, start: int = 0) -> np.ndarray:
    """float64 uniforms in [0,1) on the host."""
    u = raw_u64(key, start, count, "cpu")
    return (_lsr(u, 11).numpy().astype(np.float64)) * (2.0 ** -53)


# --------------------------------------------------------------------------
# Workloads
# --------------------------------------------------------------------------

@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    d: int
    ffn: int
    group_size: int
    rank: int
    T: int
    layers: int
    dtype: str                 # "f32" | "bf16"
    keep: Tuple[float, ...]
    n_dev: int
    plr: Optional[Tuple[float, ...]]   # None: seeded uniforms in [0, plr_max]
    plr_max: float
    steps: int
    seed: int

    @property
    def n_groups(self) -> int:
        return self.ffn // self.group_size

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def k_keep(self, keep: Optional[float] = None) -> int:
        """Number of groups kept per token: nearest integer to keep*G, at least 1.
        (A harness-side conversion; the library's interface takes the integer.)"""
        keep = self.keep[0] if keep is None else keep
        from fractions import Fraction
        import math
        q = Fraction(str(keep)) * self.n_groups + Fraction(1, 2)   # exact decimal arithmetic
        return max(1, min(self.n_groups, math.floor(q)))

    def device_plr(self) -> np.ndarray:
        if self.plr is not None:
            return np.asarray(self.plr, dtype=np.float64)
        return uniform01(self.n_dev, stream_key(self.seed, TID_PLR)) * self.plr_max


TINY = Workload("tiny", 256, 1024, 128, 64, 16, 1, "f32", (0.5,), 4,
                (0.0, 0.0, 0.1, 0.3), 0.0, 1, 0)
LLAMA7B_DECODE = Workload("llama7b_decode", 4096, 11008, 128, 256, 1, 1, "bf16", (0.5,), 4,
                          (0.0, 0.05, 0.1, 0.2), 0.0, 1024, 1)
LLAMA13B_STACK = Workload("llama13b_stack", 5120, 13824, 128, 256, 4, 40, "bf16",
                          (0.3, 0.5, 0.7), 6, None, 0.3, 1, 2)
LLAMA7B_PREFILL = Workload("llama7b_prefill", 4096, 11008, 128, 256, 512, 1, "bf16", (0.5,), 4,
                           (0.0, 0.05, 0.1, 0.2), 0.0, 1, 3)
LLAMA70B_STACK = Workload("llama70b_stack", 8192, 28672, 128, 512, 8, 80, "bf16", (0.5,), 8,
                          (0.0, 0.0, 0.05, 0.05, 0.1, 0.1, 0.2, 0.3), 0.0, 1, 4)

WORKLOADS = [TINY, LLAMA7B_DECODE, LLAMA13B_STACK, LLAMA7B_PREFILL, LLAMA70B_STACK]
BY_NAME = {w.name: w for w in WORKLOADS}


def small_variant(w: Workload, d: int, n_groups: int, rank: int, T: Optional[int] = None,
                  layers: Optional[int] = None) -> Workload:
    """Same structure as w at a reduced shape (for parity cases the oracle finishes fast)."""
    return dataclasses.replace(w, name=w.name + "_small", d=d, ffn=n_groups * w.group_size,
                               rank=rank, T=w.T if T is None else T,
                               layers=w.layers if layers is None else layers)


# --------------------------------------------------------------------------
# Tensors of one layer
# --------------------------------------------------------------------------

W_SIGMA = 0.02
X_SIGMA = 1.0


def ffn_weights(w: Workload, layer: int = 0, device="cpu", copy: int = 0):
    """(Wg, Wu, WdT), each [ffn][d] in the workload dtype.  Row m of each belongs to
    neuron m; WdT is the down projection stored neuron-major (transposed).
    `copy` selects an independent replica of the same shape (benchmark rotation)."""
    dt = w.torch_dtype
    lay = layer + 1000003 * copy
    mk = lambda tid: normal((w.ffn, w.d), W_SIGMA, dt, stream_key(w.seed, tid, lay), device)
    return mk(TID_WG), mk(TID_WU), mk(TID_WDT)


# --------------------------------------------------------------------------
# 4-bit block-quantised weights (the paper's models are 4-bit, section V-A)
# --------------------------------------------------------------------------
# Storage format (the library's, restated here because the generator writes it directly):
# blocks of Q4_BLOCK consecutive elements along the reduction dimension share one bf16
# scale s; an element is s * (c - 8) with a 4-bit code c.  Eight codes per 32-bit word:
# element 2i of the word's eight sits in bits [4i, 4i+3], element 2i+1 in bits
# [16+4i, 16+4i+3] (i = 0..3).
# Values: the code is a fixed function of 16 hashed bits (a bell shape centred on 8,
# like rounded normal weights), the scale is 2^-8 * (1 + k/128) with 7 hashed bits k, so
# element values have a standard deviation of about 0.015 and only integer operations and a
# table lookup are involved (bit-identical on CPU and GPU).

Q4_BLOCK = 128


@functools.lru_cache(maxsize=1)
def _q4_code_table_np() -> np.ndarray:
    z = _quantile_table_np().astype(np.float64)
    return np.clip(np.floor(z * 2.5 + 8.5), 0, 15).astype(np.uint8)


_code_table_cache = {}


def _q4_code_table(device="cpu") -> torch.Tensor:
    dev = torch.device(device)
    key = (dev.type, dev.index)
    if key not in _code_table_cache:
        _code_table_cache[key] = torch.from_numpy(_q4_code_table_np().copy()).to(dev)
    return _code_table_cache[key]


def q4_codes(n_elements: int, key: int, device="cpu", chunk: int = 1 << 25) -> torch.Tensor:
    """n_elements/8 int32 words holding the packed 4-bit codes of elements 0..n_elements-1."""
    assert n_elements % 8 == 0 and chunk % 8 == 0
    out = torch.empty(n_elements // 8, dtype=torch.int32, device=device)
    tab = _q4_code_table(device)
    shifts = torch.tensor([0, 16, 4, 20, 8, 24, 12, 28], dtype=torch.int64, device=device)
    for s in range(0, n_elements, chunk):
        c = min(chunk, n_elements - s)
        code = tab[_lsr(raw_u64(key, s, c, device), 48)].to(torch.int64).reshape(-1, 8)
        word = (code << shifts).sum(dim=1)                       # disjoint bit fields: sum == or
        word = torch.where(word >= (1 << 31), word - (1 << 32), word)
        out[s // 8:(s + c) // 8] = word.to(torch.int32)
    return out


def q4_scales(n_blocks: int, key: int, device="cpu") -> torch.Tensor:
    """n_blocks bf16 scales in [2^-8, 2^-7)."""
    k = _lsr(raw_u64(key, 0, n_blocks, device), 48) & 0x7F
    return (k + 0x3B80).to(torch.int16).view(torch.bfloat16)


def ffn_weights_q4(w: Workload, layer: int = 0, device="cpu", copy: int = 0):
    """4-bit FFN weights of one layer, as the library stores them:
    (Wg_codes int32 [ffn][d/8], Wg_scales bf16 [ffn][d/128], the same two for Wu,
     Wd_codes int32 [G][d][gs/8], Wd_scales bf16 [G][d]).
    Gate/up blocks run along d; the down projection is group-blocked and the block of
    output j in group g is the group's gs = 128 neurons."""
    assert w.d % Q4_BLOCK == 0 and w.group_size == Q4_BLOCK
    lay = layer + 1000003 * copy
    G, gs, d = w.n_groups, w.group_size, w.d
    out = []
    for i in range(2):
        out.append(q4_codes(w.ffn * d, stream_key(w.seed, TID_Q4_CODES + i, lay), device).reshape(w.ffn, d // 8))
        out.append(q4_scales(w.ffn * (d // Q4_BLOCK), stream_key(w.seed, TID_Q4_SCALES + i, lay),
                             device).reshape(w.ffn, d // Q4_BLOCK))
    out.append(q4_codes(G * d * gs, stream_key(w.seed, TID_Q4_CODES + 2, lay), device).reshape(G, d, gs // 8))
    out.append(q4_scales(G * d, stream_key(w.seed, TID_Q4_SCALES + 2, lay), device).reshape(G, d))
    return tuple(out)


# --------------------------------------------------------------------------
# Attention block (one head + its output-projection slice = one neuron group, section II-A)
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class MhaWorkload:
    name: str
    d: int
    n_heads: int
    head_dim: int
    rank: int
    ctx: int                   # positions already in the KV cache when the timed step runs
    max_len: int
    dtype: str
    keep: float
    n_dev: int
    plr: Tuple[float, ...]
    seed: int

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def k_keep(self, keep: Optional[float] = None) -> int:
        from fractions import Fraction
        import math
        keep = self.keep if keep is None else keep
        return max(1, min(self.n_heads, math.floor(Fraction(str(keep)) * self.n_heads + Fraction(1, 2))))

    def device_plr(self) -> np.ndarray:
        return np.asarray(self.plr, dtype=np.float64)


# LLaMA-7B attention shape: 32 heads of 128, 2048 cached positions, half the heads kept
LLAMA7B_MHA_DECODE = MhaWorkload("llama7b_mha_decode", 4096, 32, 128, 256, 2048, 2304, "bf16", 0.5, 4,
                                 (0.0, 0.05, 0.1, 0.2), 5)
MHA_BY_NAME = {LLAMA7B_MHA_DECODE.name: LLAMA7B_MHA_DECODE}


def mha_weights(w: MhaWorkload, layer: int = 0, device="cpu", copy: int = 0):
    """(Wq, Wk, Wv, WoT), each [n_heads*head_dim][d]; rows h*head_dim.. belong to head h; WoT is the
    output projection stored head-dimension-major (row n = the weights leaving dimension n)."""
    lay = layer + 1000003 * copy
    hd = w.n_heads * w.head_dim
    mk = lambda tid: normal((hd, w.d), W_SIGMA, w.torch_dtype, stream_key(w.seed, tid, lay), device)
    return mk(TID_WQ), mk(TID_WK), mk(TID_WV), mk(TID_WOT)


def mha_predictor_weights(w: MhaWorkload, layer: int = 0, device="cpu", copy: int = 0):
    lay = layer + 1000003 * copy
    At = normal((w.rank, w.d), W_SIGMA, w.torch_dtype, stream_key(w.seed, TID_AT, lay), device)
    Bt = normal((w.n_heads, w.rank), W_SIGMA, w.torch_dtype, stream_key(w.seed, TID_BT, lay), device)
    return At, Bt


def kv_cache(w: MhaWorkload, layer: int = 0, device="cpu", copy: int = 0):
    """(k_cache, v_cache), each [n_heads][max_len][head_dim] ~ N(0,1) in the workload dtype: stands in
    for the keys / values of the positions decoded so far (all max_len rows are filled; a step at
    position pos reads rows 0..pos-1 and writes row pos)."""
    lay = layer + 1000003 * copy
    shape = (w.n_heads, w.max_len, w.head_dim)
    return (normal(shape, 1.0, w.torch_dtype, stream_key(w.seed, TID_KCACHE, lay), device),
            normal(shape, 1.0, w.torch_dtype, stream_key(w.seed, TID_VCACHE, lay), device))


def mha_hidden(w: MhaWorkload, step: int = 0, device="cpu"):
    return normal((1, w.d), X_SIGMA, w.torch_dtype, stream_key(w.seed, TID_X, 0, step), device)


def mha_drop_outcomes(w: MhaWorkload, layer: int = 0, step: int = 0) -> np.ndarray:
    u = uniform01(w.n_dev, stream_key(w.seed, TID_DROP, layer, step)).reshape(1, w.n_dev)
    return (u < w.device_plr()[None, :]).astype(np.uint8)


def predictor_weights(w: Workload, layer: int = 0, device="cpu", copy: int = 0):
    """(At [rank][d], Bt [G][rank]): the two predictor matrices, stored transposed."""
    dt = w.torch_dtype
    lay = layer + 1000003 * copy
    At = normal((w.rank, w.d), W_SIGMA, dt, stream_key(w.seed, TID_AT, lay), device)
    Bt = normal((w.n_groups, w.rank), W_SIGMA, dt, stream_key(w.seed, TID_BT, lay), device)
    return At, Bt


def hidden_states(w: Workload, step: int = 0, device="cpu", T: Optional[int] = None,
                  dtype: Optional[torch.dtype] = None):
    """x [T][d] ~ N(0,1) in the workload dtype (or `dtype`)."""
    T = w.T if T is None else T
    dt = w.torch_dtype if dtype is None else dtype
    return normal((T, w.d), X_SIGMA, dt, stream_key(w.seed, TID_X, 0, step), device)


def drop_outcomes(w: Workload, layer: int = 0, step: int = 0, T: Optional[int] = None,
                  plr: Optional[np.ndarray] = None) -> np.ndarray:
    """drop[t][dev] in {0,1}: Bernoulli(plr[dev]) per (token, layer, step, device)."""
    T = w.T if T is None else T
    plr = w.device_plr() if plr is None else np.asarray(plr, dtype=np.float64)
    u = uniform01(T * w.n_dev, stream_key(w.seed, TID_DROP, layer, step)).reshape(T, w.n_dev)
    return (u < plr[None, :]).astype(np.uint8)
