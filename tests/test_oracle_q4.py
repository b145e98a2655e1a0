"""Pins for the oracle's view of 4-bit block-quantised weights (paper Sec. V-A: 4-bit models;
the storage format is the library's, stated in include/halo.h)."""
import os

import numpy as np
import torch
import torch.nn.functional as F

import halo_synth as hs
from oracle import ref
from tests.util import GOLDEN


def _golden_words():
    out = {}
    for line in open(os.path.join(GOLDEN, "q4_format.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            p, wd = line.split()
            out[int(p)] = int(wd, 16)
    return out


def test_every_element_position_lands_where_the_format_says():
    words = _golden_words()
    assert sorted(words) == list(range(8))
    cols = 256
    for p, wd in words.items():
        for word_index in (0, 5, 31):
            codes = np.zeros((1, cols // 8), np.uint32)
            codes[0, word_index] = wd
            scales = np.array([[0.5, 0.25]], np.float32)
            out = ref.dequant_q4(codes, scales)
            e = word_index * 8 + p
            s = scales[0, e // 128]
            want = np.full(cols, -8.0) * np.repeat(scales[0], 128)
            want[e] = s * (1 - 8)
            assert np.array_equal(out[0], want.astype(np.float32)), (p, word_index)


def test_code_eight_is_zero_and_codes_span_minus_eight_to_seven():
    codes = np.full((2, 16), 0x88888888, np.uint32)
    assert np.all(ref.dequant_q4(codes, np.ones((2, 1), np.float32)) == 0.0)
    # word with codes 0..7 at positions 0..7: low half holds even positions (0,2,4,6), high half odd
    lo = 0 | (2 << 4) | (4 << 8) | (6 << 12)
    hi = 1 | (3 << 4) | (5 << 8) | (7 << 12)
    codes = np.full((1, 16), 0x88888888, np.uint32)
    codes[0, 0] = lo | (hi << 16)
    codes[0, 1] = (lo | (hi << 16)) + 0x88888888          # codes 8..15
    out = ref.dequant_q4(codes, np.full((1, 1), 2.0, np.float32))[0]
    assert np.array_equal(out[:16], 2.0 * (np.arange(16) - 8))


def test_scale_of_the_right_block_and_row_is_used():
    rows, cols = 3, 384
    codes = np.full((rows, cols // 8), 0x99999999, np.uint32)     # every code 9 -> value = +scale
    scales = (np.arange(rows * 3, dtype=np.float32).reshape(rows, 3) + 1.0) / 16.0
    out = ref.dequant_q4(codes, scales)
    assert np.array_equal(out, np.repeat(scales, 128, axis=1))


def test_down_projection_layout_group_output_neuron():
    G, d, gs = 3, 5, 128
    words = _golden_words()
    codes = np.full((G, d, gs // 8), 0x88888888, np.uint32)
    scales = (np.arange(G * d, dtype=np.float32).reshape(G, d) + 1.0) / 8.0
    # one non-zero weight: group 2, output 3, neuron 77 = word 9, position 5, code 8 + 1
    codes[2, 3, 9] = 0x88888888 + words[5]
    out = ref.dequant_down_q4(codes, scales)
    assert out.shape == (G * gs, d)
    want = np.zeros((G * gs, d), np.float32)
    want[2 * gs + 77, 3] = scales[2, 3]
    assert np.array_equal(out, want)


def test_uniform_weights_closed_form_through_the_ffn():
    # every weight equals s: gate = up = s * sum(x); each surviving neuron adds s * SiLU(gate) * up
    G, d, gs, s = 4, 256, 128, 0.125
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, d)).astype(np.float32)
    nine = lambda shape: np.full(shape, 0x99999999, np.uint32)
    q4 = (nine((G * gs, d // 8)), np.full((G * gs, d // 128), s, np.float32),
          nine((G * gs, d // 8)), np.full((G * gs, d // 128), s, np.float32),
          nine((G, d, gs // 8)), np.full((G, d), s, np.float32))
    Wg, Wu, WdT = ref.dequant_ffn_q4(q4)
    mask = np.array([[1, 0, 1, 1], [0, 0, 1, 0]], np.uint8)
    y = ref.group_sparse_ffn(x, Wg, Wu, WdT, gs, mask)
    for t in range(2):
        z = s * x[t].astype(np.float64).sum()
        act = z / (1.0 + np.exp(-z)) * z
        np.testing.assert_allclose(y[t], np.full(d, mask[t].sum() * gs * s * act), rtol=1e-12)


def test_generated_weights_against_a_library_matmul_on_independently_unpacked_values():
    w = hs.small_variant(hs.LLAMA7B_DECODE, 256, 3, 64, T=2)
    q4 = hs.ffn_weights_q4(w)
    npq = [t.float().numpy() if t.dtype == torch.bfloat16 else t.numpy() for t in q4]

    def unpack(words):                       # numpy bit operations, positions from the golden file
        words = words.astype(np.int64) & 0xFFFFFFFF
        gold = _golden_words()
        shift = {p: int(np.log2(v)) for p, v in gold.items()}
        return np.stack([(words >> shift[p]) & 15 for p in range(8)], axis=-1).reshape(*words.shape[:-1], -1)

    Wg = (unpack(npq[0]) - 8) * np.repeat(npq[1].astype(np.float64), 128, axis=1)
    Wu = (unpack(npq[2]) - 8) * np.repeat(npq[3].astype(np.float64), 128, axis=1)
    Wd = (unpack(npq[4]) - 8) * npq[5].astype(np.float64)[:, :, None]        # [G][d][gs]
    x = hs.hidden_states(w).float().numpy().astype(np.float64)
    G, gs, d = w.n_groups, w.group_size, w.d
    a = (F.silu(torch.from_numpy(x @ Wg.T)) * torch.from_numpy(x @ Wu.T)).numpy().reshape(2, G, gs)
    mask = np.array([[1, 0, 1], [1, 1, 0]], np.uint8)
    want = np.einsum("tgm,gjm,tg->tj", a, Wd, mask.astype(np.float64))
    got = ref.group_sparse_ffn(x.astype(np.float32), *ref.dequant_ffn_q4(npq), gs, mask)
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)


def test_generator_statistics():
    w = hs.small_variant(hs.LLAMA7B_DECODE, 512, 4, 64)
    q4 = hs.ffn_weights_q4(w)
    Wg = ref.dequant_q4(q4[0].numpy(), q4[1].float().numpy())
    assert abs(float(Wg.mean())) < 2e-4 and 0.012 < float(Wg.std()) < 0.018
    s = q4[1].float().numpy()
    assert s.min() >= 2.0 ** -8 and s.max() < 2.0 ** -7
    again = hs.ffn_weights_q4(w)
    assert all(torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b) for a, b in zip(q4, again))
