"""Pins for the oracle's building blocks: closed forms, invariants and textbook special cases.

None of these re-types the oracle's formula with the same structure: each checks a value that the
mathematics fixes independently (a hand-computed number, a symmetry, a limiting case).
"""
import math
import os

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2506_03700_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---- RMSNorm ------------------------------------------------------------------------------------------

def test_rmsnorm_constant_vector_closed_form():
    # x = (c, c, ..., c): mean(x^2) = c^2, so every output is w_i * c / sqrt(c^2 + eps)
    n, c, eps = 48, -3.0, 1e-5
    w = np.linspace(0.5, 1.5, n).astype(np.float32)
    out = orc.rmsnorm(np.full(n, c), w, eps)
    np.testing.assert_allclose(out, w.astype(np.float64) * c / math.sqrt(c * c + eps), rtol=1e-14)


def test_rmsnorm_unit_rms_and_scale_invariance():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(256)
    w = np.ones(256, dtype=np.float32)
    out = orc.rmsnorm(x, w, 0.0)
    assert abs(np.mean(out ** 2) - 1.0) < 1e-13            # eps = 0: output has unit mean square
    np.testing.assert_allclose(orc.rmsnorm(7.5 * x, w, 0.0), out, rtol=1e-13)   # and ignores scale
    # eps matters: for a tiny input the eps term dominates and the output is x / sqrt(eps)
    tiny = 1e-9 * x
    np.testing.assert_allclose(orc.rmsnorm(tiny, w, 1e-5), tiny / math.sqrt(np.mean(tiny ** 2) + 1e-5), rtol=1e-13)
    assert np.max(np.abs(orc.rmsnorm(tiny, w, 1e-5))) < 1e-5


def test_rmsnorm_hand_example_and_bf16_weight():
    # x = (3, 4): mean square 12.5 -> (3, 4) / sqrt(12.5); weights (2, 0.5) stored as bf16 are exact
    w = synth.f32_to_bf16_bits(np.array([2.0, 0.5], dtype=np.float32))
    out = orc.rmsnorm(np.array([3.0, 4.0]), w, 0.0)
    np.testing.assert_allclose(out, [2 * 3 / math.sqrt(12.5), 0.5 * 4 / math.sqrt(12.5)], rtol=1e-15)


def test_rmsnorm_is_not_layernorm():
    # a mean shift must change the result (no mean subtraction): guards against the wrong norm
    x = np.array([1.0, 2.0, 3.0, 4.0])
    w = np.ones(4, dtype=np.float32)
    a, b = orc.rmsnorm(x, w, 0.0), orc.rmsnorm(x + 10.0, w, 0.0)
    assert np.max(np.abs(a - b)) > 0.1
    np.testing.assert_allclose(a, x / math.sqrt(7.5), rtol=1e-15)


# ---- rotary embedding --------------------------------------------------------------------------------

def test_rope_position_zero_is_identity():
    v = np.random.default_rng(2).standard_normal(64)
    np.testing.assert_array_equal(orc.rope(v, 0, 10000.0), v)


def test_rope_two_dims_is_plain_rotation():
    # head_dim 2: one pair (0, 1), frequency base^0 = 1, so position p rotates by p radians
    for p in (1, 2, 7):
        out = orc.rope(np.array([1.0, 0.0]), p, 10000.0)
        np.testing.assert_allclose(out, [math.cos(p), math.sin(p)], atol=1e-15)
        out = orc.rope(np.array([0.0, 1.0]), p, 10000.0)
        np.testing.assert_allclose(out, [-math.sin(p), math.cos(p)], atol=1e-15)


def test_rope_pairs_halves_with_geometric_frequencies():
    # head_dim 8, base 16: frequencies 16^(-2i/8) = 1, 1/2, 1/4, 1/8 for pairs (i, i+4)
    dh, base, pos = 8, 16.0, 5
    for i, freq in enumerate([1.0, 0.5, 0.25, 0.125]):
        e = np.zeros(dh)
        e[i] = 1.0
        out = orc.rope(e, pos, base)
        want = np.zeros(dh)
        want[i], want[i + 4] = math.cos(pos * freq), math.sin(pos * freq)
        np.testing.assert_allclose(out, want, atol=1e-15)


def test_rope_preserves_norm_and_relative_position():
    rng = np.random.default_rng(3)
    q, k = rng.standard_normal(128), rng.standard_normal(128)
    base = 500000.0
    assert abs(np.linalg.norm(orc.rope(q, 4097, base)) - np.linalg.norm(q)) < 1e-12
    # <rope(q, p), rope(k, p')> depends on p - p' only
    a = orc.rope(q, 100, base) @ orc.rope(k, 93, base)
    b = orc.rope(q, 4100, base) @ orc.rope(k, 4093, base)
    c = orc.rope(q, 7, base) @ orc.rope(k, 0, base)
    assert abs(a - b) < 1e-9 and abs(a - c) < 1e-9
    # and it does change with the offset
    assert abs(a - orc.rope(q, 100, base) @ orc.rope(k, 92, base)) > 1e-3


# ---- greedy confidence (Eq. 1 at temperature 0) -----------------------------------------------------------

def test_confidence_uniform_logits():
    tok, conf, margin = orc.confidence(np.full(1000, 2.5))
    assert tok == 0 and margin == 0.0 and abs(conf - 1e-3) < 1e-15      # lowest index wins a tie


def test_confidence_one_hot_closed_form():
    # z = (0, ..., a at index 17, ..., 0): conf = e^a / (e^a + V - 1), margin a
    V, a = 2048, 5.12
    z = np.zeros(V)
    z[17] = a
    tok, conf, margin = orc.confidence(z)
    assert tok == 17 and abs(margin - a) < 1e-15
    assert abs(conf - math.exp(a) / (math.exp(a) + V - 1)) < 1e-13


def test_confidence_shift_invariant_and_bounded():
    rng = np.random.default_rng(4)
    z = rng.standard_normal(500) * 3
    t0, c0, m0 = orc.confidence(z)
    t1, c1, m1 = orc.confidence(z + 1000.0)          # must not overflow: exp of (z - max)
    assert t0 == t1 == int(np.argmax(z)) and abs(c0 - c1) < 1e-12 and abs(m0 - m1) < 1e-9
    assert 1.0 / 500 <= c0 <= 1.0
    s = np.sort(z)
    assert abs(m0 - (s[-1] - s[-2])) < 1e-12
    # against the textbook softmax written with log-sum-exp from scipy
    from scipy.special import logsumexp
    assert abs(c0 - math.exp(z.max() - logsumexp(z))) < 1e-12


def test_confidence_tie_between_later_indices():
    z = np.array([0.0, 3.0, 1.0, 3.0, 3.0])
    tok, conf, margin = orc.confidence(z)
    assert tok == 1 and margin == 0.0
    assert abs(conf - 1.0 / (3 + math.exp(-3) + math.exp(-2))) < 1e-15


# ---- numbers the paper prints ------------------------------------------------------------------------------

def _paper_values():
    out = {}
    with open(os.path.join(GOLDEN, "paper_values.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out[line[0]] = [float(x) for x in line[1:]]
    return out


def test_shapes_match_paper_tables():
    pv = _paper_values()
    s8, s13 = synth.LLAMA8B, synth.LLAMA13B
    assert [s8.vocab, s8.d_model] == pv["lm_head_rows_llama31_8b"] + pv["lm_head_cols_llama31_8b"]
    assert [s13.vocab, s13.d_model] == pv["lm_head_rows_codellama_13b"] + pv["lm_head_cols_codellama_13b"]
    assert list(s8.exit_layers) == pv["exit_layers_8b"] and s8.n_layers == pv["final_layer_8b"][0]
    # Sec. 2.1: a d x d transform has 16M parameters, a full |V| x d head 0.5B, ratio about 31
    assert int(s8.d_model ** 2 / 1e6) == pv["light_head_params_millions"][0]     # 16.78M, printed as 16M
    assert round(s8.vocab * s8.d_model / 1e9, 1) == pv["full_head_params_billions"][0]
    assert int(s8.vocab * s8.d_model / s8.d_model ** 2) == pv["head_param_ratio"][0]


def test_bf16_rounding_helper():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3], dtype=np.float32)
    b = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))
    # ties go to even: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6
    np.testing.assert_array_equal(b[:4], np.array([1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6], dtype=np.float32))
    assert abs(b[4] + 0.3) < 0.3 * 2 ** -8


def test_fp16_weights_are_read_exactly():
    # every kind of half-precision value (zero, subnormals, the smallest normal, the largest finite value, both
    # signs) must come out of the oracle as numpy's own exact widening: x = ones has rms 1, so rmsnorm returns w
    rng = np.random.default_rng(0)
    w = (rng.standard_normal(2048) * 3).astype(np.float16)
    w[:10] = np.array([0.0, -0.0, 6e-8, -6e-8, 5.96e-8, 6.1e-5, 6.104e-5, 65504, -65504, 1e-7], dtype=np.float16)
    out = orc.rmsnorm(np.ones(w.size), w, 0.0)
    np.testing.assert_array_equal(out, w.astype(np.float64))


def test_fp16_storage_helper_rounds_to_nearest_even():
    # 1 + 2^-11 is a tie between 1 and 1 + 2^-10 -> 1 (even); 1 + 3*2^-11 is a tie -> 1 + 2^-9
    x = np.array([1.0 + 2 ** -11, 1.0 + 3 * 2 ** -11, 1.0 + 2 ** -10, 2.0 ** -25, 3 * 2.0 ** -25], dtype=np.float32)
    h = synth.as_f32(synth.store_as(x, synth.F16))
    np.testing.assert_array_equal(h, np.array([1.0, 1.0 + 2 ** -9, 1.0 + 2 ** -10, 0.0, 2.0 ** -23], dtype=np.float32))
