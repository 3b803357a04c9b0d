"""Pins of the CPU oracle's primitives against closed forms, invariants and
library routines (numpy / scipy / torch CPU).  No GPU."""
import itertools

import numpy as np
import pytest
import scipy.special
import torch

import synth
from oracle import ee_oracle as orc

RNG = np.random.default_rng(1234)


# ---------------------------------------------------------------- bf16 rounding

def test_round_bf16_matches_torch_cpu():
    x = np.concatenate([RNG.standard_normal(5000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.001953125, 1.005859375,  # ties
                                  3.3895314e38, 1e-40, -1e-40], np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = orc.round_bf16(x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # the input generator's own rounding is the same function
    assert np.array_equal(synth.bf16_bits_to_f32(synth.to_bf16_bits(x)).view(np.uint32), want.view(np.uint32))


def test_round_bf16_ties_to_even():
    # 1 + 2^-8 lies halfway between 1 and 1 + 2^-7: goes to the even mantissa (1.0);
    # 1 + 3*2^-8 lies halfway between 1+2^-7 and 1+2^-6: goes up to the even one
    got = orc.round_bf16(np.array([1.00390625, 1.01171875], np.float32))
    assert got[0] == 1.0 and got[1] == 1.015625


# ---------------------------------------------------------------- RMSNorm

def test_rmsnorm_constant_vector_closed_form():
    d, c, eps = 64, 3.0, 1e-5
    g = RNG.standard_normal(d).astype(np.float32)
    out = orc.rmsnorm(np.full(d, c, np.float32), g, eps)
    want = c / np.sqrt(c * c + eps) * g.astype(np.float64)
    np.testing.assert_allclose(out, want, rtol=3e-7)


def test_rmsnorm_matches_definition_fp64_and_scale_invariance():
    d = 200
    h = RNG.standard_normal(d).astype(np.float32) * 5
    g = (1 + 0.1 * RNG.standard_normal(d)).astype(np.float32)
    out = orc.rmsnorm(h, g, 1e-5)
    h64 = h.astype(np.float64)
    want = h64 / np.sqrt(np.mean(h64 ** 2) + 1e-5) * g
    np.testing.assert_allclose(out, want, rtol=5e-7)
    # with eps -> 0 the output does not change when h is multiplied by a constant
    out2 = orc.rmsnorm(h * 4, g, 0.0)
    out1 = orc.rmsnorm(h, g, 0.0)
    np.testing.assert_allclose(out2, out1, rtol=5e-7)
    # unit gain => unit RMS
    o = orc.rmsnorm(h, np.ones(d, np.float32), 0.0)
    assert abs(np.sqrt(np.mean(o.astype(np.float64) ** 2)) - 1) < 1e-6


def test_rmsnorm_bf16_rounding_point():
    d = 96
    h = RNG.standard_normal(d).astype(np.float32)
    g = np.ones(d, np.float32)
    plain = orc.rmsnorm(h, g, 1e-5, round_to_bf16=False)
    rounded = orc.rmsnorm(h, g, 1e-5, round_to_bf16=True)
    assert np.array_equal(rounded, torch.from_numpy(plain).to(torch.bfloat16).float().numpy())


# ---------------------------------------------------------------- matvec

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_matvec_vs_numpy_fp64(dtype):
    N, K = 37, 129
    W = synth.normal(3, "W", (N, K), 0.5, dtype)
    x = RNG.standard_normal(K).astype(np.float32)
    W64 = synth.bf16_bits_to_f32(W).astype(np.float64) if dtype == "bf16" else W.astype(np.float64)
    want = W64 @ x.astype(np.float64)
    got = orc.matvec(x, W)
    np.testing.assert_allclose(got, want, rtol=2e-7, atol=1e-7)
    # a transposed operand or a dropped term would not survive this:
    e = np.zeros(K, np.float32); e[5] = 1
    np.testing.assert_array_equal(orc.matvec(e, W), W64[:, 5].astype(np.float32))


# ---------------------------------------------------------------- rotary embedding

def test_rope_position_zero_is_identity():
    v = RNG.standard_normal(16).astype(np.float32)
    assert np.array_equal(orc.rope(v, 0), v)


def test_rope_preserves_pair_norms_and_first_pair_angle():
    hd = 16
    v = RNG.standard_normal(hd).astype(np.float32)
    r = orc.rope(v, 7)
    half = hd // 2
    for i in range(half):
        assert abs(np.hypot(r[i], r[i + half]) - np.hypot(v[i], v[i + half])) < 1e-6
    # pair 0 has frequency theta^0 = 1: rotation by exactly `pos` radians
    z = complex(v[0], v[half]) * np.exp(1j * 7.0)
    assert abs(r[0] - z.real) < 1e-6 and abs(r[half] - z.imag) < 1e-6
    # last pair: angle pos * theta^(-(hd-2)/hd)
    i = half - 1
    z = complex(v[i], v[i + half]) * np.exp(1j * 7.0 * 10000.0 ** (-2.0 * i / hd))
    assert abs(r[i] - z.real) < 1e-6 and abs(r[i + half] - z.imag) < 1e-6


def test_rope_inner_product_depends_on_relative_position_only():
    hd = 32
    q = RNG.standard_normal(hd).astype(np.float32)
    k = RNG.standard_normal(hd).astype(np.float32)
    a = np.dot(orc.rope(q, 11).astype(np.float64), orc.rope(k, 5))
    b = np.dot(orc.rope(q, 106).astype(np.float64), orc.rope(k, 100))
    c = np.dot(orc.rope(q, 6).astype(np.float64), orc.rope(k, 0))
    assert abs(a - b) < 1e-4 and abs(a - c) < 1e-4
    d = np.dot(orc.rope(q, 12).astype(np.float64), orc.rope(k, 5))
    assert abs(a - d) > 1e-3  # and it does depend on the offset


# ---------------------------------------------------------------- attention

def test_attention_single_position_returns_v():
    hd = 16
    q = RNG.standard_normal(hd).astype(np.float32)
    K = RNG.standard_normal((1, hd)).astype(np.float32)
    V = RNG.standard_normal((1, hd)).astype(np.float32)
    assert np.array_equal(orc.attention_head(q, K, V), V[0])


def test_attention_identical_keys_returns_mean_v():
    hd, n = 8, 13
    q = RNG.standard_normal(hd).astype(np.float32)
    K = np.tile(RNG.standard_normal((1, hd)).astype(np.float32), (n, 1))
    V = RNG.standard_normal((n, hd)).astype(np.float32)
    np.testing.assert_allclose(orc.attention_head(q, K, V), V.astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)


def test_attention_vs_scipy_softmax():
    hd, n = 64, 300
    q = RNG.standard_normal(hd).astype(np.float32)
    K = RNG.standard_normal((n, hd)).astype(np.float32)
    V = RNG.standard_normal((n, hd)).astype(np.float32)
    p = scipy.special.softmax(K.astype(np.float64) @ q.astype(np.float64) / np.sqrt(hd))
    want = p @ V.astype(np.float64)
    np.testing.assert_allclose(orc.attention_head(q, K, V), want, rtol=2e-5, atol=2e-6)
    # one dominant key => its value
    K2 = K.copy(); K2[17] = q * 50
    np.testing.assert_allclose(orc.attention_head(q, K2, V), V[17], rtol=1e-6, atol=1e-6)


# ---------------------------------------------------------------- silu

def test_silu_values():
    assert orc.silu(0.0) == 0.0
    for t in [-20.0, -3.0, -0.5, 0.7, 4.0, 30.0]:
        assert abs(orc.silu(t) - t * scipy.special.expit(t)) <= 1e-6 * max(1.0, abs(t))
    assert orc.silu(80.0) == 80.0  # saturates to identity, no overflow


# ---------------------------------------------------------------- confidence (Sec. 2.1: the
# exit decision compares a probability with the threshold)

def test_conf_uniform_logits():
    V = 512
    conf, tok = orc.softmax_conf(np.full(V, 3.25, np.float32))
    assert tok == 0 and abs(conf - 1.0 / V) < 1e-9


def test_conf_two_logits_logistic_closed_form():
    for delta in [0.0, 0.3, 2.0, 9.0]:
        conf, tok = orc.softmax_conf(np.array([1.0, 1.0 + delta], np.float32))
        assert abs(conf - 1 / (1 + np.exp(-delta))) < 1e-7
        assert tok == (1 if delta > 0 else 0)


def test_conf_is_max_softmax_probability_and_in_range():
    for V, s in [(7, 1.0), (2048, 0.5), (2048, 50.0), (32000, 10.0)]:
        z = (RNG.standard_normal(V) * s).astype(np.float32)
        conf, tok = orc.softmax_conf(z)
        p = scipy.special.softmax(z.astype(np.float64))
        assert tok == int(np.argmax(z))
        assert abs(conf - p.max()) <= 1e-6 * p.max()
        assert 1.0 / V <= conf <= 1.0


def test_conf_tie_takes_lowest_index_and_huge_logits_do_not_overflow():
    z = np.array([1.0, 7.0, 3.0, 7.0, 7.0], np.float32)
    conf, tok = orc.softmax_conf(z)
    assert tok == 1 and abs(conf - scipy.special.softmax(z.astype(np.float64)).max()) < 1e-7
    conf, tok = orc.softmax_conf(np.array([-1e30, 1e30, 0.0], np.float32))
    assert tok == 1 and conf == 1.0


# ---------------------------------------------------------------- compaction

def test_compact_exhaustive_small():
    for n in range(0, 11):
        active = np.arange(100, 100 + 3 * n, 3, dtype=np.int32)
        for bits in itertools.product([0, 1], repeat=n):
            keep, gone = orc.compact(np.array(bits, np.uint8), active)
            want_keep = [a for a, m in zip(active, bits) if not m]
            want_gone = [a for a, m in zip(active, bits) if m]
            assert keep.tolist() == want_keep and gone.tolist() == want_gone


def test_compact_order_and_count_random():
    n = 500
    active = np.sort(RNG.choice(5000, n, replace=False)).astype(np.int32)
    mask = (RNG.random(n) < 0.4).astype(np.uint8)
    keep, gone = orc.compact(mask, active)
    assert keep.size + gone.size == n
    assert np.all(np.diff(keep) > 0) and np.all(np.diff(gone) > 0)
    assert np.array_equal(keep, active[mask == 0]) and np.array_equal(gone, active[mask == 1])
