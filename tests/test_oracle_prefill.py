"""Pins of the CPU oracle's context pass (prefill, the work that bounds the time to
first token: Sec. 4.4, Appendix E.1): the dense matrix form with a causal mask in
fp64 numpy, equality with token-by-token full-depth decoding, causality, chunking
and a one-token closed form.  No GPU."""
import numpy as np
import pytest
import scipy.special

import synth
from oracle import ee_oracle as orc
from helpers import OracleSide, small_shape, f32w


def _rnd(x, bf):
    return synth.bf16_bits_to_f32(synth.to_bf16_bits(x.astype(np.float32))).astype(np.float64) if bf else x


def _side(dtype="f32", cap=24, **kw):
    s = small_shape(dtype=dtype, **kw)
    return s, OracleSide(s, std=0.3, cap=cap, fill_ctx=False)


def dense_causal_pass(s, W, tokens):
    """All positions at once, as matrices: X [n][d]; scores [n][n] with -inf above the
    diagonal; the rotary embedding as one complex multiplication per (position, pair)."""
    bf = s.dtype == "bf16"
    n, d, hd, Hq, Hkv = len(tokens), s.d_model, s.head_dim, s.n_q_heads, s.n_kv_heads
    half = hd // 2
    X = f32w(W["embed"], s.dtype)[np.asarray(tokens)]
    ang = np.exp(1j * np.arange(n)[:, None] * s.rope_theta ** (-2.0 * np.arange(half) / hd)[None, :])   # [n][half]

    def rot(T):   # T [n][heads][hd]
        z = (T[..., :half] + 1j * T[..., half:]) * ang[:, None, :]
        return np.concatenate([z.real, z.imag], axis=-1)

    mask = np.where(np.arange(n)[None, :] > np.arange(n)[:, None], -np.inf, 0.0)
    Ks, Vs = {}, {}
    for l in range(1, s.resident + 1):
        w = W["layers"][l]
        Xn = _rnd(X / np.sqrt((X * X).mean(1, keepdims=True) + s.rms_eps) * w["g_attn"], bf)
        QKV = Xn @ f32w(w["W_qkv"], s.dtype).T
        Q = rot(QKV[:, :Hq * hd].reshape(n, Hq, hd))
        K = _rnd(rot(QKV[:, Hq * hd:(Hq + Hkv) * hd].reshape(n, Hkv, hd)), bf)
        V = _rnd(QKV[:, (Hq + Hkv) * hd:].reshape(n, Hkv, hd), bf)
        Ks[l], Vs[l] = K, V
        O = np.zeros((n, Hq, hd))
        for i in range(Hq):
            g = i // (Hq // Hkv)
            P = scipy.special.softmax(Q[:, i, :] @ K[:, g, :].T / np.sqrt(hd) + mask, axis=1)
            O[:, i, :] = P @ V[:, g, :]
        X = X + _rnd(O.reshape(n, -1), bf) @ f32w(w["W_o"], s.dtype).T
        Y = _rnd(X / np.sqrt((X * X).mean(1, keepdims=True) + s.rms_eps) * w["g_ffn"], bf)
        G, U = Y @ f32w(w["W_gate"], s.dtype).T, Y @ f32w(w["W_up"], s.dtype).T
        X = X + _rnd(G * scipy.special.expit(G) * U, bf) @ f32w(w["W_down"], s.dtype).T
    return X, Ks, Vs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_matrix_form_with_causal_mask(dtype):
    s, side = _side(dtype)
    for b, n in ((0, 11), (3, 1), (4, 17)):
        tok = synth.context_tokens(s, b, n)
        rc, h = orc.prefill(side.model, side.kv, b, tok, want_h=True)
        assert rc == 0
        X, Ks, Vs = dense_causal_pass(s, side.weights, tok)
        tol = 2e-5 if dtype == "f32" else 2e-2
        np.testing.assert_allclose(h, X, rtol=0, atol=tol * np.abs(X).max())
        for l in range(1, s.resident + 1):
            ktol = (1e-5 if dtype == "f32" else 1.7e-2) * max(1.0, np.abs(Ks[l]).max())
            np.testing.assert_allclose(side.kv.K[l - 1, b, :, :n, :], Ks[l].transpose(1, 0, 2), rtol=0, atol=ktol)
            np.testing.assert_allclose(side.kv.V[l - 1, b, :, :n, :], Vs[l].transpose(1, 0, 2), rtol=0, atol=ktol)
            assert not side.kv.K[l - 1, b, :, n:, :].any()          # nothing beyond the context
    assert not side.kv.K[:, 1].any() and not side.kv.V[:, 2].any()   # other rows untouched


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_equals_token_by_token_full_depth_decoding(dtype):
    # a context pass is decoding with the tokens given instead of generated: same
    # arithmetic per (token, layer), another order of the two loops => bit for bit
    s, a = _side(dtype)
    _, v = _side(dtype)
    lens = np.array([9, 4, 13, 1, 7])
    toks = [synth.context_tokens(s, b, int(lens[b])) for b in range(s.batch)]
    hs = []
    for b in range(s.batch):
        rc, h = orc.prefill(a.model, a.kv, b, toks[b], want_h=True)
        assert rc == 0
        hs.append(h)
    # vanilla decoding runs every row each step; rows whose context is over repeat their
    # last token at a scratch position beyond it, which is cleared afterwards
    pos = np.zeros(s.batch, np.int32)
    for t in range(int(lens.max())):
        live = t < lens
        tin = np.array([toks[b][min(t, lens[b] - 1)] for b in range(s.batch)], np.int32)
        pos = np.where(live, t, lens).astype(np.int32)
        r = orc.vanilla_step(v.model, v.kv, tin, pos, None, want_h=True)
        assert r["rc"] == 0
        for b in np.nonzero(live)[0]:
            assert np.array_equal(r["h"][b], hs[b][t])
    for b in range(s.batch):
        v.kv.K[:, b, :, lens[b]:, :] = 0
        v.kv.V[:, b, :, lens[b]:, :] = 0
    assert np.array_equal(a.kv.K, v.kv.K) and np.array_equal(a.kv.V, v.kv.V)


def test_causality_and_chunking():
    s, a = _side()
    _, c = _side()
    _, p = _side()
    tok = synth.context_tokens(s, 2, 15)
    assert orc.prefill(a.model, a.kv, 2, tok)[0] == 0
    # the same context in three pieces (6 + 1 + 8) gives the same cache and hidden states
    _, h_all = orc.prefill(p.model, p.kv, 1, tok, want_h=True)
    h_parts = []
    for lo, hi in ((0, 6), (6, 7), (7, 15)):
        rc, h = orc.prefill(c.model, c.kv, 1, tok[lo:hi], pos0=lo, want_h=True)
        assert rc == 0
        h_parts.append(h)
    assert np.array_equal(np.concatenate(h_parts), h_all)
    assert np.array_equal(c.kv.K, p.kv.K) and np.array_equal(c.kv.V, p.kv.V)
    assert np.array_equal(c.kv.K[:, 1], a.kv.K[:, 2])               # and the row it sits in does not matter
    # what follows a position cannot change it: other tokens from position 9 on
    _, q = _side()
    tok2 = tok.copy()
    tok2[9:] = (tok2[9:] + 1) % s.vocab
    assert orc.prefill(q.model, q.kv, 2, tok2)[0] == 0
    assert np.array_equal(q.kv.K[:, 2, :, :9], a.kv.K[:, 2, :, :9])
    assert np.array_equal(q.kv.V[:, 2, :, :9], a.kv.V[:, 2, :, :9])
    assert not np.array_equal(q.kv.K[:, 2, :, 9:15], a.kv.K[:, 2, :, 9:15])


def test_one_token_context_closed_form():
    # position 0: the rotation is the identity and attention over one position returns its
    # value, so layer 1's K, V and the state after its attention half are plain products
    s, a = _side()
    tok = np.array([5], np.int32)
    rc, _ = orc.prefill(a.model, a.kv, 0, tok)
    assert rc == 0
    w = a.weights["layers"][1]
    e = a.weights["embed"][5].astype(np.float64)
    x = e / np.sqrt((e * e).mean() + s.rms_eps) * w["g_attn"]
    qkv = w["W_qkv"].astype(np.float64) @ x
    Hq, Hkv, hd = s.n_q_heads, s.n_kv_heads, s.head_dim
    np.testing.assert_allclose(a.kv.K[0, 0, :, 0, :].reshape(-1), qkv[Hq * hd:(Hq + Hkv) * hd], rtol=0, atol=1e-5)
    np.testing.assert_allclose(a.kv.V[0, 0, :, 0, :].reshape(-1), qkv[(Hq + Hkv) * hd:], rtol=0, atol=1e-5)


def test_rejects_bad_arguments():
    s, a = _side(cap=8)
    tok = synth.context_tokens(s, 0, 9)
    assert orc.prefill(a.model, a.kv, 0, tok)[0] == orc.ORC_ERR_ARG            # beyond the capacity
    assert orc.prefill(a.model, a.kv, 0, tok[:4], pos0=5)[0] == orc.ORC_ERR_ARG
    assert orc.prefill(a.model, a.kv, s.batch, tok[:4])[0] == orc.ORC_ERR_ARG   # no such row
    assert orc.prefill(a.model, a.kv, 0, np.array([s.vocab], np.int32))[0] != 0  # no such token
    assert orc.prefill(a.model, a.kv, 0, tok[:0])[0] == 0                       # empty context: nothing to do
    assert not a.kv.K.any()
