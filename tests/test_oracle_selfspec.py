"""Pins of the oracle's self-speculative decoding round (Sec. 6: an early-exit model with an
intermediate exit below its loaded depth can be served by exit-layer speculative decoding).  What the
scheme reaches has a plain definition, full-depth greedy decoding, so the pins are: the acceptance
rule on hand-made sequences and by brute force, token streams and caches equal to the separately
written full-depth step bit for bit for every draft length and draft exit, and the two special cases
in which the drafter is always right and always wrong.  No GPU."""
import itertools

import numpy as np
import pytest

import synth
from oracle import ee_oracle as orc
from helpers import OracleSide, small_shape


def test_acceptance_rule_on_hand_made_sequences():
    A = orc.accept_drafts
    assert A([5, 6, 7], [5, 6, 7]).tolist() == [5, 6, 7]        # all agree: k tokens, no extra one
    assert A([5, 6, 7], [5, 9, 7]).tolist() == [5, 9]           # first disagreement is replaced, the rest dropped
    assert A([5, 6, 7], [4, 6, 7]).tolist() == [4]              # nothing accepted: one token, as in plain decoding
    assert A([5, 6, 7], [5, 6, 8]).tolist() == [5, 6, 8]        # last draft wrong: still k tokens, the last corrected
    assert A([3], [3]).tolist() == [3] and A([3], [4]).tolist() == [4]


def test_acceptance_rule_brute_force():
    """every pair of sequences over a 2-symbol alphabet up to length 5, against the rule restated:
    emit the verified tokens up to and including the first disagreement, at most k of them"""
    for k in range(1, 6):
        for d in itertools.product((0, 1), repeat=k):
            for v in itertools.product((0, 1), repeat=k):
                want = []
                for j in range(k):
                    want.append(v[j])
                    if d[j] != v[j]:
                        break
                got = orc.accept_drafts(d, v).tolist()
                assert got == want, (d, v, got, want)
                assert 1 <= len(got) <= k


def _shape(**kw):
    base = dict(n_layers=5, exit_layers=(1, 3, 5), resident=5, thresholds=(2.0, 2.0, 2.0), batch=3, ctx_lo=2, ctx_hi=6, steps=12)
    base.update(kw)
    return small_shape(**base)


def _vanilla_stream(s, W, n_tokens):
    o = OracleSide(s, weights=W, gain_jitter=0, cap=64)
    toks = []
    for _ in range(n_tokens):
        r = orc.vanilla_step(o.model, o.kv, o.tok, o.pos, None)
        assert r["rc"] == 0
        o.tok = r["tok"].copy()
        toks.append(r["tok"].copy())
    return np.stack(toks, 1), o          # [B][n_tokens]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("draft_exit,k", [(0, 1), (0, 3), (1, 2), (1, 4), (0, 5)])
def test_rounds_reproduce_full_depth_greedy_decoding_bit_for_bit(dtype, draft_exit, k):
    s = _shape(dtype=dtype)
    ref = OracleSide(s, gain_jitter=0.1, cap=64)
    W = ref.weights
    n_tokens = 12
    want, ov = _vanilla_stream(s, W, n_tokens + k)
    o = OracleSide(s, weights=W, gain_jitter=0, cap=64)
    for b in range(s.batch):
        got, tok, pos = [], int(o.tok[b]), int(o.pos[b])
        p0 = pos
        while len(got) < n_tokens:
            r = orc.selfspec_round(o.model, o.kv, b, tok, pos, draft_exit, k)
            assert r["rc"] == 0
            assert 1 <= r["emitted"].size <= k and r["pos"] == pos + r["emitted"].size
            # the full-depth tokens of the accepted prefix are the drafts themselves
            a = r["emitted"].size
            assert np.array_equal(r["drafts"][:a - 1], r["emitted"][:a - 1])
            got.extend(r["emitted"].tolist())
            tok, pos = int(r["emitted"][-1]), r["pos"]
        assert got[:n_tokens] == want[b, :n_tokens].tolist(), (b, got, want[b])
        # every layer's cache below the new position is the full-depth one, bit for bit
        n = min(pos, p0 + n_tokens)
        assert np.array_equal(o.kv.K[:, b, :, :n], ov.kv.K[:, b, :, :n])
        assert np.array_equal(o.kv.V[:, b, :, :n], ov.kv.V[:, b, :, :n])


def _identity_tail(W, s, Le, same_head):
    """layers above Le leave the hidden state unchanged; the head at R is the drafter's (or its negation)"""
    W = {"layers": {l: dict(w) for l, w in W["layers"].items()}, "exits": {e: dict(w) for e, w in W["exits"].items()},
         "embed": W["embed"]}
    for l in range(Le + 1, s.resident + 1):
        W["layers"][l]["W_o"] = np.zeros_like(W["layers"][l]["W_o"])
        W["layers"][l]["W_down"] = np.zeros_like(W["layers"][l]["W_down"])
    e_draft = s.exit_layers.index(Le)
    e_last = s.exit_layers.index(s.resident)
    W["exits"][e_last]["g"] = W["exits"][e_draft]["g"].copy()
    Wd = W["exits"][e_draft]["W"]
    W["exits"][e_last]["W"] = Wd.copy() if same_head else (-Wd if Wd.dtype != np.uint16 else (Wd ^ np.uint16(0x8000)))
    return W


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_a_drafter_that_is_always_right_gets_every_draft_accepted(dtype):
    s = _shape(dtype=dtype)
    W = _identity_tail(OracleSide(s, gain_jitter=0.1, cap=64).weights, s, 3, same_head=True)
    o = OracleSide(s, weights=W, gain_jitter=0, cap=64)
    k = 4
    for b in range(s.batch):
        tok, pos = int(o.tok[b]), int(o.pos[b])
        for _ in range(3):
            r = orc.selfspec_round(o.model, o.kv, b, tok, pos, 1, k)
            assert r["rc"] == 0 and np.array_equal(r["drafts"], r["verified"])
            assert r["emitted"].tolist() == r["drafts"].tolist() and r["pos"] == pos + k
            tok, pos = int(r["emitted"][-1]), r["pos"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_a_drafter_that_is_always_wrong_degrades_to_one_token_per_round(dtype):
    """the head at R is the negated draft head on the same state: its argmax is the drafter's argmin"""
    s = _shape(dtype=dtype)
    W = _identity_tail(OracleSide(s, gain_jitter=0.1, cap=64).weights, s, 3, same_head=False)
    o = OracleSide(s, weights=W, gain_jitter=0, cap=64)
    want, _ = _vanilla_stream(s, W, 4)
    for b in range(s.batch):
        tok, pos = int(o.tok[b]), int(o.pos[b])
        for t in range(4):
            r = orc.selfspec_round(o.model, o.kv, b, tok, pos, 1, 3)
            assert r["rc"] == 0 and r["drafts"][0] != r["verified"][0]
            assert r["emitted"].tolist() == [want[b, t]] and r["pos"] == pos + 1
            tok, pos = int(r["emitted"][-1]), r["pos"]


def test_round_rejects_bad_arguments():
    s = _shape()
    o = OracleSide(s, gain_jitter=0, cap=16)
    assert orc.selfspec_round(o.model, o.kv, 0, 1, 2, 2, 2)["rc"] != 0          # the drafter is the last exit itself
    assert orc.selfspec_round(o.model, o.kv, 0, 1, 2, 5, 2)["rc"] != 0          # no such exit
    assert orc.selfspec_round(o.model, o.kv, 0, 1, 15, 0, 2)["rc"] != 0         # positions beyond the cache
    assert orc.selfspec_round(o.model, o.kv, 7, 1, 2, 0, 2)["rc"] != 0          # no such row
    assert orc.selfspec_round(o.model, o.kv, 0, 1, 2, 0, 0)["rc"] != 0          # no drafts
