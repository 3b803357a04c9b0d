"""GPU parity of exit-layer self-speculative decoding (ee_draft_step, ee_verify_drafts; Sec. 6) against
the oracle's round on the same seeded inputs, through the C ABI.

Tokens are greedy choices, so the bar is bit-exact drafts, emitted tokens and positions, except where the
oracle's own choice is closer to a tie than the logits' tolerance allows (relative margin between its two
largest logits at most 2 x 2e-2 for bf16 models, 2 x 2e-4 for fp32): such a row-round is counted and the
oracle then adopts the GPU's tokens and cache entries, as in the other sampled tests.  After every round
both sides are brought to the same state in this way, so each round is compared from identical inputs.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import ee_oracle as orc
from helpers import OracleSide
from parity import GpuSide, rows_close, TOL
from paper_2504_10724_amd import capi as ee
from paper_2504_10724_amd import session as S

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


TINY = synth.CONFIGS["tiny_f32"].with_(name="tiny_f32_spec", batch=8, ctx_lo=20, ctx_hi=64, steps=16, thresholds=(2.0, 2.0))
MID = synth.CONFIGS["llama2_7b"].with_(name="mid_bf16_spec", n_layers=6, resident=6, d_model=1024, n_q_heads=8,
                                       n_kv_heads=2, d_ffn=2816, vocab=8192, exit_layers=(2, 4, 6),
                                       thresholds=(2.0, 2.0, 2.0), batch=20, ctx_lo=20, ctx_hi=200, steps=20)
# partial residency: drafts at layer 2, verification ends at layer 4 of 6; MHA; more entries than one 256-row group
PART = synth.CONFIGS["codellama_34b_r32"].with_(name="partial_bf16_spec", n_layers=6, resident=4, d_model=512,
                                                n_q_heads=4, n_kv_heads=4, d_ffn=1024, vocab=2048,
                                                exit_layers=(2, 4, 6), thresholds=(2.0, 2.0), batch=70,
                                                ctx_lo=3, ctx_hi=90, steps=20)


def _adopt(o, g, rows, p_lo, p_hi, s):
    """the oracle takes the GPU's cache entries of positions p_lo[b] .. p_hi[b]-1 for the given rows"""
    for b in rows:
        n = int(p_hi[b] - p_lo[b])
        if n <= 0:
            continue
        for l in range(1, s.resident + 1):
            K, V = g.kv.read_context(l, int(b), n, pos0=int(p_lo[b]))
            o.kv.K[l - 1, b, :, p_lo[b]:p_hi[b]] = K
            o.kv.V[l - 1, b, :, p_lo[b]:p_hi[b]] = V


def _rounds(s, draft_exit, k, n_rounds, W=None):
    o = OracleSide(s, weights=W, gain_jitter=0.0 if W is not None else 0.1)
    g = GpuSide(s, weights=o.weights)
    sp = S.Speculator(g.model, g.kv, g.batch, draft_exit, k)
    B = s.batch
    tol = 2 * TOL[s.dtype]
    f = g.batch.field
    tok = o.tok.copy()
    pos = o.pos.copy()
    stats = dict(rounds=0, near_tie=0, emitted=0, worst_kv=0.0)
    for rnd in range(n_rounds):
        sp.round()
        torch.cuda.synchronize()
        assert int(f("status").cpu()[0]) == 0 and int(sp.entries.field("status").cpu()[0]) == 0
        d_g = sp.drafts.cpu().numpy()              # [k][B]
        n_g = sp.n_emit.cpu().numpy()
        e_g = sp.emit.cpu().numpy()                # [B][k]
        pos_g, tok_g = f("pos").cpu().numpy(), f("tok_in").cpu().numpy()
        new_pos = pos.copy()
        diverged = []
        for b in range(B):
            r = orc.selfspec_round(o.model, o.kv, b, int(tok[b]), int(pos[b]), draft_exit, k)
            assert r["rc"] == 0
            stats["rounds"] += 1
            n = int(n_g[b])
            assert 1 <= n <= k and np.all(e_g[b, n:] == -1)
            assert pos_g[b] == pos[b] + n and tok_g[b] == e_g[b, n - 1]
            # the GPU's own bookkeeping: accepted drafts are the emitted tokens, the first rejected one is not
            assert np.array_equal(d_g[:n - 1, b], e_g[b, :n - 1])
            if n < k:
                assert d_g[n - 1, b] != e_g[b, n - 1]
            same = np.array_equal(d_g[:, b], r["drafts"]) and n == r["emitted"].size and np.array_equal(e_g[b, :n], r["emitted"])
            if not same:
                # only where the oracle's choice is that close to a tie, at the first place the two differ
                jd = next((j for j in range(k) if d_g[j, b] != r["drafts"][j]), k)
                jv = next((j for j in range(min(n, r["emitted"].size)) if e_g[b, j] != r["emitted"][j]), k)
                # position j's full-depth token depends on the drafts before j only, so whichever differs first explains the rest
                ok = (r["verify_margin"][jv] <= tol) if jv <= jd and jv < k else (jd < k and r["draft_margin"][jd] <= tol)
                assert ok, (f"round {rnd} row {b}: gpu drafts {d_g[:, b].tolist()} emitted {e_g[b, :n].tolist()}; oracle drafts "
                            f"{r['drafts'].tolist()} emitted {r['emitted'].tolist()}; margins {r['draft_margin'].tolist()} "
                            f"{r['verify_margin'].tolist()}")
                stats["near_tie"] += 1
                diverged.append(b)
            else:
                # new cache entries of the emitted positions, every resident layer
                for l in range(1, s.resident + 1):
                    K, V = g.kv.read_context(l, b, n, pos0=int(pos[b]))
                    wk, okk = rows_close(K.reshape(1, -1), o.kv.K[l - 1, b, :, pos[b]:pos[b] + n].reshape(1, -1), TOL[s.dtype] if s.dtype == "bf16" else 2e-5)
                    wv, okv = rows_close(V.reshape(1, -1), o.kv.V[l - 1, b, :, pos[b]:pos[b] + n].reshape(1, -1), TOL[s.dtype] if s.dtype == "bf16" else 2e-5)
                    stats["worst_kv"] = max(stats["worst_kv"], wk, wv)
                    assert okk and okv, (rnd, b, l, wk, wv)
            stats["emitted"] += n
            new_pos[b] = pos[b] + n
        # both sides go on from the GPU's state
        _adopt(o, g, range(B), pos, new_pos, s)
        pos, tok = new_pos, tok_g.copy()
    _say(f"  {stats['rounds']} row-rounds, {stats['emitted']} tokens emitted ({stats['emitted'] / stats['rounds']:.2f} per round of "
         f"{k} drafts), {stats['near_tie']} row-rounds at a near tie; worst new cache entry {stats['worst_kv']:.2e}")
    assert stats["near_tie"] <= max(2, stats["rounds"] // 20)
    return stats


@pytest.mark.parametrize("s,draft_exit,k,n_rounds", [(TINY, 0, 3, 4), (MID, 0, 4, 4), (MID, 1, 2, 3), (PART, 0, 4, 3)],
                         ids=lambda v: v.name if hasattr(v, "name") else None)
def test_rounds_against_the_oracle(s, draft_exit, k, n_rounds):
    _say(f"[case] self-speculative rounds {s.name} B={s.batch} draft exit {draft_exit} k={k} R={s.resident}")
    _rounds(s, draft_exit, k, n_rounds)


def _tail_weights(s, Le, head):
    """layers above Le leave the hidden state unchanged; the head at R is the drafter's ("same"), its
    negation ("negated"), or the drafter's with the rows of every odd token negated ("half": the two
    heads then agree now and then, which gives rounds with some drafts accepted and some not)"""
    o = OracleSide(s, gain_jitter=0.1)
    W = {"layers": {l: dict(w) for l, w in o.weights["layers"].items()},
         "exits": {e: dict(w) for e, w in o.weights["exits"].items()}, "embed": o.weights["embed"]}
    for l in range(Le + 1, s.resident + 1):
        W["layers"][l]["W_o"] = np.zeros_like(W["layers"][l]["W_o"])
        W["layers"][l]["W_down"] = np.zeros_like(W["layers"][l]["W_down"])
    e_draft, e_last = s.exit_layers.index(Le), s.exit_layers.index(s.resident)
    Wd = W["exits"][e_draft]["W"]
    neg = (Wd ^ np.uint16(0x8000)) if Wd.dtype == np.uint16 else -Wd
    W["exits"][e_last]["g"] = W["exits"][e_draft]["g"].copy()
    if head == "same":
        W["exits"][e_last]["W"] = Wd.copy()
    elif head == "negated":
        W["exits"][e_last]["W"] = neg
    else:
        mixed = Wd.copy()
        mixed[1::2] = neg[1::2]
        W["exits"][e_last]["W"] = mixed
    return W


@pytest.mark.parametrize("s", [TINY, MID], ids=lambda s: s.name)
def test_always_right_sometimes_right_and_always_wrong_drafters(s):
    """With an identity tail above the draft layer the deep head sees the drafter's own state: the same
    head accepts every draft (k tokens per round), the negated head none (one token per round, its
    argmax being the drafter's argmin), and a head that agrees with the drafter on part of the
    vocabulary gives rounds of every length in between, each checked against the oracle's round."""
    Le, k = s.exit_layers[0], 4
    for head, want in (("same", k), ("negated", 1), ("half", None)):
        _say(f"[case] self-speculative {s.name}: deep head = the drafter's, {head}")
        st = _rounds(s, 0, k, 4, W=_tail_weights(s, Le, head))
        if want is not None:
            assert st["emitted"] == st["rounds"] * want, st
        else:
            assert st["rounds"] < st["emitted"] < st["rounds"] * k, st


def test_speculation_rejects_bad_arguments():
    s = MID
    o = OracleSide(s, gain_jitter=0.0)
    g = GpuSide(s, weights=o.weights)
    lib, m = g.model.lib, g.model
    sp = S.Speculator(m, g.kv, g.batch, 0, 2)
    args = lambda vb, e, k: (m.h, g.kv.h, g.batch.h, vb, e, k, S._ptr(sp.store.buf), S._ptr(sp.drafts), S._ptr(sp.n_emit),
                             S._ptr(sp.emit), None)
    assert lib.ee_draft_step(m.h, g.kv.h, g.batch.h, 2, None, None) == ee.EE_ERR_INVALID_ARG      # the drafter is the last exit
    assert lib.ee_draft_step(m.h, g.kv.h, g.batch.h, 7, None, None) == ee.EE_ERR_INVALID_ARG
    assert lib.ee_draft_step(None, g.kv.h, g.batch.h, 0, None, None) == ee.EE_ERR_INVALID_ARG
    assert lib.ee_verify_drafts(*args(sp.entries.h, 0, 3)) == ee.EE_ERR_CAPACITY                   # entries batch holds B * 2
    assert lib.ee_verify_drafts(*args(g.batch.h, 0, 2)) == ee.EE_ERR_INVALID_ARG                   # same batch twice
    assert lib.ee_verify_drafts(*args(sp.entries.h, 0, 0)) == ee.EE_ERR_INVALID_ARG
    assert lib.ee_verify_drafts(m.h, g.kv.h, g.batch.h, sp.entries.h, 0, 2, None, None, None, None, None) == ee.EE_ERR_INVALID_ARG
    assert lib.ee_last_error() not in (None, b"")
