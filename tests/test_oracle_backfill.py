"""Pins of the oracle's load-more-layers path (Sec. 3.3.3, the LD option): a model that starts
with R resident layers, gets layers R+1..R' later and has their keys and values filled in for the
cached tokens must, for every token that left before R in both runs, hold bit for bit the cache of
a model that had R' layers from the start.  No GPU."""
import numpy as np

import synth
from oracle import ee_oracle as orc
from helpers import OracleSide, small_shape


def _run(resident_first, steps_first, steps_after, thresholds_first):
    """decode steps_first steps with resident_first layers, then all 6 resident, backfill, decode on"""
    s = small_shape(n_layers=6, exit_layers=(2, 4, 6), resident=6, thresholds=(0.5, 0.5, 0.0), steps=4,
                    d_model=32, batch=6)
    full = OracleSide(s, std=0.3)
    part = OracleSide(s.with_(resident=resident_first, thresholds=thresholds_first), weights={
        "layers": {l: w for l, w in full.weights["layers"].items() if l <= resident_first},
        "exits": {e: w for e, w in full.weights["exits"].items() if s.exit_layers[e] <= resident_first},
        "embed": full.weights["embed"]}, std=0.3, cap=full.cap, gain_jitter=0)
    # same synthetic context on both sides for the layers they share; the partly loaded model has no
    # cache for layers it does not hold yet
    store = {}
    out = []
    for t in range(steps_first):
        pos_before = part.pos.copy()
        r = part.step(t, want_h=True)
        assert r["rc"] == 0
        for b in range(s.batch):
            store[(b, int(pos_before[b]))] = r["h"][b].copy()
        out.append(r)
    return s, full, part, store, out


def test_tokens_that_left_early_get_the_same_cache_as_with_all_layers_from_the_start():
    s, full, part, store, outs = _run(4, 2, 0, (0.5, 0.5))
    # the reference run: all six layers resident from the start, same inputs
    ref = []
    for t in range(2):
        ref.append(full.step(t, want_h=True))
    # load layers 5 and 6 into the partly loaded model (cache rows for them exist but are empty)
    kv6 = orc.OracleKV(6, s.batch, s.n_kv_heads, part.cap, s.head_dim)
    kv6.K[:4], kv6.V[:4] = part.kv.K, part.kv.V
    for l in (5, 6):
        w = full.weights["layers"][l]
        assert part.model.set_layer(l, w["g_attn"], w["W_qkv"], w["W_o"], w["g_ffn"], w["W_gate"], w["W_up"], w["W_down"]) == 0
    assert orc.backfill_kv(part.model, kv6, 4, 6, store) == 0
    ctx = part.ctx
    early = 0
    for t in range(2):
        for b in range(s.batch):
            p = int(ctx[b]) + t
            same_exit = outs[t]["layer"][b] == ref[t]["layer"][b] and outs[t]["layer"][b] < 4
            if t == 1 and not all(outs[0]["layer"][bb] == ref[0]["layer"][bb] for bb in range(s.batch)):
                continue      # the streams diverged after the first step: nothing to compare
            if same_exit:
                early += 1
                assert np.array_equal(kv6.K[:, b, :, p], full.kv.K[:, b, :, p])
                assert np.array_equal(kv6.V[:, b, :, p], full.kv.V[:, b, :, p])
            # a token forced out at layer 4 holds, in layers 5 and 6, what the fill rule gives for its state at 4
            if outs[t]["layer"][b] == 4:
                chk = orc.OracleKV(6, s.batch, s.n_kv_heads, part.cap, s.head_dim)
                assert orc.fill_skipped_kv(part.model, 4, 6, chk, b, p, store[(b, p)]) == 0
                assert np.array_equal(kv6.K[4:, b, :, p], chk.K[4:, b, :, p])
                assert kv6.K[4:, b, :, p].any()
    assert early >= 2, "the workload must have tokens that leave at the first exit"
    # positions that hold no token stay empty in the new layers
    for b in range(s.batch):
        assert not kv6.K[4:, b, :, int(ctx[b]) + 2:].any()


def test_backfill_reports_a_layer_that_is_not_resident():
    s, full, part, store, outs = _run(4, 1, 0, (0.5, 0.5))
    kv6 = orc.OracleKV(6, s.batch, s.n_kv_heads, part.cap, s.head_dim)
    assert orc.backfill_kv(part.model, kv6, 4, 6, store) == orc.ORC_ERR_NOT_RESIDENT
