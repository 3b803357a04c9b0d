"""GPU parity of the load-more-layers path (Sec. 3.3.3): a model that serves with R resident
layers gets further layers while it runs (copied and repacked on a stream of their own), the
cached tokens get keys and values in the new layers from their stored exit hidden states
(ee_backfill_kv), and decoding goes on at the new depth.  Every stage is compared with the CPU
oracle doing the same.  Run with -m gpu on an MI355X."""
import numpy as np
import pytest
import torch

import synth
from oracle import ee_oracle as orc
from helpers import OracleSide
from parity import GpuSide, compare_step, rows_close, TOL
from paper_2504_10724_amd import capi as ee
from paper_2504_10724_amd import session as S

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


F32 = synth.CONFIGS["tiny_f32"].with_(name="tiny_f32_load", n_layers=6, exit_layers=(2, 4, 6), resident=4,
                                      thresholds=(0.8, 0.8), batch=9, ctx_lo=1, ctx_hi=30, steps=4)
BF16 = synth.CONFIGS["codellama_34b_r32"].with_(name="partial_bf16_load", n_layers=6, resident=4, d_model=512,
                                                n_q_heads=8, n_kv_heads=1, d_ffn=1024, vocab=2048,
                                                exit_layers=(2, 4, 6), thresholds=(0.8, 0.8), batch=40,
                                                ctx_lo=3, ctx_hi=60, steps=4)


def _weights(s):
    full = s.with_(resident=s.n_layers)
    return {"layers": {l: synth.layer_weights(full, l) for l in range(1, s.n_layers + 1)},
            "exits": {e: synth.exit_weights(full, e) for e in range(len(s.exit_layers))},
            "embed": synth.embedding(full)}


def _sides(s):
    """oracle and library with layers 1..s.resident loaded, caches laid out for all layers, empty"""
    W = _weights(s)
    part = {"layers": {l: w for l, w in W["layers"].items() if l <= s.resident},
            "exits": {e: w for e, w in W["exits"].items() if s.exit_layers[e] <= s.resident}, "embed": W["embed"]}
    o = OracleSide(s, weights=part, fill_ctx=False, gain_jitter=0)
    o.kv = orc.OracleKV(s.n_layers, s.batch, s.n_kv_heads, o.cap, s.head_dim)
    g = GpuSide(s, weights=part, synth_rows=[])
    g.kv = S.KVCache(g.model, s.n_layers, g.cap)
    g.kv.pool.zero_()
    return W, o, g


def _context_pass(s, o, g, store, states, rows_per_call):
    for b in range(s.batch):
        rc, h = orc.prefill(o.model, o.kv, b, synth.context_tokens(s, b, int(o.ctx[b])), want_h=True)
        assert rc == 0
        for p in range(int(o.ctx[b])):
            states[(b, p)] = h[p].copy()
    pb = S.Batch(g.model, rows_per_call)
    z = np.zeros(rows_per_call, np.int32)
    pb.reset(z, z, None)
    contexts = {b: synth.context_tokens(s, b, int(o.ctx[b])) for b in range(s.batch)}
    for tok, pos, seq in S.prefill_chunks(contexts, rows_per_call):
        assert S.prefill(g.model, g.kv, pb, tok, pos, seq) == 0
        assert store.put_prefill(pb, len(tok)) == 0
    torch.cuda.synchronize()
    assert int(pb.field("status").cpu()[0]) == 0
    return pb


def _load_rest(s, W, o, g):
    loader = S.LayerLoader(g.model)
    for l in range(s.resident + 1, s.n_layers + 1):
        w = W["layers"][l]
        loader.start(l, S.LayerLoader.pin(w))
        assert o.model.set_layer(l, w["g_attn"], w["W_qkv"], w["W_o"], w["g_ffn"], w["W_gate"], w["W_up"], w["W_down"]) == 0
    assert g.model.resident_depth() == s.resident          # nothing is resident before its transfer has completed
    assert loader.poll(wait=True) == list(range(s.resident + 1, s.n_layers + 1))
    assert g.model.resident_depth() == s.n_layers
    for e, l in enumerate(s.exit_layers):
        if l > s.resident:
            g.model.set_exit(e, **W["exits"][e])
            assert o.model.set_exit(e, W["exits"][e]["g"], W["exits"][e]["W"]) == 0


def _backfill(s, o, g, pb, store, states):
    ents = sorted(states)
    seq = np.array([b for b, _ in ents], np.int32)
    pos = np.array([p for _, p in ents], np.int32)
    n = pb.B
    for lo in range(0, len(ents), n):
        assert S.backfill_kv(g.model, s.resident, s.n_layers, g.kv, pb, store, pos[lo:lo + n], seq[lo:lo + n]) == 0
    torch.cuda.synchronize()
    assert int(pb.field("status").cpu()[0]) == 0
    assert orc.backfill_kv(o.model, o.kv, s.resident, s.n_layers, states) == 0


def _compare_new_layers(s, o, g, tol):
    worst = 0.0
    for b in range(s.batch):
        n = int(o.pos[b])
        for l in range(s.resident + 1, s.n_layers + 1):
            K, V = g.kv.read_context(l, b, int(g.cap[b]))
            wk, okk = rows_close(K[:, :n].reshape(1, -1), o.kv.K[l - 1, b, :, :n].reshape(1, -1), tol)
            wv, okv = rows_close(V[:, :n].reshape(1, -1), o.kv.V[l - 1, b, :, :n].reshape(1, -1), tol)
            assert okk and okv, (b, l, wk, wv)
            assert o.kv.K[l - 1, b, :, :n].any(axis=(0, 2)).all(), "the oracle left a cached position without keys"
            assert not K[:, n:].any() and not V[:, n:].any()
            worst = max(worst, wk, wv)
    return worst


def test_serve_load_backfill_serve_fp32():
    """fp32 model: decisions bit-exact (outside the 1e-3 band) before and after the load."""
    s = F32
    _say(f"[case] load_layers {s.name} B={s.batch} resident {s.resident} -> {s.n_layers}")
    W, o, g = _sides(s)
    store = S.HiddenStore(g.model, g.kv)
    states = {}
    pb = _context_pass(s, o, g, store, states, 16)
    g.batch.reset(synth.first_tokens(s), g.ctx.astype(np.int32), None)
    sticky = np.zeros(s.batch, bool)
    for step in range(2):
        pos_before = o.pos.copy()
        rep = compare_step(s, o, g, step, sticky=sticky)
        assert rep["mismatch"] == 0, rep["detail"]
        assert store.put_step(g.batch) == 0
        for b in range(s.batch):
            states[(b, int(pos_before[b]))] = rep["oracle"]["h"][b].copy()
    assert set(rep["oracle"]["layer"].tolist()) <= {2, 4}
    _load_rest(s, W, o, g)
    _backfill(s, o, g, pb, store, states)
    worst = _compare_new_layers(s, o, g, 2e-5)
    _say(f"  new layers' cache: worst error {worst:.2e}")
    s6 = s.with_(resident=s.n_layers, thresholds=(0.8, 0.8, 0.0))
    o.s = s6
    seen = set()
    for step in range(2, 4):
        rep = compare_step(s6, o, g, step, sticky=sticky)
        assert rep["mismatch"] == 0, rep["detail"]
        seen |= set(rep["oracle"]["layer"].tolist())
    assert 6 in seen, "after the load tokens must reach the new layers"
    assert sticky.sum() <= 2


def test_backfill_from_given_states_bf16():
    """The backfill alone: the store is filled with the oracle's exit states, so both sides compute
    K and V of the new layers from identical inputs (one matrix product deep: 1e-2 normwise)."""
    s = BF16
    _say(f"[case] backfill_from_given_states {s.name}")
    W, o, g = _sides(s)
    store = S.HiddenStore(g.model, g.kv)
    rng = synth.stream(s.seed, "test.exit_states")
    states = {}
    off = np.concatenate([[0], np.cumsum(g.cap)[:-1]]).astype(np.int64)
    host = np.zeros((int(g.cap.sum()), s.d_model), np.float32)
    for b in range(s.batch):
        for p in range(int(o.ctx[b])):
            h = rng.standard_normal(s.d_model).astype(np.float32)
            states[(b, p)] = h
            host[off[b] + p] = h
    store.buf.copy_(torch.from_numpy(host.reshape(-1)))
    o.pos = o.ctx.astype(np.int32).copy()
    _load_rest(s, W, o, g)
    pb = S.Batch(g.model, 100)
    z = np.zeros(100, np.int32)
    pb.reset(z, z, None)
    _backfill(s, o, g, pb, store, states)
    worst = _compare_new_layers(s, o, g, 1e-2)
    _say(f"  {len(states)} cached tokens, layers {s.resident + 1}..{s.n_layers}: worst error {worst:.2e}")
    # the resident layers' cache rows were not touched
    K, V = g.kv.read_context(1, 0, int(g.cap[0]))
    assert not K.any() and not V.any()
    # refusals: no such cache row, a position beyond the capacity; more entries than the batch holds
    pb.reset(z, z, None)
    assert S.backfill_kv(g.model, s.resident, s.n_layers, g.kv, pb, store, np.array([0, int(g.cap[1])], np.int32),
                         np.array([s.batch, 1], np.int32)) == 0
    torch.cuda.synchronize()
    assert int(pb.field("status").cpu()[0]) == 1
    big = np.zeros(101, np.int32)
    assert S.backfill_kv(g.model, s.resident, s.n_layers, g.kv, pb, store, big, big) == ee.EE_ERR_CAPACITY
    assert S.backfill_kv(g.model, 0, s.n_layers + 1, g.kv, pb, store, z, z) == ee.EE_ERR_INVALID_ARG


def test_serve_load_backfill_serve_bf16_cache():
    """bf16 model, the whole sequence with the library's own stored states; the new layers' cache is
    compared at the bar of the other bf16 cache comparisons, then decoding runs at the new depth."""
    s = BF16
    _say(f"[case] load_layers {s.name} B={s.batch}")
    W, o, g = _sides(s)
    store = S.HiddenStore(g.model, g.kv)
    states = {}
    pb = _context_pass(s, o, g, store, states, 64)
    g.batch.reset(synth.first_tokens(s), g.ctx.astype(np.int32), None)
    th = (2.0, 2.0)        # every token runs all four layers on both sides: no decision for noise to flip
    for step in range(2):
        pos_before = o.pos.copy()
        og = o.step(step, thresholds=th, want_h=True)
        gg = g.step(step, thresholds=th)
        assert og["rc"] == 0 and gg["rc"] == 0 and gg["status"] == 0
        assert store.put_step(g.batch) == 0
        for b in range(s.batch):
            states[(b, int(pos_before[b]))] = og["h"][b].copy()
        g.batch.field("tok_in").copy_(torch.from_numpy(og["tok"]))      # both sides follow the oracle's tokens
    _load_rest(s, W, o, g)
    _backfill(s, o, g, pb, store, states)
    worst = _compare_new_layers(s, o, g, TOL["bf16"])
    _say(f"  new layers' cache: worst error {worst:.2e}")
    gg = g.step(2, thresholds=(2.0, 2.0, 0.0))
    assert gg["rc"] == 0 and gg["status"] == 0 and np.all(gg["layer"] == 6) and not gg["breach"].any()


def test_layers_loaded_after_speculative_rounds():
    """Speculative rounds (Sec. 6) on the partially loaded model, then the load action (Sec. 3.3.3): the
    store must hold, for every emitted position, the state after layer R (the verification pass has it),
    not the state after the draft layers that the round kept on the way.  The oracle gets the same
    positions by passing the inputs the GPU used (the token before, then the accepted tokens) through
    its R layers; the new layers' cache is then compared as in the other load tests."""
    s = BF16.with_(name="partial_bf16_spec_load", steps=12)
    k, rounds = 3, 3
    _say(f"[case] load_layers after {rounds} speculative rounds of {k} drafts, {s.name} B={s.batch}")
    W, o, g = _sides(s)
    store = S.HiddenStore(g.model, g.kv)
    states = {}
    pb = _context_pass(s, o, g, store, states, 64)
    g.batch.reset(synth.first_tokens(s), g.ctx.astype(np.int32), None)
    sp = S.Speculator(g.model, g.kv, g.batch, 0, k, store=store)
    tok_in, pos = synth.first_tokens(s).copy(), o.ctx.astype(np.int32).copy()
    e_last = s.exit_layers.index(s.resident)
    emitted = agree = 0
    for r in range(rounds):
        sp.round()
        torch.cuda.synchronize()
        assert int(g.batch.field("status").cpu()[0]) == 0 and int(sp.entries.field("status").cpu()[0]) == 0
        n, e = sp.n_emit.cpu().numpy(), sp.emit.cpu().numpy()
        for b in range(s.batch):
            inputs = np.array([tok_in[b]] + e[b, :n[b] - 1].tolist(), np.int32)
            rc, h = orc.prefill(o.model, o.kv, b, inputs, pos0=int(pos[b]), want_h=True)
            assert rc == 0
            for j in range(int(n[b])):
                states[(b, int(pos[b]) + j)] = h[j].copy()
                agree += int(orc.exit_head(o.model, e_last, h[j])[1] == e[b, j])
            emitted += int(n[b])
            tok_in[b], pos[b] = e[b, n[b] - 1], pos[b] + n[b]
        assert np.array_equal(g.batch.field("pos").cpu().numpy(), pos)
    _say(f"  {emitted} tokens emitted, the oracle's full-depth token is the same for {agree}")
    assert agree >= 0.9 * emitted
    o.pos = pos
    _load_rest(s, W, o, g)
    _backfill(s, o, g, pb, store, states)
    worst = _compare_new_layers(s, o, g, TOL["bf16"])
    _say(f"  new layers' cache: worst error {worst:.2e}")
    gg = g.step(0, thresholds=(2.0, 2.0, 0.0))
    assert gg["rc"] == 0 and gg["status"] == 0 and np.all(gg["layer"] == 6) and not gg["breach"].any()


def test_load_or_switch_on_measured_overheads():
    """Algorithm 1's branch fed by measurements on the device (Sec. 3.3.3, "Load More Layers Or
    Another Candidate Model?"): a partially loaded model A holds the cache of its requests; the
    overhead of loading its remaining layers (transfer + keys and values of the cached tokens in
    them) and the overhead of switching to candidate B's low-exit version (a context pass of the
    cached tokens on B) are timed with the real calls, and the branch is taken on those two numbers.
    The branch itself is checked against the oracle's on the same figures, and the cache that the
    taken action leaves behind against the oracle's."""
    from oracle.ee_pht import load_or_switch as oracle_branch
    sa = BF16.with_(name="candidate_a", steps=1)
    sb = BF16.with_(name="candidate_b", seed=1, resident=2, thresholds=(0.8,), steps=1)
    _say(f"[case] measured load-or-switch: {sa.name} R={sa.resident}/{sa.n_layers} vs {sb.name} R={sb.resident}")
    W, o, g = _sides(sa)
    store = S.HiddenStore(g.model, g.kv)
    states = {}
    pb = _context_pass(sa, o, g, store, states, 64)
    cached = [(b, p) for b in range(sa.batch) for p in range(int(o.ctx[b]))]
    pos = np.array([p for _, p in cached], np.int32)
    seq = np.array([b for b, _ in cached], np.int32)
    # option 1: the rest of A
    loader = S.LayerLoader(g.model)
    pinned = {l: S.LayerLoader.pin(W["layers"][l]) for l in range(sa.resident + 1, sa.n_layers + 1)}
    t_load = S.OverheadProbe.load(loader, pinned)
    assert g.model.resident_depth() == sa.n_layers
    t_fill = S.OverheadProbe.backfill(g.model, sa.resident, sa.n_layers, g.kv, pb, store, pos, seq)
    # option 2: candidate B's resident layers over the same cached tokens (B is in HBM already)
    ob = OracleSide(sb, fill_ctx=False, gain_jitter=0, cap=o.cap)
    gb = GpuSide(sb, weights=ob.weights, synth_rows=[], max_pos=int(g.cap.max()))
    gb.kv = S.KVCache(gb.model, sb.resident, g.cap)          # B caches the same requests as A
    gb.kv.pool.zero_()
    pbb = S.Batch(gb.model, 64)
    z = np.zeros(64, np.int32)
    pbb.reset(z, z, None)
    contexts = {b: synth.context_tokens(sa, b, int(o.ctx[b])) for b in range(sa.batch)}
    t_switch = S.OverheadProbe.context_pass(gb.model, gb.kv, pbb, contexts)
    assert int(pbb.field("status").cpu()[0]) == 0 and int(pb.field("status").cpu()[0]) == 0
    assert t_load > 0 and t_fill > 0 and t_switch > 0
    decision, figures = S.reassess(t_load + t_fill, {"candidate_b": t_switch})
    _say(f"  load {t_load * 1e3:.2f} ms + backfill {t_fill * 1e3:.2f} ms vs switch {t_switch * 1e3:.2f} ms -> {decision}")
    assert decision == oracle_branch(t_load + t_fill, {"candidate_b": t_switch})
    assert decision == (("load", None) if t_load + t_fill < t_switch else ("switch", "candidate_b"))
    # the formula from rates gives the same overheads as the direct timings it was derived from
    n_new = sa.n_layers - sa.resident
    layer_bytes = sum(t.numel() * t.element_size() for t in pinned[sa.n_layers].values())
    est = S.overhead_of_loading(n_new, layer_bytes, n_new * layer_bytes / t_load, len(cached), len(cached) * n_new / t_fill)
    assert abs(est - (t_load + t_fill)) <= 1e-9 * max(1.0, est)
    assert abs(S.overhead_of_switching(len(cached), len(cached) / t_switch) - t_switch) <= 1e-12
    # whichever way the branch went, both actions were carried out above: check what they left
    for l in range(sa.resident + 1, sa.n_layers + 1):
        w = W["layers"][l]
        assert o.model.set_layer(l, w["g_attn"], w["W_qkv"], w["W_o"], w["g_ffn"], w["W_gate"], w["W_up"], w["W_down"]) == 0
    assert orc.backfill_kv(o.model, o.kv, sa.resident, sa.n_layers, states) == 0
    for b in (0, sa.batch // 2, sa.batch - 1):
        n = int(o.ctx[b])
        for l in range(sa.resident + 1, sa.n_layers + 1):
            K, V = g.kv.read_context(l, b, n)
            wk, okk = rows_close(K.reshape(1, -1), o.kv.K[l - 1, b, :, :n].reshape(1, -1), TOL["bf16"])
            wv, okv = rows_close(V.reshape(1, -1), o.kv.V[l - 1, b, :, :n].reshape(1, -1), TOL["bf16"])
            assert okk and okv, (b, l, wk, wv)
    for b in range(sb.batch):
        rc, _ = orc.prefill(ob.model, ob.kv, b, contexts[b])
        assert rc == 0
    for b in (0, sb.batch - 1):
        n = int(o.ctx[b])
        for l in range(1, sb.resident + 1):
            K, V = gb.kv.read_context(l, b, n)
            wk, okk = rows_close(K.reshape(1, -1), ob.kv.K[l - 1, b, :, :n].reshape(1, -1), TOL["bf16"])
            wv, okv = rows_close(V.reshape(1, -1), ob.kv.V[l - 1, b, :, :n].reshape(1, -1), TOL["bf16"])
            assert okk and okv, (b, l, wk, wv)
