"""The bf16 workloads at their real widths, depths, exit sets and batch sizes against the CPU oracle.

Two kinds of test, both through the C ABI:

* teacher-forced: the per-call entry points run layer by layer; after every call the rows the
  oracle holds are compared (hidden state, appended keys/values, logits, confidence, decision,
  compaction lists, keys/values of the skipped layers) under the per-call contract -- 2e-2
  normwise for hidden states and logits, 1e-3 for the confidence, decisions bit-exact outside the
  1e-3 band around the threshold -- and then the GPU state of those rows is overwritten with the
  oracle's, so that every layer, every exit and every fill of the model is checked from identical
  inputs.
* free-running: whole ee_decode_step calls over consecutive steps at the workload's real depth;
  the oracle recomputes a sample of rows (rows are independent), classified with the noise band
  of parity.compare_step; afterwards every resident layer's cache entries at the new positions
  are compared, so a later step reading an earlier step's filled entries is covered.

Deep models take their layer weights from a few drawn layers in rotation (helpers.draw_weights):
the launch sequence, shapes and sizes are the workload's, the host and device footprint is not.
"""
import gc

import numpy as np
import pytest
import torch

import synth
from oracle import ee_oracle as orc
from helpers import OracleSide, draw_weights, draw_contexts
from parity import GpuSide, compare_step, report_line, shadow_of, rows_close, TOL, NEAR
from paper_2504_10724_amd import session as S

pytestmark = pytest.mark.gpu

C = synth.CONFIGS
KV_TOL = 1e-2          # one bf16 rounding of K (after RoPE) and V against max |.| of the head


def _say(msg):
    print(msg, flush=True)


_weights = {}


def weights_for(s, n_distinct=None):
    """drawn once per (shape, seed, residency, number of distinct layers) for the whole module"""
    key = (s.d_model, s.d_ffn, s.n_q_heads, s.n_kv_heads, s.vocab, s.seed, s.resident, s.exit_layers, n_distinct)
    if key not in _weights:
        _say(f"  [weights] {s.name}: {n_distinct or s.resident} drawn layer(s) for {s.resident} resident")
        _weights[key] = draw_weights(s, n_distinct)
    return _weights[key]


@pytest.fixture(autouse=True)
def _release_device_memory():
    yield
    gc.collect()
    torch.cuda.empty_cache()


def _bits(x):
    return synth.to_bf16_bits(np.ascontiguousarray(x, np.float32))


# ---------------------------------------------------------------- teacher-forced, call by call
def forced_steps(s, rows, W, steps):
    rows = [int(b) for b in rows]
    n = len(rows)
    ctxs = draw_contexts(s, rows)
    o = OracleSide(s, rows=rows, weights=W, gain_jitter=0, contexts=ctxs)
    g = GpuSide(s, weights=W, synth_rows=rows, contexts=ctxs)
    _say(f"  both sides ready: B={s.batch}, sampled rows {rows}, R={s.resident}, exits {s.resident_exits}")
    f = g.batch.field
    rows_t = torch.as_tensor(rows, device="cuda", dtype=torch.long)
    R, res_exits = s.resident, s.resident_exits
    tol = TOL[s.dtype]
    worst = dict(h=0.0, kv=0.0, logits=0.0, conf=0.0, fill=0.0)
    tally = dict(layer_rows=0, head_rows=0, near=0, tok_close=0, fill_entries=0)
    tok_all = synth.first_tokens(s).copy()
    pos_all = g.ctx.astype(np.int32).copy()
    logits = torch.zeros((s.batch, s.vocab), dtype=torch.float32, device="cuda")
    for step in range(steps):
        scale = synth.row_scale(s, step)
        g.batch.reset(tok_all, pos_all, scale)
        g.batch.begin_step()
        torch.cuda.synchronize()
        h_o = np.stack([orc.embed(o.model, t) for t in o.tok]).astype(np.float32)
        assert np.array_equal(f("h")[rows_t].cpu().numpy(), h_o), "embedding rows differ"
        active = np.ones(n, np.uint8)
        out_tok_o = np.full(n, -1, np.int32)
        for l in range(1, R + 1):
            act = np.nonzero(active)[0]
            assert S.layer_forward(g.model, l, g.kv, g.batch) == 0
            torch.cuda.synchronize()
            assert orc.layer_forward(o.model, l, o.kv, active, o.pos, h_o) == 0
            hg = f("h")[rows_t].cpu().numpy()
            if act.size:
                w, ok = rows_close(hg[act], h_o[act], tol)
                worst["h"] = max(worst["h"], w)
                assert ok, f"step {step} layer {l}: hidden state {w:.2e}"
            gone = np.nonzero(active == 0)[0]
            assert np.array_equal(hg[gone], h_o[gone]), f"layer {l} moved a row that had left"
            for i in act:
                p = int(o.pos[i])
                K, V = g.kv.read_context(l, rows[i], 1, pos0=p)
                wk, okk = rows_close(K[:, 0], o.kv.K[l - 1, i, :, p], KV_TOL)
                wv, okv = rows_close(V[:, 0], o.kv.V[l - 1, i, :, p], KV_TOL)
                worst["kv"] = max(worst["kv"], wk, wv)
                assert okk and okv, f"step {step} layer {l} row {rows[i]}: appended K/V {wk:.2e} {wv:.2e}"
                # the next call starts from the oracle's state: hidden rows below, cache entry here
                g.kv.write_context(l, rows[i], _bits(o.kv.K[l - 1, i, :, p:p + 1]), _bits(o.kv.V[l - 1, i, :, p:p + 1]), pos0=p)
            tally["layer_rows"] += int(act.size)
            if act.size:
                f("h")[rows_t[torch.as_tensor(act, device="cuda")]] = torch.from_numpy(h_o[act]).cuda()
            if l not in res_exits:
                continue
            e = res_exits.index(l)
            th, force = np.float32(s.thresholds[e]), l == R
            assert S.exit_head(g.model, s.exit_layers.index(l), float(th), force, g.batch, logits) == 0
            torch.cuda.synchronize()
            n_act = int(f("n_active").cpu()[0])
            idx = f("active_idx").cpu().numpy()[:n_act]
            where = {int(r): j for j, r in enumerate(idx)}
            assert sorted(rows[i] for i in act) == sorted(r for r in rows if r in where), "active lists differ"
            conf_g, tok_g = f("head_conf").cpu().numpy(), f("head_tok").cpu().numpy()
            exit_g, br_g = f("head_exit").cpu().numpy().copy(), f("head_breach").cpu().numpy().copy()
            leaves = []
            for i in act:
                j = where[rows[i]]
                c_o, t_o, z_o = orc.exit_head(o.model, s.exit_layers.index(l), h_o[i], float(scale[rows[i]]), want_logits=True)
                w, ok = rows_close(logits[j:j + 1].cpu().numpy(), z_o[None], tol)
                worst["logits"] = max(worst["logits"], w)
                assert ok, f"step {step} exit {l} row {rows[i]}: logits {w:.2e}"
                ce = abs(float(conf_g[j]) - c_o)
                worst["conf"] = max(worst["conf"], ce)
                assert ce <= NEAR, f"step {step} exit {l} row {rows[i]}: confidence {conf_g[j]} vs {c_o}"
                met = np.float32(c_o) >= th
                ex_o, br_o = int(met or force), int(force and not met)
                near = (0.0 < th <= 1.0) and abs(c_o - float(th)) <= NEAR
                tally["head_rows"] += 1
                if near:
                    tally["near"] += 1
                else:
                    assert int(exit_g[j]) == ex_o and int(br_g[j]) == br_o, f"step {step} exit {l} row {rows[i]}: decision"
                if int(tok_g[j]) != t_o:
                    # only where the oracle's own two best candidates are closer than the confidence tolerance
                    p_ = np.exp(z_o.astype(np.float64) - z_o.max()); p_ /= p_.sum()
                    assert p_.max() - p_[int(tok_g[j])] <= 2 * NEAR, f"step {step} exit {l} row {rows[i]}: token"
                    tally["tok_close"] += 1
                # the compaction and what follows run on the oracle's decision
                exit_g[j], br_g[j] = ex_o, br_o
                f("head_exit")[j] = ex_o
                f("head_breach")[j] = br_o
                f("head_tok")[j] = int(t_o)
                f("head_conf")[j] = float(c_o)
                if ex_o:
                    leaves.append(i)
                    out_tok_o[i] = t_o
            assert S.compact_active(g.batch, s.exit_layers.index(l), l) == 0
            torch.cuda.synchronize()
            keep_o, gone_o = orc.compact(exit_g[:n_act], idx)
            n_keep, n_gone = int(f("n_active").cpu()[0]), int(f("n_exited").cpu()[0])
            assert (n_keep, n_gone) == (keep_o.size, gone_o.size)
            assert np.array_equal(f("active_idx").cpu().numpy()[:n_keep], keep_o), "survivor list"
            assert np.array_equal(f("exited_idx").cpu().numpy()[:n_gone], gone_o), "leaver list"
            assert np.all(f("out_layer").cpu().numpy()[gone_o] == l)
            if force:
                assert n_keep == 0
            if l < R:
                assert S.fill_skipped_kv(g.model, l, R, g.kv, g.batch) == 0
                torch.cuda.synchronize()
                for i in leaves:
                    p = int(o.pos[i])
                    assert orc.fill_skipped_kv(o.model, l, R, o.kv, int(i), p, h_o[i]) == 0
                    for l2 in range(l + 1, R + 1):
                        K, V = g.kv.read_context(l2, rows[i], 1, pos0=p)
                        wk, okk = rows_close(K[:, 0], o.kv.K[l2 - 1, i, :, p], KV_TOL)
                        wv, okv = rows_close(V[:, 0], o.kv.V[l2 - 1, i, :, p], KV_TOL)
                        worst["fill"] = max(worst["fill"], wk, wv)
                        assert okk and okv, f"step {step} fill ({l}, {R}] layer {l2} row {rows[i]}: {wk:.2e} {wv:.2e}"
                        g.kv.write_context(l2, rows[i], _bits(o.kv.K[l2 - 1, i, :, p:p + 1]),
                                           _bits(o.kv.V[l2 - 1, i, :, p:p + 1]), pos0=p)
                        tally["fill_entries"] += 1
            for i in leaves:
                active[i] = 0
        assert not active.any() and int(f("status").cpu()[0]) == 0
        tok_all = f("out_tok").cpu().numpy().copy()
        assert np.all(tok_all >= 0)
        tok_all[rows] = out_tok_o
        o.tok = out_tok_o.copy()
        o.pos += 1
        pos_all += 1
        _say(f"  step {step}: every layer, exit and fill within the per-call contract; worst so far: hidden {worst['h']:.2e}, "
             f"appended K/V {worst['kv']:.2e}, logits {worst['logits']:.2e}, confidence {worst['conf']:.2e}, "
             f"filled K/V {worst['fill']:.2e}")
    _say(f"  checked {tally['layer_rows']} row-layers, {tally['head_rows']} exit-head rows ({tally['near']} inside the "
         f"1e-3 band, {tally['tok_close']} tokens between near-equal candidates), {tally['fill_entries']} filled entries")
    assert tally["fill_entries"] > 0 and tally["head_rows"] > n, "workload must fill and reach a second exit"
    return tally


# all exits of the workload, two layers per segment, real width and batch
FORCED = [
    (C["llama2_70b"].with_(name="70b_w_forced", n_layers=8, resident=8, exit_layers=(2, 4, 6, 8), steps=3), [0, 37, 101, 255], 2),
    (C["codellama_34b_r32"].with_(name="34b_w_forced", n_layers=12, resident=8, exit_layers=(2, 4, 6, 8, 10, 12), steps=2),
     [5, 64, 127], 2),
    (C["llama2_7b"].with_(name="7b_w_forced", n_layers=8, resident=8, exit_layers=(2, 4, 6, 8), steps=2), [0, 21, 40, 63], 2),
    (C["switch_7b_a"].with_(name="7b_b512_forced", n_layers=6, resident=4, exit_layers=(2, 4, 6), steps=2),
     [0, 255, 256, 511], 2),
]


@pytest.mark.parametrize("s,rows,n_distinct", FORCED, ids=lambda v: v.name if hasattr(v, "name") else None)
def test_every_layer_exit_and_fill_teacher_forced(s, rows, n_distinct):
    _say(f"[case] teacher-forced {s.name} B={s.batch} d={s.d_model} R={s.resident}/{s.n_layers} steps={s.steps}")
    forced_steps(s, rows, weights_for(s, n_distinct), s.steps)


def test_step_equals_its_calls_at_70b_width():
    """ee_decode_step against the per-call sequence, bit for bit, with four exits and two layers per
    segment at d = 8192 and 256 rows: together with the teacher-forced test of the calls this puts
    the step's own paths (operand hand-over between kernels, segmented fill) under the per-call contract."""
    s = C["llama2_70b"].with_(name="70b_w_step_vs_calls", n_layers=8, resident=8, exit_layers=(2, 4, 6, 8), steps=1)
    _say(f"[case] step_vs_calls {s.name} B={s.batch}")
    W = weights_for(s, 2)
    g1 = GpuSide(s, weights=W, synth_rows=[])
    g2 = GpuSide(s, weights=W, synth_rows=[])
    assert torch.equal(g1.kv.pool.view(torch.int64), g2.kv.pool.view(torch.int64))
    sc = synth.row_scale(s, 0)
    r1 = g1.step(0, scale=sc)
    g2.batch.set_row_scale(sc)
    g2.batch.begin_step()
    for l in range(1, s.resident + 1):
        assert S.layer_forward(g2.model, l, g2.kv, g2.batch) == 0
        if l in s.exit_layers:
            e = s.exit_layers.index(l)
            assert S.exit_head(g2.model, e, float(s.thresholds[e]), l == s.resident, g2.batch) == 0
            assert S.compact_active(g2.batch, e, l) == 0
            assert S.fill_skipped_kv(g2.model, l, s.resident, g2.kv, g2.batch) == 0
    torch.cuda.synchronize()
    f1, f2 = g1.batch.field, g2.batch.field
    for k in ("out_tok", "out_layer", "out_conf", "out_breach", "h"):
        assert torch.equal(f1(k), f2(k)), k
    assert len(set(r1["layer"].tolist())) == 4, "all four exits must be used"
    # the whole pool: every appended and every filled entry of every row and layer
    assert torch.equal(g1.kv.pool.view(torch.int64), g2.kv.pool.view(torch.int64))


# ---------------------------------------------------------------- free-running, real depth
def free_steps(s, rows, W, steps, n_shadows=2, band_floor=1e-2, g=None):
    rows = [int(b) for b in rows]
    ctxs = draw_contexts(s, rows)
    o = OracleSide(s, rows=rows, weights=W, gain_jitter=0, contexts=ctxs)
    if g is None:
        g = GpuSide(s, weights=W, synth_rows=rows, contexts=ctxs)
    shadows = [shadow_of(o, seed=7 + k, contexts=ctxs) for k in range(n_shadows)]
    del ctxs
    _say(f"  both sides ready: B={s.batch}, sampled rows {rows}, R={s.resident}, exits {s.resident_exits}")
    th = np.asarray(s.thresholds, np.float32)
    res_exits = s.resident_exits
    ctx0 = g.ctx.copy()
    compared = excluded = 0
    for step in range(steps):
        rep = compare_step(s, o, g, step, shadow=shadows, band_floor=band_floor)
        _say(report_line(step, rep))
        out = rep["excluded_now"]
        for i in range(len(rows)):
            og, gg = rep["oracle"], rep["gpu"]
            _say(f"    row {rows[i]}: oracle (tok {og['tok'][i]}, layer {og['layer'][i]}, conf {og['conf'][i]:.4f}) "
                 f"gpu (tok {gg['tok'][i]}, layer {gg['layer'][i]}, conf {gg['conf'][i]:.4f})"
                 f"{' excluded' if out[i] else ''}")
        for d in rep["detail"]:
            _say(f"    MISMATCH {d}")
        assert rep["mismatch"] == 0, rep["detail"]
        compared += rep["rows"]
        excluded += int(out.sum())
        # A row excluded in this step (inside a band) may have taken the other decision on the GPU.
        # It is counted, and then the oracles adopt the GPU's token and this step's cache entries of
        # that row, so that the row is compared again from a common state in the following steps.
        for i in np.nonzero(out)[0]:
            p = int(ctx0[rows[i]]) + step
            o.tok[i] = rep["gpu"]["tok"][i]
            for l in range(1, s.resident + 1):
                K, V = g.kv.read_context(l, rows[i], 1, pos0=p)
                for side in [o] + shadows:
                    side.kv.K[l - 1, i, :, p] = K[:, 0]
                    side.kv.V[l - 1, i, :, p] = V[:, 0]
        # what holds for every row of the batch at any size
        ga = rep["gpu_all"]
        assert ga["n_active"] == 0 and np.all(np.isin(ga["layer"], res_exits))
        assert np.all(ga["conf"] > 0) and np.all(ga["conf"] <= 1.0 + 1e-6)
        assert np.all((ga["tok"] >= 0) & (ga["tok"] < s.vocab))
        assert int(ga["counts"][:len(res_exits)].sum()) == s.batch * (step + 1)
        for e, l in enumerate(res_exits):
            at = ga["layer"] == l
            if l < s.resident:
                assert np.all(ga["conf"][at] >= th[e]) and not ga["breach"][at].any()
            else:
                assert np.array_equal(ga["breach"][at] != 0, ga["conf"][at] < th[e])
        assert np.array_equal(ga["pos"], ctx0 + step + 1)
    _say(f"  {compared} sampled row-steps compared, {excluded} excluded (inside a band)")
    assert compared >= max(1, len(rows) * steps // 3), "too few sampled row-steps were comparable"
    # every resident layer's entries at the positions of these steps (executed or filled), normwise per
    # (row, layer): within the 2e-2 of the hidden states they come from, or, where the shadows' own
    # entries have drifted further from the oracle's than a quarter of that, within four times their drift
    worst = over = 0.0
    for i, b in enumerate(rows):
        p0 = int(ctx0[b])
        for l in range(1, s.resident + 1):
            K, V = g.kv.read_context(l, b, steps, pos0=p0)
            for got, ref in ((K, "K"), (V, "V")):
                want = getattr(o.kv, ref)[l - 1, i, :, p0:p0 + steps]
                scale = max(float(np.abs(want).max()), 1e-30)
                err = float(np.abs(got - want).max()) / scale
                drift = max(float(np.abs(getattr(sh.kv, ref)[l - 1, i, :, p0:p0 + steps] - want).max()) / scale for sh in shadows)
                worst = max(worst, err)
                over = max(over, err / max(TOL["bf16"], 4 * drift))
                assert err <= max(TOL["bf16"], 4 * drift), (b, l, ref, err, drift)
    _say(f"  cache of the sampled rows, {s.resident} layers x {steps} new positions: worst (row, layer) {worst:.2e}, "
         f"at most {over:.2f} of its bound")
    return g, o, excluded


def test_config2_llama2_7b_whole():
    """32 drawn layers, exits 8/16/24/32, batch 64, contexts 128..1024, 8 consecutive steps."""
    s = C["llama2_7b"].with_(name="cfg2_7b_whole", steps=8)
    _say(f"[case] free-running {s.name} B={s.batch} R={s.resident} steps={s.steps}")
    free_steps(s, [0, 13, 21, 40, 63], weights_for(s), s.steps)


def test_config3_codellama_34b_r32_of_48():
    """48-layer model with layers 1..32 resident, exits every 8 layers, batch 128, 3 steps: the rows
    still in at layer 32 leave there, below the threshold or not."""
    s = C["codellama_34b_r32"].with_(name="cfg3_34b_r32", steps=3)
    _say(f"[case] free-running {s.name} B={s.batch} R={s.resident}/{s.n_layers} steps={s.steps}")
    g, o, _ = free_steps(s, [5, 64, 127], weights_for(s, 4), s.steps)
    assert int(g.batch.field("breach_count").cpu()[0]) > 0, "some row must be forced out at layer 32 below 0.8"


def test_config4_llama2_70b_full_depth():
    """80 layers, exits 20/40/60/80, batch 256, contexts 512..2048: the benchmark's launch sequence,
    including the three 20-layer fill segments, over 3 consecutive steps."""
    s = C["llama2_70b"].with_(name="cfg4_70b_full", steps=3)
    _say(f"[case] free-running {s.name} B={s.batch} R={s.resident} steps={s.steps}")
    free_steps(s, [0, 37, 101, 180, 255], weights_for(s, 4), s.steps, n_shadows=2)


@pytest.mark.parametrize("batch", [1, 16], ids=lambda b: f"b{b}")
def test_config4_small_batches_full_depth(batch):
    """the sweep's small batches at full depth: position shares in attention, K-sliced products"""
    s = C["llama2_70b"].with_(name=f"cfg4_70b_b{batch}", batch=batch, steps=2)
    _say(f"[case] free-running {s.name} B={s.batch} R={s.resident} steps={s.steps}")
    free_steps(s, [0] if batch == 1 else [0, 7, 15], weights_for(s, 4), s.steps)


def test_config5_two_7b_models_one_window_each():
    """Two 20-of-32-layer models resident together, batch 512; each serves one real 32-step window,
    then the routing rule picks the model with the larger fraction of confident exits."""
    sa = C["switch_7b_a"].with_(name="cfg5_a")
    sb = C["switch_7b_b"].with_(name="cfg5_b")
    _say(f"[case] free-running two models {sa.name}/{sb.name} B={sa.batch} R={sa.resident} window={sa.steps}")
    lanes, fractions = [], []
    for s in (sa, sb):
        g, o, _ = free_steps(s, [0, 255, 256, 511], weights_for(s, 4), s.steps)
        breaches = int(g.batch.field("breach_count").cpu()[0])
        fractions.append(1.0 - breaches / (s.steps * s.batch))
        lanes.append((g.model, g.kv, g.batch, s.thresholds))
        _say(f"  {s.name}: confident-exit fraction over the window {fractions[-1]:.4f}")
    sw = S.WindowSwitcher(lanes, sa.steps)
    sw.last_fraction = list(fractions)
    sw.steps_done = [sa.steps, sb.steps]
    want = 0 if fractions[0] >= fractions[1] else 1
    assert sw.choose() == want
    # the model with the logit scales shifted up is the more confident one
    assert fractions[0] > fractions[1]
