"""GPU-vs-oracle comparison helpers (test infrastructure).

Per call (same inputs on both sides): exit masks, tokens, breach flags and
compaction indices bit-exact, except rows whose oracle confidence lies within
NEAR = 1e-3 of the threshold, which are counted separately.  Hidden states and
logits: per row, max |gpu - oracle| <= tol * max |oracle| with tol = 2e-2 for
bf16 models and 2e-4 for fp32 models.  The teacher-forced tests
(test_gpu_configs.py) apply exactly this at every layer, exit and fill of a
model: before each call the GPU is given the oracle's state.

Whole decode steps run both sides freely through many layers.  Under the
bf16 contract every matrix-product operand is rounded to bfloat16, and a chain
of such roundings turns a difference of one fp32 ulp (a different summation
order) into differences of bf16 size within a few layers, in the oracle as in
any other implementation.  The step comparison therefore measures that noise
with the oracle itself: further oracles whose fp32 RMSNorm gains are perturbed
by one part in 10^6 ("shadows") run beside the first, and the largest confidence
change they show at an exit is that exit's band (never below 1e-3).  A row
whose confidence lies inside the band of an exit with a deciding threshold (or
whose decision a shadow changed) may decide otherwise; rows within the 1e-3
band are also counted on their own.  A row that uses this is excluded from then
on (or resynchronised, in the sampled tests) and counted.  Every other row,
rows inside a band that took the oracle's decision included,
must match bit-exactly on exit layer, token and breach flag, its confidence
within the band of the exit it left at and its hidden state there within the
hidden-state band (2e-2, or the largest drift the shadows show at their exits if
that is more: after tens of layers the contract's own noise reaches 2e-2).  A
row whose confidence or hidden state differs by more than its band but less than
four times the band is excluded and counted too (a band is the largest of a few
hundred draws of the noise; one more draw exceeds it now and then); beyond four
times the band it is a mismatch.
"""
import numpy as np
import torch

import synth
from oracle import ee_oracle as orc
from helpers import OracleSide
from paper_2504_10724_amd import session as S

NEAR = 1e-3
TOL = {"bf16": 2e-2, "f32": 2e-4}


def rows_close(got, want, tol):
    """normwise per-row closeness; returns the worst ratio err/scale"""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    err = np.abs(got - want).reshape(got.shape[0], -1).max(1)
    scale = np.abs(want).reshape(want.shape[0], -1).max(1)
    worst = float((err / np.maximum(scale, 1e-30)).max()) if got.size else 0.0
    return worst, worst <= tol


class GpuSide:
    """libee model + cache + batch state for the same synthetic workload the oracle sees."""

    def __init__(self, s, weights=None, std=0.02, cap_multiple=32, max_pos=None, synth_rows=None, contexts=None):
        """synth_rows: if given, only these rows get their cached context from the seeded host
        generator (the rows an oracle will recompute); the others are filled on the device from
        the same distribution, which is much faster for large batches.  contexts: what
        helpers.draw_contexts returned for those rows (drawn once for both sides)."""
        self.s = s
        if weights is None:
            weights = {
                "layers": {l: synth.layer_weights(s, l, std) for l in range(1, s.resident + 1)},
                "exits": {e: synth.exit_weights(s, e, std) for e, l in enumerate(s.exit_layers) if l <= s.resident},
                "embed": synth.embedding(s, std),
            }
        self.ctx = synth.context_lengths(s)
        self.cap = synth.capacity_for(self.ctx, s.steps, cap_multiple)
        mp = int(self.cap.max()) if max_pos is None else max_pos
        self.model = S.Model.from_shape(s, max_pos=mp)
        on_device = {}                      # layers that share their host tensors share the device copies
        for l, w in weights["layers"].items():
            if id(w) not in on_device:
                self.model.set_layer(l, **w)
                on_device[id(w)] = self.model._keep[("layer", l)]
            else:
                g_attn, w_qkv, w_o, g_ffn, w_gate_up, w_down = on_device[id(w)]
                self.model.set_layer_device(l, g_attn=g_attn, w_qkv=w_qkv, w_o=w_o, g_ffn=g_ffn,
                                            w_gate_up=w_gate_up, w_down=w_down)
        for e, w in weights["exits"].items():
            self.model.set_exit(e, **w)
        self.model.set_embed(weights["embed"])
        self.kv = S.KVCache(self.model, s.resident, self.cap)
        if synth_rows is not None:
            gen = torch.Generator(device="cuda")
            gen.manual_seed(s.seed + 1)
            pool = self.kv.pool.view(torch.bfloat16 if s.dtype == "bf16" else torch.float32)
            chunk = 1 << 30
            for i in range(0, pool.numel(), chunk):
                pool[i:i + chunk].normal_(0.0, 0.02 * float(np.sqrt(s.d_model)), generator=gen)
        for l in range(1, s.resident + 1):
            for b in (range(s.batch) if synth_rows is None else synth_rows):
                K, V = contexts[(l, int(b))] if contexts is not None else synth.kv_rows(s, l, b, int(self.ctx[b]))
                self.kv.write_context(l, b, K, V)
        self.batch = S.Batch(self.model, s.batch)
        self.batch.reset(synth.first_tokens(s), self.ctx.astype(np.int32), None)

    def step(self, step_idx, thresholds=None, scale=None):
        th = self.s.thresholds if thresholds is None else thresholds
        sc = synth.row_scale(self.s, step_idx) if scale is None else scale
        self.batch.set_row_scale(sc)
        rc = S.decode_step(self.model, self.kv, self.batch, list(th))
        torch.cuda.synchronize()
        f = self.batch.field
        return dict(rc=rc, tok=f("out_tok").cpu().numpy(), layer=f("out_layer").cpu().numpy(),
                    conf=f("out_conf").cpu().numpy(), breach=f("out_breach").cpu().numpy(),
                    counts=f("exit_counts").cpu().numpy(), status=int(f("status").cpu()[0]),
                    n_active=int(f("n_active").cpu()[0]), pos=f("pos").cpu().numpy(),
                    tok_in=f("tok_in").cpu().numpy(), h=f("h").cpu().numpy())


def shadow_of(o, rel=1e-6, seed=7, contexts=None):
    """A further oracle on the same workload (same rows) whose fp32 norm gains differ by `rel`
    (relative): the probe of how far the precision contract's own rounding
    lets two correct implementations drift apart."""
    s = o.s
    rng = np.random.default_rng(seed)
    w2 = {"layers": {l: dict(w) for l, w in o.weights["layers"].items()},
          "exits": o.weights["exits"], "embed": o.weights["embed"]}
    for w in w2["layers"].values():
        for k in ("g_attn", "g_ffn"):
            w[k] = (w[k].astype(np.float64) * (1 + rel * rng.standard_normal(s.d_model))).astype(np.float32)
    return OracleSide(s, rows=o.rows, weights=w2, cap=o.cap, gain_jitter=0, contexts=contexts)


def compare_step(s, o, g, step_idx, thresholds=None, sticky=None, shadow=None, band_floor=NEAR):
    """Runs decode step `step_idx` on the oracle, on the GPU and on the shadow oracles (one, a
    list, or none), and classifies every row the oracle holds (o.rows: all rows of the batch, or a
    sample; the GPU always runs the whole batch).  `sticky`: rows (indices into o.rows) already
    excluded.  band_floor: lowest band (a handful of sampled rows cannot estimate the tail of the
    noise, so the sampled tests keep the floor that the batch-wide tests measure)."""
    th = np.asarray(s.thresholds if thresholds is None else thresholds, np.float32)
    rows = np.asarray(o.rows)
    n = rows.size
    sc_all = synth.row_scale(s, step_idx)
    sc = sc_all[rows]
    shadows = [] if shadow is None else (list(shadow) if isinstance(shadow, (list, tuple)) else [shadow])
    for sh in shadows:
        sh.tok = o.tok.copy()              # the probes follow the oracle's token stream
    og = o.step(step_idx, thresholds=th, want_h=True, scale=sc)
    ga = g.step(step_idx, thresholds=th, scale=sc_all)
    assert og["rc"] == 0 and ga["rc"] == 0, (og["rc"], ga["rc"])
    assert ga["status"] == 0, f"device status {ga['status']}"
    per_row = ("tok", "layer", "conf", "breach", "pos", "tok_in", "h")
    gg = {k: (v[rows] if k in per_row else v) for k, v in ga.items()}
    res_exits = s.resident_exits
    tr = og["conf_trace"]
    band = np.full(len(res_exits), max(NEAR, band_floor), np.float64)
    unstable = np.zeros(n, bool)
    own = np.zeros((n, len(res_exits)), np.float64)   # largest confidence change the shadows show for this very row
    h_scale = np.maximum(np.abs(og["h"]).max(1), 1e-30)
    h_band = TOL[s.dtype]                  # hidden state where the row left: the per-call bar, or the shadows' drift
    for sh in shadows:
        sg = sh.step(step_idx, thresholds=th, want_h=True, scale=sc)
        assert sg["rc"] == 0
        unstable |= (sg["tok"] != og["tok"]) | (sg["layer"] != og["layer"])
        same = sg["layer"] == og["layer"]
        if same.any():
            h_band = max(h_band, float((np.abs(sg["h"].astype(np.float64) - og["h"]).max(1) / h_scale)[same].max()))
        for e in range(len(res_exits)):
            both = np.isfinite(tr[:, e]) & np.isfinite(sg["conf_trace"][:, e])
            if both.any():
                dev = np.abs(tr[:, e].astype(np.float64) - sg["conf_trace"][:, e])
                band[e] = max(band[e], float(dev[both].max()))
                own[both, e] = np.maximum(own[both, e], dev[both])
    strict = np.zeros(n, bool)
    noisy = np.zeros(n, bool)
    for e in range(len(res_exits)):
        if not (0.0 < th[e] <= 1.0):
            continue   # a threshold <= 0 is always met and one above 1 never: nothing to decide
        c = tr[:, e]
        reached = np.isfinite(c)
        strict |= reached & (np.abs(c - th[e]) <= NEAR)
        # the exit's band, or four times what the shadows show for this row if that is more (rows with a
        # large logit scale are far more sensitive than the rest, and a few shadows sample their noise poorly)
        noisy |= reached & (np.abs(c - th[e]) <= np.maximum(band[e], 4 * own[:, e]))
    left_at = np.array([res_exits.index(int(l)) if int(l) in res_exits else 0 for l in og["layer"]])
    # a different token is tolerated only where the oracle's own top candidates are closer than
    # the noise allows (one probability may fall by the band while the other rises by it):
    # p_oracle(tok_oracle) - p_oracle(tok_gpu) <= 2 * band at the exit the row left
    tok_amb = np.zeros(n, bool)
    for i in np.nonzero((og["tok"] != gg["tok"]) & (og["layer"] == gg["layer"]))[0]:
        e = left_at[i]
        _, _, z = orc.exit_head(o.model, s.exit_layers.index(res_exits[e]), og["h"][i], float(sc[i]), want_logits=True)
        p = np.exp(z.astype(np.float64) - z.max()); p /= p.sum()
        tok_amb[i] = (p.max() - p[gg["tok"][i]]) <= 2 * max(band[e], 4 * own[i, e])
    cerr = np.abs(og["conf"].astype(np.float64) - gg["conf"])
    row_band = np.maximum(band[left_at], 4 * own[np.arange(n), left_at]) if s.dtype == "bf16" else np.full(n, 1e-4)
    same_exit = og["layer"] == gg["layer"]
    conf_soft = same_exit & (cerr > row_band) & (cerr <= 4 * row_band)
    # hidden state where the row left the stack
    herr = np.abs(gg["h"].astype(np.float64) - og["h"]).max(1) / h_scale
    h_soft = same_exit & (herr > h_band) & (herr <= 4 * h_band)
    # A band permits a difference, it does not ask for one: a row inside a band that took the
    # oracle's decision stays in the comparison (and must then meet every check); a row is excluded
    # only where it used what its band permits.
    decided_other = ~same_exit | (og["breach"] != gg["breach"])
    tok_other = same_exit & (og["tok"] != gg["tok"])
    may_decide = noisy | unstable
    near = (may_decide & decided_other) | (tok_amb & tok_other) | conf_soft | h_soft
    near_now = near.copy()
    if sticky is not None:
        sticky |= near
        near = sticky.copy()
    ok = ~near
    bad = ok & (decided_other | tok_other)
    bad |= ok & (cerr > row_band)
    bad |= ok & (herr > h_band)
    # what the strict contract alone (1e-3 band, nothing else excluded) would report
    differs = decided_other | tok_other
    rep = dict(mismatch=int(bad.sum()), near=int(near.sum()), near_strict=int(strict.sum()), inside_band=int(may_decide.sum()),
               near_noise=int((may_decide & decided_other).sum()), near_token=int((tok_amb & tok_other).sum()),
               near_conf=int((conf_soft & ~decided_other).sum()), near_hidden=int((h_soft & ~conf_soft).sum()), h_band=h_band,
               rows=int(ok.sum()), band=band.tolist(),
               max_conf_err=float(cerr[ok].max()) if ok.any() else 0.0,
               max_h_err=float(herr[ok].max()) if ok.any() else 0.0,
               strict_only_differs=int((differs & ~strict).sum()), excluded_now=near_now, own=own, oracle=og, gpu=gg, gpu_all=ga)
    rep["detail"] = [dict(row=int(rows[i]), oracle=(int(og["tok"][i]), int(og["layer"][i]), float(og["conf"][i])),
                          gpu=(int(gg["tok"][i]), int(gg["layer"][i]), float(gg["conf"][i])), h_err=float(herr[i]),
                          trace=tr[i].tolist(), shadow_dev=own[i].tolist()) for i in np.nonzero(bad)[0][:8]]
    assert np.array_equal(gg["pos"], o.pos), "positions diverged"
    if n == s.batch and not near.any() and not bad.any():
        assert np.array_equal(gg["tok_in"], og["tok"])
    return rep


def report_line(step, rep):
    return (f"  step {step}: compared {rep['rows']} rows, mismatch {rep['mismatch']}; {rep['inside_band']} rows inside a "
            f"decision band ({rep['near_strict']} inside 1e-3); excluded now: decided otherwise inside a band "
            f"{rep['near_noise']}, token between near-equal candidates {rep['near_token']}, confidence beyond its band "
            f"{rep['near_conf']}, hidden state beyond its band {rep['near_hidden']} (confidence bands "
            f"{['%.1e' % x for x in rep['band']]}, hidden band {rep['h_band']:.1e}); "
            f"under the 1e-3 band alone {rep['strict_only_differs']} rows would differ; max conf err "
            f"{rep['max_conf_err']:.2e}, max hidden err {rep['max_h_err']:.2e}; exits "
            f"{np.bincount(rep['oracle']['layer'])[1:].tolist()}")
