"""GPU-vs-oracle comparison helpers (test infrastructure).

Per call (same inputs on both sides): exit masks, tokens, breach flags and
compaction indices bit-exact, except rows whose oracle confidence lies within
NEAR = 1e-3 of the threshold, which are counted separately.  Hidden states and
logits: per row, max |gpu - oracle| <= tol * max |oracle| with tol = 2e-2 for
bf16 models and 2e-4 for fp32 models.

Whole decode steps run both sides freely through several layers.  Under the
bf16 contract every matrix-product operand is rounded to bfloat16, and a chain
of such roundings turns a difference of one fp32 ulp (a different summation
order) into differences of bf16 size within a few layers, in the oracle as in
any other implementation.  The step comparison therefore measures that noise
with the oracle itself: a second oracle whose fp32 RMSNorm gains are perturbed
by one part in 10^6 runs beside the first, and the largest confidence change it
shows at an exit widens that exit's band (never below 1e-3).  Rows inside a band
are "near"; rows within the 1e-3 band are also counted on their own.  Every
other row must match bit-exactly on exit layer, token and breach flag.
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

    def __init__(self, s, weights=None, std=0.02, cap_multiple=32, max_pos=None, synth_rows=None):
        """synth_rows: if given, only these rows get their cached context from the seeded host
        generator (the rows an oracle will recompute); the others are filled on the device from
        the same distribution, which is much faster for large batches."""
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
        for l, w in weights["layers"].items():
            self.model.set_layer(l, **w)
        for e, w in weights["exits"].items():
            self.model.set_exit(e, **w)
        self.model.set_embed(weights["embed"])
        self.kv = S.KVCache(self.model, s.resident, self.cap)
        if synth_rows is not None:
            gen = torch.Generator(device="cuda")
            gen.manual_seed(s.seed + 1)
            pool = self.kv.pool.view(torch.bfloat16 if s.dtype == "bf16" else torch.float32)
            pool.normal_(0.0, 0.02 * float(np.sqrt(s.d_model)), generator=gen)
        for l in range(1, s.resident + 1):
            for b in (range(s.batch) if synth_rows is None else synth_rows):
                K, V = synth.kv_rows(s, l, b, int(self.ctx[b]))
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
                    tok_in=f("tok_in").cpu().numpy())


def shadow_of(o, rel=1e-6, seed=7):
    """A second oracle on the same workload whose fp32 norm gains differ by `rel`
    (relative): the probe of how far the precision contract's own rounding
    lets two correct implementations drift apart."""
    s = o.s
    rng = np.random.default_rng(seed)
    w2 = {"layers": {l: dict(w) for l, w in o.weights["layers"].items()},
          "exits": o.weights["exits"], "embed": o.weights["embed"]}
    for w in w2["layers"].values():
        for k in ("g_attn", "g_ffn"):
            w[k] = (w[k].astype(np.float64) * (1 + rel * rng.standard_normal(s.d_model))).astype(np.float32)
    return OracleSide(s, rows=o.rows, weights=w2, cap=o.cap, gain_jitter=0)


def compare_step(s, o, g, step_idx, thresholds=None, sticky=None, shadow=None):
    """Runs decode step `step_idx` on the oracle, on the GPU and (if given) on the
    shadow oracle, and classifies every row.  `sticky`: rows already excluded."""
    th = np.asarray(s.thresholds if thresholds is None else thresholds, np.float32)
    sc = o.scale(step_idx)
    if shadow is not None:
        shadow.tok = o.tok.copy()          # the probe follows the oracle's token stream
    og = o.step(step_idx, thresholds=th, want_h=True, scale=sc)
    gg = g.step(step_idx, thresholds=th, scale=sc)
    assert og["rc"] == 0 and gg["rc"] == 0, (og["rc"], gg["rc"])
    assert gg["status"] == 0, f"device status {gg['status']}"
    B = s.batch
    res_exits = s.resident_exits
    tr = og["conf_trace"]
    band = np.full(len(res_exits), NEAR, np.float64)
    unstable = np.zeros(B, bool)
    if shadow is not None:
        sg = shadow.step(step_idx, thresholds=th, scale=sc)
        assert sg["rc"] == 0
        unstable |= (sg["tok"] != og["tok"]) | (sg["layer"] != og["layer"])
        for e in range(len(res_exits)):
            both = np.isfinite(tr[:, e]) & np.isfinite(sg["conf_trace"][:, e])
            if both.any():
                band[e] = max(NEAR, float(np.abs(tr[both, e] - sg["conf_trace"][both, e]).max()))
    strict = np.zeros(B, bool)
    noisy = np.zeros(B, bool)
    for e in range(len(res_exits)):
        if not (0.0 < th[e] <= 1.0):
            continue   # a threshold <= 0 is always met and one above 1 never: nothing to decide
        c = tr[:, e]
        reached = np.isfinite(c)
        strict |= reached & (np.abs(c - th[e]) <= NEAR)
        noisy |= reached & (np.abs(c - th[e]) <= band[e])
    # a different token is tolerated only where the oracle's own top candidates are closer than
    # the noise allows (one probability may fall by the band while the other rises by it):
    # p_oracle(tok_oracle) - p_oracle(tok_gpu) <= 2 * band at the exit the row left
    tok_amb = np.zeros(B, bool)
    for b in np.nonzero((og["tok"] != gg["tok"]) & (og["layer"] == gg["layer"]))[0]:
        e = res_exits.index(int(og["layer"][b]))
        _, _, z = orc.exit_head(o.model, s.exit_layers.index(res_exits[e]), og["h"][b], float(sc[b]), want_logits=True)
        p = np.exp(z.astype(np.float64) - z.max()); p /= p.sum()
        tok_amb[b] = (p.max() - p[gg["tok"][b]]) <= 2 * band[e]
    near = noisy | unstable | tok_amb
    if sticky is not None:
        sticky |= near
        near = sticky.copy()
    ok = ~near
    bad = ok & ((og["tok"] != gg["tok"]) | (og["layer"] != gg["layer"]) | (og["breach"] != gg["breach"]))
    conf_tol = 1e-4 if s.dtype == "f32" else max(5e-3, 4 * float(band.max()))
    cerr = np.abs(og["conf"] - gg["conf"])
    bad |= ok & (cerr > conf_tol)
    rep = dict(mismatch=int(bad.sum()), near=int(near.sum()), near_strict=int(strict.sum()),
               near_noise=int((noisy & ~strict).sum()), near_unstable=int((unstable & ~noisy).sum()),
               near_token=int((tok_amb & ~noisy & ~unstable).sum()), rows=int(ok.sum()), band=band.tolist(),
               max_conf_err=float(cerr[ok].max()) if ok.any() else 0.0, oracle=og, gpu=gg)
    rep["detail"] = [dict(row=int(b), oracle=(int(og["tok"][b]), int(og["layer"][b]), float(og["conf"][b])),
                          gpu=(int(gg["tok"][b]), int(gg["layer"][b]), float(gg["conf"][b])),
                          trace=tr[b].tolist()) for b in np.nonzero(bad)[0][:8]]
    assert np.array_equal(gg["pos"], o.pos), "positions diverged"
    if not near.any() and not bad.any():
        assert np.array_equal(gg["tok_in"], og["tok"])
    return rep
