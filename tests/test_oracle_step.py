"""Pins of the CPU oracle's decode step: the special cases the paper fixes
(threshold 0, threshold above 1, greedy exit at the last resident layer), the
invariants of the method (keys/values for skipped layers, batch independence,
threshold monotonicity) and a brute-force fp64 recomputation on tiny inputs.
No GPU."""
import numpy as np
import pytest
import scipy.special

import synth
from oracle import ee_oracle as orc
from helpers import OracleSide, small_shape, f32w


# ------------------------------------------------------------------ brute force (fp64, numpy)
# Written independently of the oracle: whole-matrix numpy products, scipy's
# softmax, complex-number rotation for the rotary embedding.

def _rnd(x, bf):
    return synth.bf16_bits_to_f32(synth.to_bf16_bits(x.astype(np.float32))).astype(np.float64) if bf else x


def _norm(h, g, eps, bf):
    return _rnd(h / np.sqrt(np.mean(h * h) + eps) * g, bf)


def _rot(v, pos, hd, theta):
    half = hd // 2
    z = (v[:half] + 1j * v[half:]) * np.exp(1j * pos * theta ** (-2.0 * np.arange(half) / hd))
    return np.concatenate([z.real, z.imag])


def brute_step(s, W, Kc, Vc, tok, pos, scale, th):
    """Kc, Vc: dict (layer,row) -> list of per-position [H_kv][hd] arrays (fp64). Mutated."""
    bf = s.dtype == "bf16"
    d, hd, Hq, Hkv = s.d_model, s.head_dim, s.n_q_heads, s.n_kv_heads
    R = s.resident
    out = {}
    for b in range(len(tok)):
        h = f32w(W["embed"], s.dtype)[tok[b]].copy()
        done = False
        for l in range(1, R + 1):
            w = W["layers"][l]
            Wqkv = f32w(w["W_qkv"], s.dtype)
            if not done:
                x = _norm(h, w["g_attn"], s.rms_eps, bf)
                qkv = Wqkv @ x
                q = qkv[:Hq * hd].reshape(Hq, hd)
                k = qkv[Hq * hd:(Hq + Hkv) * hd].reshape(Hkv, hd)
                v = qkv[(Hq + Hkv) * hd:].reshape(Hkv, hd)
                k = np.stack([_rot(k[g], pos[b], hd, s.rope_theta) for g in range(Hkv)])
                Kc[(l, b)].append(_rnd(k, bf)); Vc[(l, b)].append(_rnd(v, bf))
                Ks, Vs = np.stack(Kc[(l, b)]), np.stack(Vc[(l, b)])   # [pos+1][Hkv][hd]
                o = np.zeros((Hq, hd))
                for i in range(Hq):
                    g = i // (Hq // Hkv)
                    qi = _rot(q[i], pos[b], hd, s.rope_theta)
                    p = scipy.special.softmax(Ks[:, g, :] @ qi / np.sqrt(hd))
                    o[i] = p @ Vs[:, g, :]
                h = h + f32w(w["W_o"], s.dtype) @ _rnd(o.reshape(-1), bf)
                y = _norm(h, w["g_ffn"], s.rms_eps, bf)
                gate, up = f32w(w["W_gate"], s.dtype) @ y, f32w(w["W_up"], s.dtype) @ y
                h = h + f32w(w["W_down"], s.dtype) @ _rnd(gate * scipy.special.expit(gate) * up, bf)
                if l in s.exit_layers:
                    e = s.exit_layers.index(l)
                    z = scale[b] * (f32w(W["exits"][e]["W"], s.dtype) @ _norm(h, W["exits"][e]["g"], s.rms_eps, bf))
                    p = scipy.special.softmax(z)
                    conf = p.max()
                    if conf >= th[e] or l == R:
                        out[b] = (int(np.argmax(z)), l, conf, int(l == R and conf < th[e]), h.copy())
                        done = True
            else:
                # skipped layer: key/value from the exit hidden state
                x = _norm(h, w["g_attn"], s.rms_eps, bf)
                qkv = Wqkv @ x
                k = qkv[Hq * hd:(Hq + Hkv) * hd].reshape(Hkv, hd)
                v = qkv[(Hq + Hkv) * hd:].reshape(Hkv, hd)
                k = np.stack([_rot(k[g], pos[b], hd, s.rope_theta) for g in range(Hkv)])
                Kc[(l, b)].append(_rnd(k, bf)); Vc[(l, b)].append(_rnd(v, bf))
    return out


def _brute_cache(side):
    s = side.s
    Kc, Vc = {}, {}
    for l in range(1, s.resident + 1):
        for i, b in enumerate(side.rows):
            n = int(side.ctx[i])
            Kc[(l, i)] = [side.kv.K[l - 1, i, :, t, :].astype(np.float64) for t in range(n)]
            Vc[(l, i)] = [side.kv.V[l - 1, i, :, t, :].astype(np.float64) for t in range(n)]
    return Kc, Vc


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_brute_force_two_steps(dtype):
    s = small_shape(dtype=dtype, n_layers=3, resident=3, exit_layers=(1, 3), thresholds=(0.3, 0.3),
                    d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=4, d_ffn=24, vocab=16, batch=4,
                    ctx_lo=2, ctx_hi=5)
    side = OracleSide(s, std=0.35)
    Kc, Vc = _brute_cache(side)
    tok = side.tok.copy()
    pos = side.pos.copy()
    layers_seen = set()
    for step in range(2):
        sc = side.scale(step)
        want = brute_step(s, side.weights, Kc, Vc, tok, pos, sc.astype(np.float64), s.thresholds)
        got = side.step(step, want_h=True)
        assert got["rc"] == 0
        for b in range(s.batch):
            wt, wl, wc, wb, wh = want[b]
            assert abs(wc - s.thresholds[s.exit_layers.index(wl)]) > 1e-3  # decision is not marginal
            assert (got["tok"][b], got["layer"][b], got["breach"][b]) == (wt, wl, wb)
            assert abs(got["conf"][b] - wc) < (1e-5 if dtype == "f32" else 2e-3)
            np.testing.assert_allclose(got["h"][b], wh, rtol=0, atol=(2e-5 if dtype == "f32" else 2e-2) * np.abs(wh).max())
            layers_seen.add(wl)
            # cache after the step: every resident layer holds pos+1 entries, equal to the brute force
            for l in range(1, s.resident + 1):
                n = pos[b] + 1
                np.testing.assert_allclose(side.kv.K[l - 1, b, :, :n, :], np.stack(Kc[(l, b)]).transpose(1, 0, 2),
                                           rtol=0, atol=(1e-5 if dtype == "f32" else 1.7e-2))
                np.testing.assert_allclose(side.kv.V[l - 1, b, :, :n, :], np.stack(Vc[(l, b)]).transpose(1, 0, 2),
                                           rtol=0, atol=(1e-5 if dtype == "f32" else 1.7e-2))
        tok = got["tok"].copy()
        pos = pos + 1
        assert np.array_equal(side.pos, pos)
    assert layers_seen == {1, 3}, "workload must exercise both exits"


# ------------------------------------------------------------------ special cases the paper fixes

def _mk(dtype="f32", **kw):
    s = small_shape(dtype=dtype, **kw)
    return s, OracleSide(s, std=0.3)


def test_threshold_zero_everyone_leaves_at_first_exit():
    # Sec. 3.1 (Insight 2): with the threshold at 0 every token takes the first exit
    s, side = _mk()
    r = side.step(0, thresholds=(0.0, 0.0))
    assert r["rc"] == 0
    assert np.all(r["layer"] == s.exit_layers[0]) and not r["breach"].any()
    assert r["counts"][0] == s.batch and r["counts"][1] == 0
    assert r["layers_run"] == s.batch * s.exit_layers[0]   # deeper layers were never executed


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_threshold_above_one_equals_vanilla_decoding(dtype):
    # Sec. 3.1: a threshold that no probability can meet keeps every token in
    # the stack => ordinary full-depth decoding, bit for bit (tokens, hidden
    # states and the whole cache)
    s, side = _mk(dtype)
    s2, van = _mk(dtype)
    assert np.array_equal(side.kv.K, van.kv.K)
    for step in range(2):
        sc = side.scale(step)
        r = side.step(step, thresholds=(2.0, 2.0), want_h=True)
        v = orc.vanilla_step(van.model, van.kv, van.tok, van.pos, sc, want_h=True)
        assert r["rc"] == 0 and v["rc"] == 0
        van.tok = v["tok"].copy()
        assert np.all(r["layer"] == s.resident) and r["breach"].all()
        assert np.array_equal(r["tok"], v["tok"])
        assert np.array_equal(r["conf"], v["conf"])
        assert np.array_equal(r["h"], v["h"])
        assert np.array_equal(side.kv.K, van.kv.K) and np.array_equal(side.kv.V, van.kv.V)
        assert np.array_equal(side.pos, van.pos)
        assert r["layers_run"] == s.batch * s.resident


def test_final_threshold_zero_never_breaches():
    s, side = _mk()
    r = side.step(0, thresholds=(2.0, 0.0))
    assert np.all(r["layer"] == s.resident) and not r["breach"].any()


def test_partial_residency_forces_exit_at_last_resident_layer():
    # Sec. 3.3.3 / Sec. 5.4: only layers 1..R are loaded; every token stops at R
    s = small_shape(n_layers=6, exit_layers=(2, 4, 6), resident=4, thresholds=(2.0, 2.0))
    side = OracleSide(s, std=0.3)
    assert side.model.resident_depth() == 4
    r = side.step(0)
    assert r["rc"] == 0 and np.all(r["layer"] == 4) and r["breach"].all()
    assert r["layers_run"] == s.batch * 4
    # the layers that were not loaded cannot be run
    h = np.zeros((s.batch, s.d_model), np.float32)
    assert orc.layer_forward(side.model, 5, side.kv, np.ones(s.batch), side.pos, h) == orc.ORC_ERR_NOT_RESIDENT
    # one threshold per resident exit
    assert side.step(1, thresholds=(0.5, 0.5, 0.5))["rc"] == orc.ORC_ERR_ARG
    assert side.step(1, thresholds=(np.nan, 0.5))["rc"] == orc.ORC_ERR_ARG


def test_deepest_resident_layer_must_be_an_exit():
    s = small_shape(n_layers=6, exit_layers=(2, 4, 6), resident=3, thresholds=(0.5,))
    side = OracleSide(s, std=0.3)
    assert side.step(0)["rc"] == orc.ORC_ERR_NOT_RESIDENT


def test_confidences_are_probabilities_and_spread():
    s = small_shape(batch=40, vocab=256, d_model=64, n_q_heads=4, n_kv_heads=4, head_dim=16)
    side = OracleSide(s)          # N(0, 0.02) weights as in the workloads
    r = side.step(0, thresholds=(0.0, 0.0))
    assert np.all(r["conf"] >= 1.0 / s.vocab - 1e-9) and np.all(r["conf"] <= 1.0)


# ------------------------------------------------------------------ invariants

def test_batch_independence_and_row_permutation():
    s, side = _mk(batch=6)
    r = side.step(0, want_h=True)
    for b in range(s.batch):
        one = OracleSide(s, rows=[b], weights=side.weights, cap=side.cap)
        rb = one.step(0, want_h=True)
        assert (rb["tok"][0], rb["layer"][0], rb["breach"][0]) == (r["tok"][b], r["layer"][b], r["breach"][b])
        assert rb["conf"][0] == r["conf"][b]
        assert np.array_equal(rb["h"][0], r["h"][b])
        assert np.array_equal(one.kv.K[:, 0], side.kv.K[:, b])
    perm = [3, 0, 5, 1, 4, 2]
    p = OracleSide(s, rows=perm, weights=side.weights, cap=side.cap)
    rp = p.step(0)
    assert np.array_equal(rp["tok"], r["tok"][perm]) and np.array_equal(rp["layer"], r["layer"][perm])


def test_no_holes_and_skipped_layer_kv_formula():
    # Sec. 2.2: keys/values exist for every layer, also the skipped ones.
    s, side = _mk("bf16", batch=6)
    s2, van = _mk("bf16", batch=6)
    before_K = side.kv.K.copy()
    r = side.step(0, want_h=True)
    sc = side.scale(0)
    orc.vanilla_step(van.model, van.kv, van.tok, van.pos, sc)
    assert len(set(r["layer"].tolist())) > 1, "need rows leaving at different exits"
    hd, Hq, Hkv = s.head_dim, s.n_q_heads, s.n_kv_heads
    for b in range(s.batch):
        p = int(side.ctx[b])
        for l in range(1, s.resident + 1):
            newK, newV = side.kv.K[l - 1, b, :, p, :], side.kv.V[l - 1, b, :, p, :]
            assert np.any(newK != 0) and np.any(newV != 0)                    # no hole
            assert np.array_equal(side.kv.K[l - 1, b, :, :p], before_K[l - 1, b, :, :p])  # history untouched
            assert not np.any(side.kv.K[l - 1, b, :, p + 1:])                 # nothing beyond
            if l <= r["layer"][b]:
                assert np.array_equal(newK, van.kv.K[l - 1, b, :, p, :])      # executed layers = vanilla
                assert np.array_equal(newV, van.kv.V[l - 1, b, :, p, :])
            else:
                w = side.weights["layers"][l]
                x = orc.rmsnorm(r["h"][b], w["g_attn"], s.rms_eps, round_to_bf16=True)
                kv = orc.matvec(x, w["W_qkv"][Hq * hd:])
                for g in range(Hkv):
                    k = orc.round_bf16(orc.rope(kv[g * hd:(g + 1) * hd], p, s.rope_theta))
                    v = orc.round_bf16(kv[(Hkv + g) * hd:(Hkv + g + 1) * hd])
                    assert np.array_equal(newK[g], k) and np.array_equal(newV[g], v)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fill_of_a_layer_range_equals_the_fills_of_its_parts(dtype):
    # Sec. 2.2: a skipped layer's key/value depends on the token's exit state, the layer and the
    # position only, so the layers of a range may be filled in any grouping and at any later time
    # within the step; a step that fills (exit layer, next exit layer] for all rows that have left
    # so far ends with the same cache as one that fills (exit layer, R] at every exit.
    s = small_shape(dtype=dtype, n_layers=6, resident=6, exit_layers=(1, 3, 6), thresholds=(0.8, 0.8, 0.8), batch=4)
    a, b2 = OracleSide(s, std=0.3), OracleSide(s, std=0.3)
    rng = np.random.default_rng(5)
    for b in range(s.batch):
        h = rng.standard_normal(s.d_model).astype(np.float32)
        p = int(a.ctx[b])
        assert orc.fill_skipped_kv(a.model, 1, 6, a.kv, b, p, h) == 0
        for lo, hi in ((3, 6), (1, 3)):                      # parts, deliberately out of order
            assert orc.fill_skipped_kv(b2.model, lo, hi, b2.kv, b, p, h) == 0
    assert np.array_equal(a.kv.K, b2.kv.K) and np.array_equal(a.kv.V, b2.kv.V)
    assert np.any(a.kv.K[5] != 0) and not np.any(a.kv.K[0, :, :, int(a.ctx.max()):])   # layer 1 untouched at the new positions


def test_identity_tail_makes_early_exit_equal_to_vanilla():
    # If the layers after the exit add nothing to the hidden state (W_o = W_d = 0)
    # then leaving at the exit and filling the skipped layers' keys/values from
    # the exit hidden state must reproduce full-depth decoding exactly.
    s = small_shape(exit_layers=(2, 4), batch=5)
    base = OracleSide(s, std=0.3)
    W = base.weights
    for l in (3, 4):
        W["layers"][l]["W_o"] = np.zeros_like(W["layers"][l]["W_o"])
        W["layers"][l]["W_down"] = np.zeros_like(W["layers"][l]["W_down"])
    W["exits"][1] = W["exits"][0]          # same head at the end
    early = OracleSide(s, weights=W)
    full = OracleSide(s, weights=W)
    sc = early.scale(0)
    r = early.step(0, thresholds=(0.0, 0.0), want_h=True)
    v = orc.vanilla_step(full.model, full.kv, full.tok, full.pos, sc, want_h=True)
    assert np.all(r["layer"] == 2)
    assert np.array_equal(r["tok"], v["tok"]) and np.array_equal(r["conf"], v["conf"])
    assert np.array_equal(r["h"], v["h"])
    assert np.array_equal(early.kv.K, full.kv.K) and np.array_equal(early.kv.V, full.kv.V)


def test_threshold_monotonicity():
    s = small_shape(batch=12, n_layers=6, exit_layers=(2, 4, 6), resident=6, thresholds=(0.5, 0.5, 0.5))
    prev = None
    W = None
    for th in [0.0, 0.05, 0.1, 0.2, 0.4, 0.7, 0.95, 1.5]:
        side = OracleSide(s, std=0.3, weights=W)
        W = side.weights
        r = side.step(0, thresholds=(th, th, th))
        if prev is not None:
            assert np.all(r["layer"] >= prev)   # raising the threshold never lets a row leave earlier
        prev = r["layer"].copy()
    assert prev.min() == 6


def test_exit_counts_and_layers_run_are_consistent():
    s, side = _mk(batch=10)
    r = side.step(0)
    for e, l in enumerate(s.exit_layers):
        assert r["counts"][e] == int(np.sum(r["layer"] == l))
    assert r["layers_run"] == int(r["layer"].sum())
    assert np.array_equal(r["breach"] == 1, (r["layer"] == s.resident) & (r["conf"] < s.thresholds[-1]))


def test_exit_head_call_matches_step_and_logits_scale():
    s, side = _mk(batch=4)
    r = side.step(0, thresholds=(0.0, 0.0), want_h=True)
    sc = side.scale(0)
    for b in range(s.batch):
        conf, tok, z = orc.exit_head(side.model, 0, r["h"][b], sc[b], want_logits=True)
        assert conf == r["conf"][b] and tok == r["tok"][b]
        _, _, z1 = orc.exit_head(side.model, 0, r["h"][b], 1.0, want_logits=True)
        np.testing.assert_array_equal(z, z1 * np.float32(sc[b]))
        assert abs(conf - scipy.special.softmax(z.astype(np.float64)).max()) < 1e-6


# ------------------------------------------------------------------ what the paper prints

def test_parameter_counts_against_printed_weight_footprints():
    """Table "Memory footprint ... for the ShareGPT dataset" prints the weight
    footprints of the model families whose shapes the workloads use."""
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "weights_footprint.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, gb = line.split()
                rows[name] = float(gb)
    for name, key in [("Llama2-7B", "llama2_7b"), ("CodeLlama-34B", "codellama_34b_r32"), ("Llama2-70B", "llama2_70b")]:
        s = synth.CONFIGS[key]
        params = s.n_layers * s.layer_params() + 2 * s.vocab * s.d_model   # layers + embedding + LM head
        gib = params * 2 / 2 ** 30
        assert abs(gib - rows[name]) / rows[name] < 0.04, (name, gib, rows[name])


def test_meets_means_greater_or_equal():
    # Sec. 2.1: a token leaves when its probability *meets* the threshold
    s, side = _mk(batch=4)
    r0 = side.step(0, thresholds=(0.0, 0.0))
    b = int(np.argmin(r0["conf"]))
    th = float(r0["conf"][b])                 # exactly this row's confidence at the first exit
    s2, again = _mk(batch=4)
    r = again.step(0, thresholds=(th, 0.0))
    assert r["layer"][b] == s.exit_layers[0] and r["conf"][b] == r0["conf"][b]
    s3, above = _mk(batch=4)
    r = above.step(0, thresholds=(float(np.nextafter(np.float32(th), np.float32(2))), 0.0))
    assert r["layer"][b] == s.exit_layers[1]


def test_bf16_contract_noise_floor_is_measurable_with_the_oracle_alone():
    """Two correct implementations of the bf16 contract that differ by one part in 10^6 in an fp32
    operand drift apart by bf16-sized amounts within a few layers; fp32 models do not.  This is what
    the whole-step GPU comparison allows for (and only that)."""
    from parity import shadow_of
    for dtype, lo, hi in (("bf16", 1e-4, 2e-2), ("f32", 0.0, 2e-5)):
        s = small_shape(dtype=dtype, n_layers=6, resident=6, exit_layers=(2, 4, 6), thresholds=(2.0, 2.0, 2.0),
                        d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=512, vocab=512, batch=12,
                        ctx_lo=10, ctx_hi=40)
        a = OracleSide(s, gain_jitter=0)
        b = shadow_of(a)
        sc = a.scale(0)
        ra = a.step(0, want_h=True, scale=sc)
        rb = b.step(0, want_h=True, scale=sc)
        err = np.abs(ra["h"] - rb["h"]).max(1) / np.abs(ra["h"]).max(1)
        assert lo <= err.max() <= hi, (dtype, err.max())
