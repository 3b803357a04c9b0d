"""Test-side glue: builds the CPU oracle's model / cache from the seeded
synthetic inputs.  Imports the oracle, so it is test infrastructure too."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import synth
from oracle import ee_oracle as orc


def draw_weights(s, n_distinct=None, std=0.02):
    """Weights of the resident layers, the resident exit heads and the embedding.  With
    n_distinct, only that many layers are drawn and layer l takes the tensors of drawn layer
    ((l - 1) mod n_distinct) + 1 (the same objects): a model of the workload's real depth and
    shapes whose host and device footprint stays small.  Both sides get the same dict."""
    n = s.resident if n_distinct is None else min(n_distinct, s.resident)
    base = {k: synth.layer_weights(s, k, std) for k in range(1, n + 1)}
    return {"layers": {l: base[(l - 1) % n + 1] for l in range(1, s.resident + 1)},
            "exits": {e: synth.exit_weights(s, e, std) for e, l in enumerate(s.exit_layers) if l <= s.resident},
            "embed": synth.embedding(s, std)}


def draw_contexts(s, rows):
    """Cached context {(layer, row): (K, V)} of the given rows in every resident layer, drawn by a
    thread pool (each (layer, row) has its own stream, so the order does not matter)."""
    ctx = synth.context_lengths(s)
    keys = [(l, int(b)) for l in range(1, s.resident + 1) for b in rows]
    with ThreadPoolExecutor(synth._workers()) as pool:
        vals = list(pool.map(lambda k: synth.kv_rows(s, k[0], k[1], int(ctx[k[1]])), keys))
    return dict(zip(keys, vals))


def small_shape(**kw):
    base = dict(name="small", n_layers=4, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8,
                d_ffn=48, vocab=64, exit_layers=(2, 4), dtype="f32", resident=4,
                thresholds=(0.8, 0.8), batch=5, ctx_lo=3, ctx_hi=9, steps=2, seed=0)
    base.update(kw)
    return synth.Shape(**base)


class OracleSide:
    """Oracle model + dense cache for rows `rows` (default: all) of a workload."""

    def __init__(self, s, rows=None, weights=None, std=0.02, cap=None, fill_ctx=True, gain_jitter=0.1,
                 contexts=None):
        self.s = s
        self.rows = list(range(s.batch)) if rows is None else list(rows)
        self.model = orc.OracleModel(n_layers=s.n_layers, d_model=s.d_model, n_q_heads=s.n_q_heads,
                                     n_kv_heads=s.n_kv_heads, head_dim=s.head_dim, d_ffn=s.d_ffn,
                                     vocab=s.vocab, dtype=s.dtype, exit_layers=s.exit_layers,
                                     rms_eps=s.rms_eps)
        self.weights = weights if weights is not None else {
            "layers": {l: synth.layer_weights(s, l, std) for l in range(1, s.resident + 1)},
            "exits": {e: synth.exit_weights(s, e, std) for e, l in enumerate(s.exit_layers) if l <= s.resident},
            "embed": synth.embedding(s, std),
        }
        if weights is None and gain_jitter:
            # the workloads use unit gains; the logic tests perturb them so that a
            # wrong or missing gain cannot go unnoticed
            g = synth.stream(s.seed, "test.gains")
            jit = lambda: (1 + gain_jitter * g.standard_normal(s.d_model)).astype(np.float32)
            for w in self.weights["layers"].values():
                w["g_attn"], w["g_ffn"] = jit(), jit()
            for w in self.weights["exits"].values():
                w["g"] = jit()
        for l, w in self.weights["layers"].items():
            assert self.model.set_layer(l, w["g_attn"], w["W_qkv"], w["W_o"], w["g_ffn"], w["W_gate"],
                                        w["W_up"], w["W_down"]) == 0
        for e, w in self.weights["exits"].items():
            assert self.model.set_exit(e, w["g"], w["W"]) == 0
        assert self.model.set_embed(self.weights["embed"]) == 0
        self.ctx_all = synth.context_lengths(s)
        self.ctx = self.ctx_all[self.rows].copy()
        self.cap = int(cap if cap is not None else (int(self.ctx_all.max()) + s.steps))
        assert self.model.set_rope(s.rope_theta, self.cap) == 0
        self.kv = orc.OracleKV(s.resident, len(self.rows), s.n_kv_heads, self.cap, s.head_dim)
        if fill_ctx:
            for l in range(1, s.resident + 1):
                for i, b in enumerate(self.rows):
                    K, V = contexts[(l, b)] if contexts is not None else synth.kv_rows(s, l, b, int(self.ctx_all[b]))
                    if s.dtype == "bf16":
                        K, V = synth.bf16_bits_to_f32(K), synth.bf16_bits_to_f32(V)
                    n = int(self.ctx_all[b])
                    self.kv.K[l - 1, i, :, :n, :] = K
                    self.kv.V[l - 1, i, :, :n, :] = V
        self.pos = self.ctx.astype(np.int32).copy()
        self.tok = synth.first_tokens(s)[self.rows].copy()

    def scale(self, step):
        return synth.row_scale(self.s, step)[self.rows].copy()

    def step(self, step_idx, thresholds=None, want_h=False, scale=None):
        th = self.s.thresholds if thresholds is None else thresholds
        sc = self.scale(step_idx) if scale is None else scale
        r = orc.decode_step(self.model, self.kv, self.tok, self.pos, sc, th, want_h=want_h)
        if r["rc"] == 0:
            self.tok = r["tok"].copy()
        return r


def f32w(w, dtype):
    """weights in fp64 regardless of storage type"""
    if dtype == "bf16":
        return synth.bf16_bits_to_f32(w).astype(np.float64)
    return np.asarray(w, dtype=np.float64)
