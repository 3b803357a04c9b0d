"""GPU parity of the context pass (ee_prefill, through the C ABI) against the CPU
oracle's orc_prefill on the same seeded token streams.  Run with -m gpu on an MI355X.

Bars: fp32 models, cached K, V and hidden states within 2e-5 / 2e-4 (normwise per
cache row and layer / per entry); bf16 models within 2e-2, the bar of the decode
tests: a context pass chains the same bf16 operand roundings through the layers.
Decode steps that follow a context pass are compared as every other decode step
(bit-exact decisions outside the noise band a shadow oracle measures)."""
import numpy as np
import pytest
import torch

import synth
from oracle import ee_oracle as orc
from helpers import OracleSide
from parity import GpuSide, compare_step, shadow_of, rows_close, TOL
from paper_2504_10724_amd import capi as ee
from paper_2504_10724_amd import session as S

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


TINY = synth.CONFIGS["tiny_f32"].with_(name="tiny_f32_ctx", batch=7, ctx_lo=1, ctx_hi=40, steps=2)
MHA = synth.CONFIGS["llama2_7b"].with_(name="mha_bf16_ctx", n_layers=2, resident=2, d_model=512, n_q_heads=4,
                                       n_kv_heads=4, d_ffn=1024, vocab=2048, exit_layers=(1, 2),
                                       thresholds=(0.7, 0.0), batch=19, ctx_lo=1, ctx_hi=97, steps=2)
MID = synth.CONFIGS["llama2_7b"].with_(name="mid_bf16_ctx", n_layers=6, resident=6, d_model=1024, n_q_heads=8,
                                       n_kv_heads=2, d_ffn=2816, vocab=8192, exit_layers=(2, 4, 6),
                                       thresholds=(0.9, 0.8, 0.0), batch=20, ctx_lo=1, ctx_hi=140, steps=2)
# more entries per call than one 256-row group holds, one kv head shared by 8 query heads
WIDE = synth.CONFIGS["llama2_7b"].with_(name="wide_bf16_ctx", n_layers=2, resident=2, d_model=512, n_q_heads=8,
                                        n_kv_heads=1, d_ffn=1536, vocab=4096, exit_layers=(1, 2),
                                        thresholds=(0.8, 0.0), batch=40, ctx_lo=5, ctx_hi=70, steps=1)
# enough (kv head, entry) pairs per call that the attention kernel serves several entries per workgroup
# (shared K/V stream where they sit in the same cache row), G = 4 query heads per kv head: four entries
PAIRS = synth.CONFIGS["llama2_7b"].with_(name="pairs_bf16_ctx", n_layers=2, resident=2, d_model=512, n_q_heads=32,
                                         n_kv_heads=8, d_ffn=1024, vocab=2048, exit_layers=(1, 2),
                                         thresholds=(0.8, 0.0), batch=10, ctx_lo=1, ctx_hi=150, steps=1)
# G = 2 and G = 3 query heads per kv head: 8 and 5 entries per workgroup share a K/V stream (5 x 3 of the 16
# MFMA columns in use); contexts short enough that several cache rows meet inside one workgroup's entries
GQA2 = synth.CONFIGS["llama2_7b"].with_(name="gqa2_bf16_ctx", n_layers=2, resident=2, d_model=512, n_q_heads=8,
                                        n_kv_heads=4, d_ffn=1024, vocab=2048, exit_layers=(1, 2),
                                        thresholds=(0.8, 0.0), batch=14, ctx_lo=1, ctx_hi=60, steps=1)
GQA3 = GQA2.with_(name="gqa3_bf16_ctx", n_q_heads=6, n_kv_heads=2, d_model=768)
# partially loaded model: the pass stops at the last resident layer
PARTIAL = synth.CONFIGS["codellama_34b_r32"].with_(name="partial_bf16_ctx", n_layers=6, resident=4, d_model=512,
                                                   n_q_heads=8, n_kv_heads=1, d_ffn=1024, vocab=2048,
                                                   exit_layers=(2, 4, 6), thresholds=(0.8, 0.8), batch=12,
                                                   ctx_lo=3, ctx_hi=60, steps=1)


def _contexts(s, rows=None):
    ctx = synth.context_lengths(s)
    return {b: synth.context_tokens(s, b, int(ctx[b])) for b in (range(s.batch) if rows is None else rows)}


def _oracle_context_pass(o):
    """orc_prefill of every row the oracle side holds; returns the hidden states per row"""
    hs = {}
    for i, b in enumerate(o.rows):
        rc, h = orc.prefill(o.model, o.kv, i, synth.context_tokens(o.s, b, int(o.ctx_all[b])), want_h=True)
        assert rc == 0
        hs[b] = h
    return hs


def _gpu_context_pass(g, contexts, rows_per_call, check_h=None, tol=None):
    """ee_prefill in calls of rows_per_call entries; after each call the hidden states of its
    entries are compared with check_h[cache row][position] where given.  Returns the call count."""
    pb = S.Batch(g.model, rows_per_call)
    zero = np.zeros(rows_per_call, np.int32)
    pb.reset(zero, zero, None)                      # clears the status word
    calls = 0
    for tok, pos, seq in S.prefill_chunks(contexts, rows_per_call):
        rc = S.prefill(g.model, g.kv, pb, tok, pos, seq)
        torch.cuda.synchronize()
        assert rc == 0, ee.load().ee_last_error()
        assert int(pb.field("status").cpu()[0]) == 0
        assert int(pb.field("n_active").cpu()[0]) == len(tok)
        calls += 1
        if check_h is not None:
            h = pb.field("h").cpu().numpy()[:len(tok)]
            keep = [i for i in range(len(tok)) if int(seq[i]) in check_h]
            if keep:
                want = np.stack([check_h[int(seq[i])][int(pos[i])] for i in keep])
                worst, ok = rows_close(h[keep], want, tol)
                assert ok, f"hidden states after the last layer: worst entry error {worst:.2e}"
    pb.close()
    return calls


def _compare_cache(s, o, g, tol):
    worst = 0.0
    for i, b in enumerate(o.rows):
        n = int(o.ctx_all[b])
        for l in range(1, s.resident + 1):
            K, V = g.kv.read_context(l, b, int(g.cap[b]))
            wk, okk = rows_close(K[:, :n].reshape(1, -1), o.kv.K[l - 1, i, :, :n].reshape(1, -1), tol)
            wv, okv = rows_close(V[:, :n].reshape(1, -1), o.kv.V[l - 1, i, :, :n].reshape(1, -1), tol)
            assert okk and okv, (b, l, wk, wv)
            assert not K[:, n:].any() and not V[:, n:].any(), "positions beyond the context were written"
            worst = max(worst, wk, wv)
    return worst


@pytest.mark.parametrize("s,rows_per_call", [(TINY, 13), (MHA, 50), (MID, 72), (WIDE, 300), (PARTIAL, 33), (PAIRS, 72), (GQA2, 64),
                                             (GQA3, 47)],
                         ids=lambda v: v.name if hasattr(v, "name") else None)
def test_context_pass_cache_and_hidden_states(s, rows_per_call):
    _say(f"[case] context_pass {s.name} seed={s.seed} cache rows={s.batch} entries per call={rows_per_call}")
    o = OracleSide(s, fill_ctx=False, gain_jitter=0.1)
    hs = _oracle_context_pass(o)
    _say(f"  oracle pass done: {int(o.ctx_all.sum())} tokens")
    g = GpuSide(s, weights=o.weights, synth_rows=[])
    g.kv.pool.zero_()
    tol_h, tol_kv = (2e-4, 2e-5) if s.dtype == "f32" else (TOL["bf16"], TOL["bf16"])
    calls = _gpu_context_pass(g, _contexts(s), rows_per_call, check_h=hs, tol=tol_h)
    worst = _compare_cache(s, o, g, tol_kv)
    _say(f"  {calls} calls; worst cache error (normwise per row and layer) {worst:.2e}")
    assert calls >= 2, "the workload must split contexts over several calls"


@pytest.mark.parametrize("s,rows_per_call", [(TINY, 16), (MID, 96)], ids=lambda v: v.name if hasattr(v, "name") else None)
def test_decode_steps_after_a_context_pass(s, rows_per_call):
    """The cache the decode step reads was built by ee_prefill / orc_prefill instead of being
    synthetic: time to first token = context pass + first decode step."""
    _say(f"[case] decode_after_context_pass {s.name} seed={s.seed} B={s.batch}")
    o = OracleSide(s, fill_ctx=False, gain_jitter=0.0)
    _oracle_context_pass(o)
    shadow = None
    if s.dtype == "bf16":
        shadow = shadow_of(o)
        shadow.kv.K[:] = 0
        shadow.kv.V[:] = 0
        _oracle_context_pass(shadow)
    g = GpuSide(s, weights=o.weights, synth_rows=[])
    g.kv.pool.zero_()
    _gpu_context_pass(g, _contexts(s), rows_per_call)
    g.batch.reset(synth.first_tokens(s), g.ctx.astype(np.int32), None)
    sticky = np.zeros(s.batch, bool)
    for step in range(s.steps):
        rep = compare_step(s, o, g, step, sticky=sticky, shadow=shadow)
        _say(f"  step {step}: compared {rep['rows']} rows, mismatch {rep['mismatch']}, near {rep['near']} "
             f"(bands {['%.1e' % x for x in rep['band']]}); max conf err {rep['max_conf_err']:.2e}; "
             f"exits {np.bincount(rep['oracle']['layer'])[1:].tolist()}")
        assert rep["mismatch"] == 0, rep["detail"]
    assert sticky.sum() <= max(3, s.batch * s.steps // 10), f"{sticky.sum()} of {s.batch} rows excluded"


@pytest.mark.parametrize("entries,ctx_hi", [(256, 12), (1024, 40)], ids=["one_row_group", "four_row_groups"])
def test_full_width_context_pass_sampled_cache_rows(entries, ctx_hi):
    """The 70B workload's layer shapes on a two-layer model: 256 entries per call (the decode
    benchmark's row count, so the same tile variants and grids) and 1024 entries per call (four
    256-row groups of a column tile on one XCD, the launch shape of the benchmark's context pass);
    64 short contexts, of which the oracle recomputes a sample from their first token on."""
    base = synth.CONFIGS["llama2_70b"]
    s = base.with_(name=f"70b_shape_ctx_{entries}", n_layers=2, resident=2, exit_layers=(1, 2), thresholds=(0.9, 0.0),
                   batch=64, ctx_lo=1, ctx_hi=ctx_hi, steps=1)
    rows = [0, 29, 63]
    _say(f"[case] full-width context pass {s.name} cache rows={s.batch} entries per call={entries} sampled={rows}")
    o = OracleSide(s, rows=rows, fill_ctx=False, gain_jitter=0.0)
    hs = _oracle_context_pass(o)
    _say("  oracle side ready")
    g = GpuSide(s, weights=o.weights, synth_rows=[])
    g.kv.pool.zero_()
    calls = _gpu_context_pass(g, _contexts(s), entries, check_h=hs, tol=TOL["bf16"])
    worst = _compare_cache(s, o, g, TOL["bf16"])
    _say(f"  {calls} calls, {int(g.ctx.sum())} entries; worst sampled cache error {worst:.2e}")
    if entries > 256:
        assert int(g.ctx.sum()) > 768, "a call must fill more than three row groups"
    # every cache row, at any size: exactly its context was written, nothing beyond
    for b in range(s.batch):
        K, V = g.kv.read_context(2, b, int(g.cap[b]))
        n = int(g.ctx[b])
        assert K[:, :n].any(axis=(0, 2)).all() and V[:, :n].any(axis=(0, 2)).all()
        assert not K[:, n:].any() and not V[:, n:].any()


def test_context_pass_refusals():
    s = TINY
    _say(f"[case] context_pass_refusals {s.name}")
    o = OracleSide(s, fill_ctx=False, gain_jitter=0.0)
    g = GpuSide(s, weights=o.weights, synth_rows=[])
    g.kv.pool.zero_()
    lib = ee.load()
    pb = S.Batch(g.model, 8)
    z8 = np.zeros(8, np.int32)
    pb.reset(z8, z8, None)
    status = lambda: int(pb.field("status").cpu()[0])
    # more entries than the batch has rows
    nine = np.zeros(9, np.int32)
    assert S.prefill(g.model, g.kv, pb, nine, np.arange(9, dtype=np.int32), nine) == ee.EE_ERR_CAPACITY
    # no entries: nothing to do
    e0 = np.zeros(0, np.int32)
    assert lib.ee_prefill(g.model.h, g.kv.h, pb.h, None, None, None, 0, None) == 0
    # a cache row that does not exist, a position beyond the capacity: refused in the status word,
    # the other entries of the call are served, nothing is written for the refused ones
    cap0 = int(g.cap[0])
    tok = np.array([3, 4, 5, 6], np.int32)
    assert S.prefill(g.model, g.kv, pb, tok, np.array([0, 0, cap0, 1], np.int32),
                     np.array([0, s.batch, 0, 0], np.int32)) == 0
    torch.cuda.synchronize()
    assert status() == 1
    K, _ = g.kv.read_context(1, 0, cap0)
    assert K[:, 0].any() and K[:, 1].any() and not K[:, 2:].any()
    pb.reset(z8, z8, None)
    assert S.prefill(g.model, g.kv, pb, np.array([s.vocab], np.int32), np.array([2], np.int32),
                     np.array([1], np.int32)) == 0
    torch.cuda.synchronize()
    assert status() == 2
    # a cache bound for fewer layers than are resident
    small = S.KVCache(g.model, s.resident - 1, g.cap)
    assert S.prefill(g.model, small, pb, tok, np.arange(4, dtype=np.int32), np.zeros(4, np.int32)) == ee.EE_ERR_CAPACITY
    # a batch bound to another model
    g2 = GpuSide(s, weights=o.weights, synth_rows=[])
    assert S.prefill(g2.model, g2.kv, pb, tok, np.arange(4, dtype=np.int32), np.zeros(4, np.int32)) == ee.EE_ERR_INVALID_ARG
