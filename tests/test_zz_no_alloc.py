"""ee_exit_head_static (the exit head on the library's own scratch array, for callers that cannot
allocate) against ee_exit_head, through the C ABI: same kernels, so every output must be bit-equal.
Two calls in a row on one GPU, the second with a smaller batch and model, so the second call finds
the first one's contents in the array."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth
from helpers import OracleSide
from parity import GpuSide
from paper_2504_10724_amd import capi as ee
from paper_2504_10724_amd import session as S

pytestmark = pytest.mark.gpu

BIG = synth.CONFIGS["llama2_7b"].with_(name="static_big", n_layers=2, resident=2, d_model=1024, n_q_heads=8,
                                       n_kv_heads=2, d_ffn=2816, vocab=8192, exit_layers=(1, 2),
                                       thresholds=(0.6, 0.0), batch=72, ctx_lo=20, ctx_hi=130, steps=1)
SMALL = synth.CONFIGS["llama2_7b"].with_(name="static_small", n_layers=2, resident=2, d_model=512, n_q_heads=4,
                                         n_kv_heads=4, d_ffn=1024, vocab=2048, exit_layers=(1, 2),
                                         thresholds=(0.7, 0.0), batch=19, ctx_lo=1, ctx_hi=97, steps=1)
TINY = synth.CONFIGS["tiny_f32"]
HEAD = ("head_conf", "head_tok", "head_exit", "head_breach")


def _both_heads(s, g, exit_idx, th, force):
    """the workspace call, then the static call, on the same batch state; returns both outputs"""
    f = g.batch.field
    n = int(f("n_active").cpu()[0])
    assert S.exit_head(g.model, exit_idx, th, force, g.batch) == 0
    torch.cuda.synchronize()
    want = {k: f(k).cpu().numpy()[:n].copy() for k in HEAD}
    for k in HEAD:
        f(k).zero_()
    assert S.exit_head_static(g.model, exit_idx, th, force, g.batch) == 0
    torch.cuda.synchronize()
    got = {k: f(k).cpu().numpy()[:n].copy() for k in HEAD}
    return n, want, got


def _prepare(s):
    o = OracleSide(s, gain_jitter=0.1)
    g = GpuSide(s, weights=o.weights)
    g.batch.set_row_scale(synth.row_scale(s, 0))
    g.batch.begin_step()
    assert S.layer_forward(g.model, 1, g.kv, g.batch) == 0
    return g


def test_static_exit_head_equals_the_workspace_exit_head_twice_in_a_row():
    print("[case] ee_exit_head_static vs ee_exit_head: big then small", flush=True)
    sides = [(s, _prepare(s)) for s in (BIG, SMALL, TINY)]
    for s, g in sides:                              # big first, then smaller ones: stale contents stay in the array
        n, want, got = _both_heads(s, g, 0, float(s.thresholds[0]), 0)
        assert n == s.batch
        for k in HEAD:
            assert np.array_equal(want[k], got[k]), (s.name, k)
        assert want["head_exit"].any() and not want["head_exit"].all(), "case must decide both ways"
        print(f"  {s.name}: {n} rows, all four outputs bit-equal", flush=True)
    # after a compaction the same batch has fewer active rows: smaller again, forced exit this time
    s, g = sides[0]
    assert S.compact_active(g.batch, 0, 1) == 0
    assert S.layer_forward(g.model, 2, g.kv, g.batch) == 0
    n, want, got = _both_heads(s, g, 1, 0.9, 1)
    assert 0 < n < s.batch
    for k in HEAD:
        assert np.array_equal(want[k], got[k]), k
    assert want["head_exit"].all() and want["head_breach"].any()
    print(f"  {s.name} after compaction: {n} rows, forced exit, bit-equal", flush=True)


def test_static_exit_head_rejects_what_does_not_fit_and_bad_arguments():
    lib = ee.load()
    assert lib.ee_exit_head_static(None, 0, 0.5, 0, None, None) == ee.EE_ERR_INVALID_ARG
    s = SMALL.with_(name="static_too_big", vocab=32000, batch=2048)
    m = S.Model.from_shape(s, max_pos=64)
    ones = torch.ones(s.d_model, dtype=torch.float32, device="cuda")
    w = torch.zeros((s.vocab, s.d_model), dtype=torch.bfloat16, device="cuda")
    m.set_exit_device(0, ones, w)
    b = S.Batch(m, s.batch)
    rc = S.exit_head_static(m, 0, 0.5, 0, b)
    assert rc == ee.EE_ERR_CAPACITY and b"scratch" in lib.ee_last_error()
    assert S.exit_head_static(m, 1, 0.5, 0, b) == ee.EE_ERR_EXIT_NOT_RESIDENT
    assert S.exit_head_static(m, 0, float("nan"), 0, b) == ee.EE_ERR_INVALID_ARG
    assert S.exit_head_static(m, 7, 0.5, 0, b) == ee.EE_ERR_INVALID_ARG
