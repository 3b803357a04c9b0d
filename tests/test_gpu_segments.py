"""The decode step in pieces (ee_decode_segment, ee_decode_finish) against ee_decode_step, through the C ABI.

A caller with one or a few requests in the batch looks at n_active after every exit and ends the step
as soon as no row is left; the layers that no row reaches are then never launched.  Whatever the point
at which it ends, outputs, batch state and every layer's cache entries must be those of ee_decode_step
bit for bit (the step itself is compared with the oracle elsewhere): the rows that left get the keys and
values of the layers that were not run from ee_decode_finish in one go instead of exit by exit.
"""
import ctypes as C

import numpy as np
import pytest
import torch

import synth
from parity import GpuSide
from paper_2504_10724_amd import capi as ee
from paper_2504_10724_amd import session as S

pytestmark = pytest.mark.gpu

FIELDS = ("out_tok", "out_layer", "out_conf", "out_breach", "h", "pos", "tok_in", "exit_counts", "breach_count",
          "n_active", "status")
TINY = synth.CONFIGS["tiny_f32"].with_(name="tiny_f32_seg", n_layers=6, resident=6, exit_layers=(2, 4, 6),
                                       thresholds=(0.8, 0.8, 0.0), batch=5, ctx_lo=4, ctx_hi=40, steps=6)
SMALL = synth.CONFIGS["llama2_7b"].with_(name="small_bf16_seg", n_layers=8, resident=8, d_model=1024, n_q_heads=8,
                                         n_kv_heads=2, d_ffn=2816, vocab=8192, exit_layers=(2, 4, 6, 8),
                                         thresholds=(0.6, 0.5, 0.4, 0.0), batch=3, ctx_lo=20, ctx_hi=200, steps=8)
ONE = SMALL.with_(name="one_row_bf16_seg", batch=1)
# enough rows that some of them stay to the end in most steps, many layers per fill range
WIDE = synth.CONFIGS["llama2_7b"].with_(name="mid_bf16_seg", n_layers=12, resident=9, d_model=512, n_q_heads=8,
                                        n_kv_heads=8, d_ffn=1024, vocab=2048, exit_layers=(1, 5, 9, 12),
                                        thresholds=(0.7, 0.6, 0.0), batch=70, ctx_lo=5, ctx_hi=70, steps=4)


def _say(msg):
    print(msg, flush=True)


def _same_state(g1, g2, what):
    for k in FIELDS:
        assert torch.equal(g1.batch.field(k), g2.batch.field(k)), (what, k)


def _same_cache(g1, g2, n_new):
    s = g1.s
    for b in sorted({0, s.batch // 2, s.batch - 1}):
        for l in range(1, s.resident + 1):
            K1, V1 = g1.kv.read_context(l, b, int(g1.ctx[b]) + n_new)
            K2, V2 = g2.kv.read_context(l, b, int(g2.ctx[b]) + n_new)
            assert np.array_equal(K1, K2) and np.array_equal(V1, V2), (b, l)


@pytest.mark.parametrize("s", [TINY, SMALL, ONE, WIDE], ids=lambda s: s.name)
def test_step_in_segments_equals_the_step(s):
    _say(f"[case] segments {s.name} B={s.batch} exits {s.resident_exits}")
    g1, g2 = GpuSide(s), GpuSide(s)
    n_exits = len(s.resident_exits)
    ran = []
    plans = [list(s.thresholds)] * s.steps
    plans[1] = [0.0] * n_exits                           # every row leaves at the first exit: all deeper layers filled at once
    plans[2] = [2.0] * (n_exits - 1) + [0.0]             # no row leaves before the last resident layer: every segment runs
    plans[3] = [2.0] + [0.0] * (n_exits - 1)             # every row leaves at the second exit: the step ends midway
    for t, th in enumerate(plans):
        sc = synth.row_scale(s, t)
        for g in (g1, g2):
            g.batch.set_row_scale(sc)
        assert S.decode_step(g1.model, g1.kv, g1.batch, th) == 0
        ran.append(S.decode_step_checked(g2.model, g2.kv, g2.batch, th))
        torch.cuda.synchronize()
        _same_state(g1, g2, f"step {t}")
        assert int(g1.batch.field("status").cpu()[0]) == 0
    _say(f"  segments run per step: {ran} of {n_exits}")
    assert ran[1] == 1 and ran[2] == n_exits and ran[3] == 2
    _same_cache(g1, g2, len(plans))


def test_segment_calls_reject_bad_arguments():
    s = SMALL
    g = GpuSide(s)
    lib, th = g.model.lib, (C.c_float * 4)(0.5, 0.5, 0.5, 0.0)
    h = (g.model.h, g.kv.h, g.batch.h)
    assert lib.ee_decode_segment(*h, th, 4, 4, None) == ee.EE_ERR_INVALID_ARG
    assert lib.ee_decode_segment(*h, th, 4, -1, None) == ee.EE_ERR_INVALID_ARG
    assert lib.ee_decode_segment(*h, th, 3, 0, None) == ee.EE_ERR_INVALID_ARG          # one threshold per resident exit
    assert lib.ee_decode_segment(*h, None, 4, 0, None) == ee.EE_ERR_INVALID_ARG
    assert lib.ee_decode_segment(None, g.kv.h, g.batch.h, th, 4, 0, None) == ee.EE_ERR_INVALID_ARG
    assert lib.ee_decode_finish(*h, 4, None) == ee.EE_ERR_INVALID_ARG
    assert lib.ee_decode_finish(None, g.kv.h, g.batch.h, 0, None) == ee.EE_ERR_INVALID_ARG
    assert lib.ee_last_error() not in (None, b"")
