"""A decode step (and a speculative round) recorded once into a HIP graph and replayed.

Every call of the step is enqueue-only, takes its counts from device memory and allocates nothing, so a
caller may record it on a capturing stream and replay the graph once per token.  Each replay is the
next step (the step itself advances positions and input tokens on the device), so n replays must give
the bits of n eager steps on a twin with the same seeded state: outputs of every replay, and the cache
at the end.  Between replays the program does eager work of its own and synchronises, the way a serving
loop would.
"""
import numpy as np
import pytest
import torch

import synth
from parity import GpuSide
from paper_2504_10724_amd import session as S

pytestmark = pytest.mark.gpu

TINY = synth.CONFIGS["tiny_f32"]
MID = synth.CONFIGS["llama2_7b"].with_(name="mid_bf16_graph", n_layers=6, resident=6, d_model=1024, n_q_heads=8,
                                       n_kv_heads=2, d_ffn=2816, vocab=8192, exit_layers=(2, 4, 6),
                                       thresholds=(0.9, 0.8, 0.0), batch=72, ctx_lo=20, ctx_hi=330, steps=6)
FIELDS = ("out_tok", "out_layer", "out_conf", "out_breach", "h", "pos", "tok_in", "exit_counts", "breach_count")


def _say(msg):
    print(msg, flush=True)


def _snapshot(batch):
    return {k: batch.field(k).clone() for k in FIELDS}


def _same_cache(g1, g2, n_new):
    s = g1.s
    for b in (0, s.batch // 2, s.batch - 1):
        for l in range(1, s.resident + 1):
            K1, V1 = g1.kv.read_context(l, b, int(g1.ctx[b]) + n_new)
            K2, V2 = g2.kv.read_context(l, b, int(g2.ctx[b]) + n_new)
            assert np.array_equal(K1, K2) and np.array_equal(V1, V2), (b, l)


@pytest.mark.parametrize("s", [TINY, MID], ids=lambda s: s.name)
def test_decode_step_replayed_from_a_graph(s):
    n = min(5, s.steps)
    _say(f"[case] graph replay of ee_decode_step {s.name} B={s.batch}, {n} replays")
    g1, g2 = GpuSide(s), GpuSide(s)
    for g in (g1, g2):
        g.batch.set_row_scale(synth.row_scale(s, 0))       # spreads the confidences, so rows leave at several exits
    th = list(s.thresholds)
    want = []
    for t in range(n):
        assert S.decode_step(g1.model, g1.kv, g1.batch, th) == 0
        torch.cuda.synchronize()
        want.append(_snapshot(g1.batch))
    left_at = np.unique(np.concatenate([w["out_layer"].cpu().numpy() for w in want]))
    _say(f"  rows left at layers {left_at.tolist()}")
    assert left_at.size > 1, "every row left at the same layer: the case would not show a compaction"

    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            assert S.decode_step(g2.model, g2.kv, g2.batch, th) == 0
    torch.cuda.synchronize()
    # recording runs nothing: the twin still stands before its first step
    assert torch.equal(g2.batch.field("pos").cpu(), torch.as_tensor(g2.ctx.astype(np.int32)))
    scratch = torch.zeros(1 << 20, device="cuda")
    for t in range(n):
        graph.replay()
        torch.cuda.synchronize()
        got = _snapshot(g2.batch)
        for k in FIELDS:
            assert torch.equal(got[k], want[t][k]), (t, k)
        # the program's own eager work between two replays
        scratch.add_(1.0)
        assert float(scratch.sum().cpu()) == float(scratch.numel() * (t + 1))
    assert int(g2.batch.field("status").cpu()[0]) == 0
    _same_cache(g1, g2, n)


def test_speculative_round_replayed_from_a_graph():
    s = MID.with_(name="mid_bf16_graph_spec", thresholds=(2.0, 2.0, 2.0), batch=20, ctx_hi=200, steps=16)
    k, rounds = 3, 3
    _say(f"[case] graph replay of a speculative round {s.name} B={s.batch} k={k}, {rounds} replays")
    g1, g2 = GpuSide(s), GpuSide(s)
    sp1 = S.Speculator(g1.model, g1.kv, g1.batch, 0, k)
    sp2 = S.Speculator(g2.model, g2.kv, g2.batch, 0, k)
    want = []
    for r in range(rounds):
        sp1.round()
        torch.cuda.synchronize()
        want.append((sp1.drafts.clone(), sp1.n_emit.clone(), sp1.emit.clone(), g1.batch.field("pos").clone(),
                     g1.batch.field("tok_in").clone()))
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sp2.round()
    torch.cuda.synchronize()
    for r in range(rounds):
        graph.replay()
        torch.cuda.synchronize()
        got = (sp2.drafts, sp2.n_emit, sp2.emit, g2.batch.field("pos"), g2.batch.field("tok_in"))
        for a, b in zip(got, want[r]):
            assert torch.equal(a, b), r
        assert float(torch.ones(4096, device="cuda").sum().cpu()) == 4096.0
    assert int(g2.batch.field("status").cpu()[0]) == 0 and int(sp2.entries.field("status").cpu()[0]) == 0
