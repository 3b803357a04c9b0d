"""Degenerate cases of the exit head on the GPU that the oracle pins on the CPU: logits that are
bit-equal (the lowest index wins, wherever the two columns sit in the kernel's tiling) and a
confidence that equals the threshold exactly (">=": the row leaves).  Through the C ABI."""
import numpy as np
import pytest
import torch

import synth
from oracle import ee_oracle as orc
from helpers import OracleSide
from parity import GpuSide
from paper_2504_10724_amd import session as S

pytestmark = pytest.mark.gpu

# one 256-row tile kernel launch with a ragged tail; vocabulary spanning many 128- and 256-column tiles
TIES = synth.CONFIGS["llama2_7b"].with_(name="ties_bf16", n_layers=1, resident=1, d_model=512, n_q_heads=4,
                                        n_kv_heads=4, d_ffn=1024, vocab=4096, exit_layers=(1,),
                                        thresholds=(0.0,), batch=40, ctx_lo=1, ctx_hi=20, steps=1)
TIES_F32 = synth.CONFIGS["tiny_f32"].with_(name="ties_f32", batch=8)
# where the copy of the winning column goes, relative to the winner t (all inside the vocabulary):
# same lane and register run, other half-wave of the same 32-column tile, other tile of the same wave,
# other wave, other 128-column workgroup, other 256-column workgroup, far away; both directions
OFFSETS = [1, 4, 32, 64, 128, 256, 1777, -1, -4, -32, -64, -128, -256, -1777]


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("s", [TIES, TIES_F32], ids=lambda s: s.name)
def test_bit_equal_logits_give_the_lowest_index(s):
    _say(f"[case] argmax ties {s.name} B={s.batch} V={s.vocab}")
    o = OracleSide(s, gain_jitter=0.1)
    B, V = s.batch, s.vocab
    scale = synth.row_scale(s, 0)
    h = np.stack([orc.embed(o.model, t) for t in o.tok]).astype(np.float32)
    W = o.weights["exits"][0]["W"]                      # [V][d], storage type of the model
    # each row's own winner, then a copy of that weight row somewhere else: two bit-equal logits
    # that are the row's maximum.  Rows are handled one after the other so that a later copy
    # cannot destroy an earlier row's pair; a row whose pair cannot be kept is left without one.
    want_pair = {}
    taken = set()
    for b in range(B):
        _, t, _ = orc.exit_head(o.model, 0, h[b], float(scale[b]))
        off = OFFSETS[b % len(OFFSETS)]
        t2 = t + off
        if not (0 <= t2 < V) or t in taken or t2 in taken:
            continue
        W[t2] = W[t]
        taken |= {t, t2}
        want_pair[b] = (min(t, t2), max(t, t2))
    assert len(want_pair) >= B // 2
    conf_o, tok_o = np.zeros(B, np.float32), np.zeros(B, np.int32)
    for b in range(B):
        conf_o[b], tok_o[b], z = orc.exit_head(o.model, 0, h[b], float(scale[b]), want_logits=True)
        if b in want_pair and tok_o[b] in want_pair[b]:
            lo, hi = want_pair[b]
            assert z[lo] == z[hi] == z.max() and tok_o[b] == lo          # the oracle's own rule
    tied = [b for b in want_pair if tok_o[b] == want_pair[b][0]]
    assert len(tied) >= B // 3, "too few rows kept their pair as the maximum"
    g = GpuSide(s, weights=o.weights)
    f = g.batch.field
    g.batch.set_row_scale(scale)
    g.batch.begin_step()
    logits = torch.zeros((B, V), dtype=torch.float32, device="cuda")
    assert S.exit_head(g.model, 0, 0.5, 0, g.batch, logits) == 0
    torch.cuda.synchronize()
    tok_g, conf_g = f("head_tok").cpu().numpy(), f("head_conf").cpu().numpy()
    z_g = logits.cpu().numpy()
    for b in tied:
        lo, hi = want_pair[b]
        assert z_g[b, lo] == z_g[b, hi], f"row {b}: the two columns are not bit-equal on the GPU"
        assert tok_g[b] == lo, f"row {b}: token {tok_g[b]}, tie between {lo} and {hi} (offset {hi - lo})"
        assert conf_g[b] <= 0.5 + 1e-6
    assert np.array_equal(tok_g, tok_o), "tokens differ"
    assert np.abs(conf_g - conf_o).max() <= 1e-3
    _say(f"  {len(tied)} rows with a bit-equal maximum, offsets {sorted(set(want_pair[b][1] - want_pair[b][0] for b in tied))}: "
         f"lowest index on every one; all {B} tokens equal the oracle's")


@pytest.mark.parametrize("s", [TIES.with_(name="flat_bf16", vocab=2048), TIES_F32.with_(name="flat_f32")], ids=lambda s: s.name)
def test_confidence_equal_to_the_threshold_leaves(s):
    """All logits equal: confidence = 1/V exactly (V a power of two) and token 0 on both sides.  A
    threshold of exactly 1/V is met, the next float above it is not."""
    _say(f"[case] confidence == threshold {s.name} V={s.vocab}")
    o = OracleSide(s, gain_jitter=0.0)
    o.weights["exits"][0]["W"][:] = 0
    B, V = s.batch, s.vocab
    h = np.stack([orc.embed(o.model, t) for t in o.tok]).astype(np.float32)
    c, t, _ = orc.exit_head(o.model, 0, h[0], 3.0)
    th = np.float32(1.0) / np.float32(V)
    assert c == th and t == 0
    g = GpuSide(s, weights=o.weights)
    f = g.batch.field
    g.batch.set_row_scale(synth.row_scale(s, 0))
    above = np.nextafter(th, np.float32(1.0), dtype=np.float32)
    for thr, leaves in ((th, 1), (above, 0)):
        g.batch.begin_step()
        assert S.exit_head(g.model, 0, float(thr), 0, g.batch) == 0
        torch.cuda.synchronize()
        assert np.all(f("head_conf").cpu().numpy() == th), "confidence is not exactly 1/V"
        assert np.all(f("head_tok").cpu().numpy() == 0)
        assert np.all(f("head_exit").cpu().numpy() == leaves), f"threshold {thr!r}"
        assert not f("head_breach").cpu().numpy().any()
    # forced at the last resident layer below the threshold: leaves, and is a breach
    g.batch.begin_step()
    assert S.exit_head(g.model, 0, float(above), 1, g.batch) == 0
    torch.cuda.synchronize()
    assert np.all(f("head_exit").cpu().numpy() == 1) and np.all(f("head_breach").cpu().numpy() == 1)
    _say(f"  1/V = {th!r}: meets itself, does not meet {above!r}")
