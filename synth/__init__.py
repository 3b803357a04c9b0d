"""Seeded synthetic inputs for the early-exit decode step.

This module only *draws inputs* (weights, cached keys/values, tokens, context
lengths, per-row logit scales) and names the workload shapes.  It holds none of
the decode step's arithmetic and is the one piece of code that both the GPU
library's callers and the CPU oracle's callers use, so that both sides see the
same bytes.

Recipe (stands in for the trained early-exit checkpoints and request traces the
paper evaluates on, which are not available here):
  * every weight matrix, the embedding and every exit head: i.i.d. N(0, 0.02^2),
    stored row-major [out_features][in_features]; RMSNorm gains are 1;
  * cached context: K and V entries i.i.d. N(0, (0.02*sqrt(d))^2), which is the
    distribution a unit-RMS input has after an N(0, 0.02^2) projection;
  * context length per row: integer-uniform (inclusive) in the workload's range;
  * first input token per row: uniform over the vocabulary;
  * per-row logit scale ("temperature"): log-uniform in [0.5, 50], one draw per
    (row, decode step), so that the largest softmax probability of a
    random-init exit head spreads over roughly 0.01 .. 0.99.
Each tensor has its own counter-based stream keyed by (seed, tensor name), so a
tensor's values do not depend on which other tensors were drawn before it.
"""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
import hashlib
import os

import numpy as np

__all__ = ["Shape", "CONFIGS", "stream", "normal", "to_bf16_bits", "bf16_bits_to_f32",
           "layer_weights", "exit_weights", "embedding", "context_lengths", "kv_rows",
           "first_tokens", "row_scale", "capacity_for"]


@dataclass(frozen=True)
class Shape:
    name: str
    n_layers: int            # L, depth of the full model
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    exit_layers: tuple       # 1-based layers that carry an exit head
    dtype: str               # "f32" or "bf16"
    resident: int            # R: layers 1..R are loaded
    thresholds: tuple        # one per resident exit
    batch: int
    ctx_lo: int
    ctx_hi: int
    steps: int
    seed: int = 0
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5
    log_scale_shift: float = 0.0   # added to ln(scale)

    @property
    def resident_exits(self):
        return tuple(l for l in self.exit_layers if l <= self.resident)

    @property
    def qkv_rows(self):
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    def layer_params(self):
        d, F = self.d_model, self.d_ffn
        return self.qkv_rows * d + d * self.n_q_heads * self.head_dim + 3 * d * F

    def with_(self, **kw):
        return replace(self, **kw)


# The five workloads (shapes of the model families the paper serves: Llama2-7B,
# CodeLlama-34B, Llama2-70B; Tables "Overview of models" / "Summary of Models").
CONFIGS = {
    "tiny_f32": Shape("tiny_f32", 4, 256, 4, 4, 64, 688, 2048, (2, 4), "f32", 4, (0.8, 0.8),
                      batch=8, ctx_lo=64, ctx_hi=64, steps=1),
    "llama2_7b": Shape("llama2_7b", 32, 4096, 32, 32, 128, 11008, 32000, (8, 16, 24, 32), "bf16", 32,
                       (0.9, 0.85, 0.8, 0.0), batch=64, ctx_lo=128, ctx_hi=1024, steps=64),
    "codellama_34b_r32": Shape("codellama_34b_r32", 48, 8192, 64, 8, 128, 22016, 32000,
                               (8, 16, 24, 32, 40, 48), "bf16", 32, (0.8, 0.8, 0.8, 0.8),
                               batch=128, ctx_lo=256, ctx_hi=2048, steps=32),
    "llama2_70b": Shape("llama2_70b", 80, 8192, 64, 8, 128, 28672, 32000, (20, 40, 60, 80), "bf16", 80,
                        (0.9, 0.85, 0.8, 0.0), batch=256, ctx_lo=512, ctx_hi=2048, steps=16),
    "switch_7b_a": Shape("switch_7b_a", 32, 4096, 32, 32, 128, 11008, 32000, (10, 20, 32), "bf16", 20,
                         (0.8, 0.8), batch=512, ctx_lo=128, ctx_hi=1024, steps=32, seed=0,
                         log_scale_shift=+0.5),
    "switch_7b_b": Shape("switch_7b_b", 32, 4096, 32, 32, 128, 11008, 32000, (10, 20, 32), "bf16", 20,
                         (0.8, 0.8), batch=512, ctx_lo=128, ctx_hi=1024, steps=32, seed=1,
                         log_scale_shift=-0.5),
}


def stream(seed, name):
    """Counter-based generator for one named tensor."""
    digest = hashlib.blake2b(f"{seed}/{name}".encode(), digest_size=16).digest()
    key = int.from_bytes(digest[:8], "little")
    ctr = int.from_bytes(digest[8:], "little")
    return np.random.Generator(np.random.Philox(key=key, counter=ctr))


def to_bf16_bits(x):
    """fp32 -> bfloat16 storage (round to nearest even), as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


_CHUNK = 1 << 22      # values per independently seeded piece of a tensor


def _workers():
    n = int(os.environ.get("OMP_NUM_THREADS", 0) or os.cpu_count() or 1)
    return max(1, min(16, n))


def normal(seed, name, shape, std, dtype):
    """N(0, std^2) tensor in the storage type of the model: float32 for "f32",
    bfloat16 bit patterns (uint16) for "bf16".  The tensor is drawn in pieces of
    _CHUNK values (flat, row-major order), piece k from the stream (seed,
    "name#k"), so the values do not depend on how many threads draw them."""
    n = int(np.prod(shape))
    out = np.empty(n, np.uint16 if dtype == "bf16" else np.float32)

    def piece(k):
        lo, hi = k * _CHUNK, min(n, (k + 1) * _CHUNK)
        x = stream(seed, f"{name}#{k}").standard_normal(size=hi - lo, dtype=np.float32)
        x *= np.float32(std)
        out[lo:hi] = to_bf16_bits(x) if dtype == "bf16" else x

    n_pieces = (n + _CHUNK - 1) // _CHUNK
    if n_pieces <= 1:
        for k in range(n_pieces):
            piece(k)
    else:
        with ThreadPoolExecutor(_workers()) as pool:
            list(pool.map(piece, range(n_pieces)))
    return out.reshape(shape)


def layer_weights(s: Shape, layer: int, std=0.02):
    """Weights of decoder layer `layer` (1-based), row-major [out][in].
    W_qkv rows: H_q*hd query rows, then H_kv*hd key rows, then H_kv*hd value rows."""
    d, F, qd = s.d_model, s.d_ffn, s.n_q_heads * s.head_dim
    t = f"layer{layer}"
    return dict(
        g_attn=np.ones(d, np.float32),
        W_qkv=normal(s.seed, f"{t}.W_qkv", (s.qkv_rows, d), std, s.dtype),
        W_o=normal(s.seed, f"{t}.W_o", (d, qd), std, s.dtype),
        g_ffn=np.ones(d, np.float32),
        W_gate=normal(s.seed, f"{t}.W_gate", (F, d), std, s.dtype),
        W_up=normal(s.seed, f"{t}.W_up", (F, d), std, s.dtype),
        W_down=normal(s.seed, f"{t}.W_down", (d, F), std, s.dtype),
    )


def exit_weights(s: Shape, exit_idx: int, std=0.02):
    return dict(g=np.ones(s.d_model, np.float32),
                W=normal(s.seed, f"exit{exit_idx}.W", (s.vocab, s.d_model), std, s.dtype))


def embedding(s: Shape, std=0.02):
    return normal(s.seed, "embed", (s.vocab, s.d_model), std, s.dtype)


def context_lengths(s: Shape, batch=None):
    B = s.batch if batch is None else batch
    g = stream(s.seed, "ctx")
    return g.integers(s.ctx_lo, s.ctx_hi + 1, size=B, dtype=np.int64).astype(np.int32)


def capacity_for(ctx, steps, multiple=32):
    """Cache capacity (positions) of a row: its context plus the tokens it will
    decode, rounded up to a multiple."""
    need = np.asarray(ctx, dtype=np.int64) + steps
    return (((need + multiple - 1) // multiple) * multiple).astype(np.int32)


def kv_rows(s: Shape, layer: int, row: int, n_pos: int):
    """Cached context of one (layer, row): K and V, each [H_kv][n_pos][hd], in the
    model's storage type."""
    std = 0.02 * float(np.sqrt(s.d_model))
    shp = (s.n_kv_heads, n_pos, s.head_dim)
    K = normal(s.seed, f"kv.K.{layer}.{row}", shp, std, s.dtype)
    V = normal(s.seed, f"kv.V.{layer}.{row}", shp, std, s.dtype)
    return K, V


def first_tokens(s: Shape, batch=None):
    B = s.batch if batch is None else batch
    g = stream(s.seed, "tok0")
    return g.integers(0, s.vocab, size=B, dtype=np.int64).astype(np.int32)


def row_scale(s: Shape, step: int, batch=None, lo=0.5, hi=50.0):
    """Per-row multiplier of the exit-head logits for decode step `step`."""
    B = s.batch if batch is None else batch
    g = stream(s.seed, f"scale.{step}")
    u = g.random(size=B, dtype=np.float64)
    ln = np.log(lo) + u * (np.log(hi) - np.log(lo)) + s.log_scale_shift
    return np.exp(ln).astype(np.float32)


def context_tokens(s: Shape, row: int, n: int):
    """Token ids of the first n context positions of a row (uniform over the vocabulary)."""
    g = stream(s.seed, f"ctx.tok.{row}")
    return g.integers(0, s.vocab, size=n, dtype=np.int64).astype(np.int32)
