"""ctypes binding of the CPU oracle.  TEST INFRASTRUCTURE ONLY: imported by
tests/, by the smoke check and by the benchmark's cpu_baseline leg, never by
the product package."""
import ctypes as C
import os

import numpy as np

from . import build as _build

ORC_F32, ORC_BF16 = 0, 1
ORC_OK, ORC_ERR_ARG, ORC_ERR_NOT_RESIDENT = 0, -1, -2


class OrcConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("dtype", C.c_int32), ("rms_eps", C.c_float),
                ("n_exits", C.c_int32), ("exit_layers", C.c_int32 * 16)]


class OrcKV(C.Structure):
    _fields_ = [("K", C.c_void_p), ("V", C.c_void_p), ("B", C.c_int32), ("cap", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        _lib = C.CDLL(path)
        _lib.orc_silu.restype = C.c_float
        _lib.orc_silu.argtypes = [C.c_float]
        _lib.orc_model_destroy.restype = None
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


class OracleModel:
    """Holds an orc_model and keeps the numpy arrays it points to alive."""

    def __init__(self, *, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab,
                 dtype, exit_layers, rms_eps=1e-5):
        cfg = OrcConfig()
        cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads = n_layers, d_model, n_q_heads, n_kv_heads
        cfg.head_dim, cfg.d_ffn, cfg.vocab = head_dim, d_ffn, vocab
        cfg.dtype = ORC_BF16 if dtype in ("bf16", ORC_BF16) else ORC_F32
        cfg.rms_eps = rms_eps
        cfg.n_exits = len(exit_layers)
        for i, l in enumerate(exit_layers):
            cfg.exit_layers[i] = l
        self.cfg = cfg
        self.dtype = cfg.dtype
        self.exit_layers = list(exit_layers)
        self._keep = []
        h = C.c_void_p()
        rc = lib().orc_model_create(C.byref(cfg), C.byref(h))
        if rc != ORC_OK:
            raise ValueError(f"orc_model_create failed: {rc}")
        self.h = h

    def __del__(self):
        try:
            if getattr(self, "h", None):
                lib().orc_model_destroy(self.h)
                self.h = None
        except Exception:   # interpreter shutdown
            pass

    def _w(self, a):
        want = np.uint16 if self.dtype == ORC_BF16 else np.float32
        a = np.ascontiguousarray(a)
        assert a.dtype == want, (a.dtype, want)
        self._keep.append(a)
        return _p(a)

    def _g(self, a):
        a = _f32(a)
        self._keep.append(a)
        return _p(a)

    def set_layer(self, layer, g_attn, W_qkv, W_o, g_ffn, W_gate, W_up, W_down):
        return lib().orc_model_set_layer(self.h, layer, self._g(g_attn), self._w(W_qkv), self._w(W_o),
                                         self._g(g_ffn), self._w(W_gate), self._w(W_up), self._w(W_down))

    def set_exit(self, e, g, W):
        return lib().orc_model_set_exit(self.h, e, self._g(g), self._w(W))

    def set_embed(self, emb):
        return lib().orc_model_set_embed(self.h, self._w(emb))

    def set_rope(self, theta, max_pos):
        return lib().orc_model_set_rope(self.h, C.c_double(theta), int(max_pos))

    def resident_depth(self):
        return lib().orc_model_resident_depth(self.h)


class OracleKV:
    """Dense fp32 cache: K, V [R][B][H_kv][cap][hd]."""

    def __init__(self, R, B, n_kv_heads, cap, head_dim):
        self.K = np.zeros((R, B, n_kv_heads, cap, head_dim), dtype=np.float32)
        self.V = np.zeros_like(self.K)
        self.B, self.cap = B, cap

    def struct(self):
        s = OrcKV()
        s.K, s.V, s.B, s.cap = self.K.ctypes.data, self.V.ctypes.data, self.B, self.cap
        return s


# ---------------------------------------------------------------- primitives

def round_bf16(x):
    x = _f32(x).copy()
    lib().orc_round_bf16(_p(x), C.c_size_t(x.size))
    return x


def rmsnorm(h, g, eps=1e-5, round_to_bf16=False):
    h, g = _f32(h), _f32(g)
    out = np.empty_like(h)
    lib().orc_rmsnorm(_p(h), _p(g), h.size, C.c_float(eps), int(round_to_bf16), _p(out))
    return out


def matvec(x, W):
    x = _f32(x)
    W = np.ascontiguousarray(W)
    dt = ORC_BF16 if W.dtype == np.uint16 else ORC_F32
    out = np.empty(W.shape[0], dtype=np.float32)
    lib().orc_matvec(_p(x), _p(W), dt, W.shape[0], W.shape[1], _p(out))
    return out


def rope(v, pos, theta=10000.0):
    v = _f32(v).copy()
    lib().orc_rope(_p(v), v.size, int(pos), C.c_double(theta))
    return v


def attention_head(q, K, V):
    q, K, V = _f32(q), _f32(K), _f32(V)
    out = np.empty_like(q)
    lib().orc_attention_head(_p(q), _p(K), _p(V), K.shape[0], q.size, _p(out))
    return out


def silu(t):
    return float(lib().orc_silu(C.c_float(t)))


def softmax_conf(z):
    z = _f32(z)
    conf, tok = C.c_float(), C.c_int32()
    lib().orc_softmax_conf(_p(z), z.size, C.byref(conf), C.byref(tok))
    return conf.value, tok.value


def compact(exit_mask, active):
    m = np.ascontiguousarray(exit_mask, dtype=np.uint8)
    a = np.ascontiguousarray(active, dtype=np.int32)
    n = a.size
    oa, oe = np.empty(n, np.int32), np.empty(n, np.int32)
    on, om = C.c_int32(), C.c_int32()
    lib().orc_compact(_p(m), _p(a), n, _p(oa), C.byref(on), _p(oe), C.byref(om))
    return oa[:on.value].copy(), oe[:om.value].copy()


# ------------------------------------------------------------ calls of the path

def embed(model, tok):
    h = np.empty(model.cfg.d_model, np.float32)
    rc = lib().orc_embed(model.h, int(tok), _p(h))
    if rc != ORC_OK:
        raise ValueError(rc)
    return h


def layer_forward(model, layer, kv, active, pos, h):
    """h [B][d] float32 is updated in place."""
    assert h.dtype == np.float32 and h.flags.c_contiguous
    a = np.ascontiguousarray(active, dtype=np.uint8)
    p = np.ascontiguousarray(pos, dtype=np.int32)
    s = kv.struct()
    return lib().orc_layer_forward(model.h, layer, C.byref(s), _p(a), _p(p), _p(h))


def exit_head(model, e, h_row, scale=1.0, want_logits=False):
    h_row = _f32(h_row)
    logits = np.empty(model.cfg.vocab, np.float32) if want_logits else None
    conf, tok = C.c_float(), C.c_int32()
    rc = lib().orc_exit_head(model.h, e, _p(h_row), C.c_float(scale), _p(logits), C.byref(conf), C.byref(tok))
    if rc != ORC_OK:
        raise ValueError(rc)
    return conf.value, tok.value, logits


def fill_skipped_kv(model, from_excl, to_incl, kv, b, pos_b, h_row):
    h_row = _f32(h_row)
    s = kv.struct()
    return lib().orc_fill_skipped_kv(model.h, from_excl, to_incl, C.byref(s), b, int(pos_b), _p(h_row))


def decode_step(model, kv, tok_in, pos, scale, thresholds, want_h=False):
    """pos (int32 array) is advanced in place.  Returns a dict."""
    B = kv.B
    tok_in = np.ascontiguousarray(tok_in, dtype=np.int32)
    assert pos.dtype == np.int32 and pos.flags.c_contiguous
    sc = None if scale is None else _f32(scale)
    th = _f32(thresholds)
    out_tok = np.full(B, -1, np.int32)
    out_layer = np.zeros(B, np.int32)
    out_conf = np.zeros(B, np.float32)
    out_breach = np.zeros(B, np.uint8)
    counts = np.zeros(16, np.int32)
    layers_run = C.c_int64(0)
    h_out = np.zeros((B, model.cfg.d_model), np.float32) if want_h else None
    trace = np.full((B, model.cfg.n_exits), np.nan, np.float32)
    s = kv.struct()
    rc = lib().orc_decode_step(model.h, C.byref(s), _p(tok_in), _p(pos), _p(sc), _p(th), th.size,
                               _p(out_tok), _p(out_layer), _p(out_conf), _p(out_breach), _p(counts),
                               C.byref(layers_run), _p(h_out), _p(trace))
    return dict(rc=rc, tok=out_tok, layer=out_layer, conf=out_conf, breach=out_breach,
                counts=counts, layers_run=layers_run.value, h=h_out, conf_trace=trace)


def vanilla_step(model, kv, tok_in, pos, scale, want_h=False):
    B = kv.B
    tok_in = np.ascontiguousarray(tok_in, dtype=np.int32)
    assert pos.dtype == np.int32 and pos.flags.c_contiguous
    sc = None if scale is None else _f32(scale)
    out_tok = np.full(B, -1, np.int32)
    out_conf = np.zeros(B, np.float32)
    h_out = np.zeros((B, model.cfg.d_model), np.float32) if want_h else None
    s = kv.struct()
    rc = lib().orc_vanilla_step(model.h, C.byref(s), _p(tok_in), _p(pos), _p(sc), _p(out_tok),
                                _p(out_conf), _p(h_out))
    return dict(rc=rc, tok=out_tok, conf=out_conf, h=h_out)


def prefill(model, kv, b, tokens, pos0=0, want_h=False):
    """Context pass of row b: tokens take positions pos0 .. pos0+n-1; K, V of every resident
    layer are appended.  Returns (rc, hidden states after the last resident layer or None)."""
    tok = np.ascontiguousarray(tokens, dtype=np.int32)
    h = np.zeros((tok.size, model.cfg.d_model), np.float32) if want_h else None
    s = kv.struct()
    rc = lib().orc_prefill(model.h, C.byref(s), int(b), _p(tok), tok.size, int(pos0), _p(h))
    return rc, h


def backfill_kv(model, kv, from_excl, to_incl, exit_states):
    """Keys and values of newly resident layers (from_excl, to_incl] for tokens that are cached
    already (Sec. 3.3.3: more layers of the current model are loaded while it serves; Sec. 2.2:
    every layer needs the keys and values of every earlier token).  exit_states maps
    (row, position) to the hidden state the token had where it left the layer stack; a layer
    it did not run leaves that state unchanged, so each new layer takes its K, V from it,
    exactly as orc_fill_skipped_kv does inside a decode step."""
    for (b, p), h in exit_states.items():
        rc = fill_skipped_kv(model, from_excl, to_incl, kv, b, p, h)
        if rc != ORC_OK:
            return rc
    return ORC_OK


def accept_drafts(drafts, verified):
    d = np.ascontiguousarray(drafts, dtype=np.int32)
    v = np.ascontiguousarray(verified, dtype=np.int32)
    out = np.zeros(d.size, np.int32)
    n = lib().orc_accept_drafts(_p(d), _p(v), d.size, _p(out))
    return out[:n].copy()


def selfspec_round(model, kv, b, tok_in, pos, draft_exit, k):
    """One self-speculative round of row b (Sec. 6; see ee_oracle.h).  Returns a dict with the
    drafts, the full-depth tokens of the same positions, the emitted tokens and the new position."""
    drafts, verified, emitted = np.zeros(k, np.int32), np.zeros(k, np.int32), np.zeros(k, np.int32)
    dm, vm = np.zeros(k, np.float32), np.zeros(k, np.float32)
    n, p = C.c_int32(), C.c_int32(int(pos))
    s = kv.struct()
    rc = lib().orc_selfspec_round(model.h, C.byref(s), int(b), int(tok_in), C.byref(p), int(draft_exit), int(k),
                                  _p(drafts), _p(verified), C.byref(n), _p(emitted), _p(dm), _p(vm))
    return dict(rc=rc, drafts=drafts, verified=verified, emitted=emitted[:n.value].copy(), pos=p.value,
                draft_margin=dm, verify_margin=vm)
