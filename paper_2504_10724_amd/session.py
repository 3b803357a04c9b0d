"""Device-memory plumbing around libee: PyTorch allocates the buffers and
provides the stream, libee does all the work.  Nothing here computes anything
on the decode path."""
import ctypes as C

import numpy as np
import torch

from . import capi as ee


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def _to_device(a, dtype):
    """numpy (float32, or uint16 bf16 bit patterns) or torch tensor -> device tensor in the model dtype"""
    if isinstance(a, torch.Tensor):
        t = a
    else:
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            t = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16)
        else:
            t = torch.from_numpy(a)
    t = t.to("cuda", non_blocking=False).contiguous()
    assert t.dtype == dtype, (t.dtype, dtype)
    return t


class Model:
    """An early-exit decoder description plus the device tensors its resident layers use."""

    def __init__(self, *, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, dtype,
                 exit_layers, max_pos, rms_eps=1e-5, rope_theta=10000.0):
        if not torch.cuda.is_available():
            raise RuntimeError("libee needs a HIP device; there is no CPU path")
        self.lib = ee.load()
        cfg = ee.ee_model_config()
        cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads = n_layers, d_model, n_q_heads, n_kv_heads
        cfg.head_dim, cfg.d_ffn, cfg.vocab = head_dim, d_ffn, vocab
        cfg.dtype = ee.EE_BF16 if dtype == "bf16" else ee.EE_F32
        cfg.rms_eps, cfg.rope_theta, cfg.max_pos = rms_eps, rope_theta, max_pos
        cfg.n_exits = len(exit_layers)
        for i, l in enumerate(exit_layers):
            cfg.exit_layers[i] = l
        self.cfg = cfg
        self.bf16 = cfg.dtype == ee.EE_BF16
        self.tdtype = torch.bfloat16 if self.bf16 else torch.float32
        self.exit_layers = list(exit_layers)
        self.h = C.c_void_p()
        ee.check(self.lib.ee_model_create(C.byref(cfg), C.byref(self.h)))
        self._keep = {}

    @classmethod
    def from_shape(cls, s, max_pos):
        return cls(n_layers=s.n_layers, d_model=s.d_model, n_q_heads=s.n_q_heads, n_kv_heads=s.n_kv_heads,
                   head_dim=s.head_dim, d_ffn=s.d_ffn, vocab=s.vocab, dtype=s.dtype,
                   exit_layers=s.exit_layers, max_pos=max_pos, rms_eps=s.rms_eps, rope_theta=s.rope_theta)

    def close(self):
        if self.h:
            self.lib.ee_model_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights --------------------------------------------------------------
    def _matrix(self, W):
        """row-major [out][in] -> device tensor in the form the kernels read"""
        t = _to_device(W, self.tdtype)
        if not self.bf16:
            return t
        out = torch.empty_like(t)
        ee.check(self.lib.ee_pack_weight(_ptr(t), t.shape[0], t.shape[1], _ptr(out), 0, 1, t.shape[0], _stream()))
        torch.cuda.current_stream().synchronize()
        return out

    def _gate_up(self, Wg, Wu):
        g, u = _to_device(Wg, self.tdtype), _to_device(Wu, self.tdtype)
        if not self.bf16:
            return torch.cat([g, u], dim=0).contiguous()
        out = torch.empty((2 * g.shape[0], g.shape[1]), dtype=self.tdtype, device="cuda")
        ee.check(self.lib.ee_pack_weight(_ptr(g), g.shape[0], g.shape[1], _ptr(out), 0, 2, 2 * g.shape[0], _stream()))
        ee.check(self.lib.ee_pack_weight(_ptr(u), u.shape[0], u.shape[1], _ptr(out), 1, 2, 2 * g.shape[0], _stream()))
        torch.cuda.current_stream().synchronize()
        return out

    def set_layer(self, layer, *, g_attn, W_qkv, W_o, g_ffn, W_gate, W_up, W_down):
        t = dict(g_attn=_to_device(g_attn, torch.float32), w_qkv=self._matrix(W_qkv), w_o=self._matrix(W_o),
                 g_ffn=_to_device(g_ffn, torch.float32), w_gate_up=self._gate_up(W_gate, W_up),
                 w_down=self._matrix(W_down))
        self.set_layer_device(layer, **t)

    def set_layer_device(self, layer, *, g_attn, w_qkv, w_o, g_ffn, w_gate_up, w_down):
        """device tensors already in the kernels' format"""
        w = ee.ee_layer_weights(_ptr(g_attn), _ptr(w_qkv), _ptr(w_o), _ptr(g_ffn), _ptr(w_gate_up), _ptr(w_down))
        ee.check(self.lib.ee_model_set_layer(self.h, layer, C.byref(w)))
        self._keep[("layer", layer)] = (g_attn, w_qkv, w_o, g_ffn, w_gate_up, w_down)

    def set_exit(self, e, *, g, W):
        gt, wt = _to_device(g, torch.float32), self._matrix(W)
        self.set_exit_device(e, gt, wt)

    def set_exit_device(self, e, g, w):
        ee.check(self.lib.ee_model_set_exit(self.h, e, _ptr(g), _ptr(w)))
        self._keep[("exit", e)] = (g, w)

    def set_embed(self, emb):
        t = _to_device(emb, self.tdtype)
        ee.check(self.lib.ee_model_set_embed(self.h, _ptr(t)))
        self._keep["embed"] = t

    def resident_depth(self):
        return self.lib.ee_model_resident_depth(self.h)


class KVCache:
    def __init__(self, model, n_layers, capacity):
        self.model = model
        cap = np.ascontiguousarray(capacity, dtype=np.int32)
        self.capacity = cap
        self.B = int(cap.size)
        self.n_layers = n_layers
        capp = cap.ctypes.data_as(C.POINTER(C.c_int32))
        nbytes = model.lib.ee_kv_pool_bytes(model.h, n_layers, capp, self.B)
        if nbytes == 0:
            raise ee.EEError(ee.EE_ERR_CAPACITY, "invalid key/value pool description")
        self.pool = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.h = C.c_void_p()
        ee.check(model.lib.ee_kv_bind(model.h, _ptr(self.pool), nbytes, n_layers, capp, self.B, C.byref(self.h)))

    def close(self):
        if self.h:
            self.model.lib.ee_kv_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def write_context(self, layer, row, K, V, pos0=0):
        """K, V: [H_kv][n_pos][hd] in the model dtype (numpy or torch)"""
        k, v = _to_device(K, self.model.tdtype), _to_device(V, self.model.tdtype)
        ee.check(self.model.lib.ee_kv_write_context(self.model.h, self.h, layer, row, pos0, k.shape[1],
                                                    _ptr(k), _ptr(v), _stream()))
        torch.cuda.current_stream().synchronize()

    def read_context(self, layer, row, n_pos, pos0=0):
        c = self.model.cfg
        k = torch.empty((c.n_kv_heads, n_pos, c.head_dim), dtype=self.model.tdtype, device="cuda")
        v = torch.empty_like(k)
        ee.check(self.model.lib.ee_kv_read_context(self.model.h, self.h, layer, row, pos0, n_pos, _ptr(k), _ptr(v),
                                                   _stream()))
        torch.cuda.current_stream().synchronize()
        return k.float().cpu().numpy(), v.float().cpu().numpy()


_FIELD_TYPES = dict(h=torch.float32, tok_in=torch.int32, pos=torch.int32, row_scale=torch.float32,
                    active_idx=torch.int32, n_active=torch.int32, exited_idx=torch.int32, n_exited=torch.int32,
                    head_conf=torch.float32, head_tok=torch.int32, head_exit=torch.uint8, head_breach=torch.uint8,
                    out_tok=torch.int32, out_layer=torch.int32, out_conf=torch.float32, out_breach=torch.uint8,
                    exit_counts=torch.int32, breach_count=torch.int32, status=torch.int32)


class Batch:
    def __init__(self, model, B):
        self.model, self.B = model, B
        lib = model.lib
        sb, wb = lib.ee_batch_state_bytes(model.h, B), lib.ee_workspace_bytes(model.h, B)
        self.state = torch.zeros(sb, dtype=torch.uint8, device="cuda")
        self.workspace = torch.empty(wb, dtype=torch.uint8, device="cuda")
        self.h = C.c_void_p()
        ee.check(lib.ee_batch_bind(model.h, B, _ptr(self.state), sb, _ptr(self.workspace), wb, C.byref(self.h)))
        self.layout = ee.ee_batch_layout()
        ee.check(lib.ee_batch_get_layout(model.h, B, C.byref(self.layout)))

    def close(self):
        if self.h:
            self.model.lib.ee_batch_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def field(self, name):
        """torch view of a field of the batch state (see ee_batch_layout)"""
        off = getattr(self.layout, name)
        dt = _FIELD_TYPES[name]
        count = {"h": self.B * self.model.cfg.d_model, "n_active": 1, "n_exited": 1, "breach_count": 1,
                 "status": 1, "exit_counts": ee.EE_MAX_EXITS}.get(name, self.B)
        nbytes = count * torch.empty(0, dtype=dt).element_size()
        v = self.state[off:off + nbytes].view(dt)
        return v.view(self.B, -1) if name == "h" else v

    def reset(self, tok, pos, scale=None):
        t = torch.as_tensor(np.asarray(tok, dtype=np.int32)).cuda()
        p = torch.as_tensor(np.asarray(pos, dtype=np.int32)).cuda()
        s = None if scale is None else torch.as_tensor(np.asarray(scale, dtype=np.float32)).cuda()
        ee.check(self.model.lib.ee_batch_reset(self.h, _ptr(t), _ptr(p), _ptr(s), _stream()))
        torch.cuda.current_stream().synchronize()

    def set_row_scale(self, scale):
        s = scale if isinstance(scale, torch.Tensor) else torch.as_tensor(np.asarray(scale, dtype=np.float32)).cuda()
        ee.check(self.model.lib.ee_batch_set_row_scale(self.h, _ptr(s), _stream()))
        self._scale_keep = s

    def begin_step(self):
        ee.check(self.model.lib.ee_batch_begin_step(self.model.h, self.h, _stream()))


def layer_forward(model, layer, kv, batch):
    return model.lib.ee_layer_forward(model.h, layer, kv.h, batch.h, _stream())


def exit_head(model, exit_idx, threshold, force_exit, batch, dbg_logits=None):
    return model.lib.ee_exit_head(model.h, exit_idx, threshold, int(force_exit), batch.h, _ptr(dbg_logits), _stream())


def exit_head_static(model, exit_idx, threshold, force_exit, batch):
    """ee_exit_head on the library's own scratch array: no workspace, no allocation"""
    return model.lib.ee_exit_head_static(model.h, exit_idx, threshold, int(force_exit), batch.h, _stream())


def compact_active(batch, exit_idx, exit_layer):
    return batch.model.lib.ee_compact_active(batch.h, exit_idx, exit_layer, _stream())


def fill_skipped_kv(model, from_excl, to_incl, kv, batch):
    return model.lib.ee_fill_skipped_kv(model.h, from_excl, to_incl, kv.h, batch.h, _stream())


def decode_step(model, kv, batch, thresholds):
    th = (C.c_float * len(thresholds))(*thresholds)
    return model.lib.ee_decode_step(model.h, kv.h, batch.h, th, len(thresholds), _stream())


def decode_step_checked(model, kv, batch, thresholds):
    """One decode step run segment by segment (ee_decode_segment), with a look at n_active after every
    exit but the last: once no row is left, ee_decode_finish ends the step and the deeper layers are
    never launched.  For small batches; each look synchronises the stream.  Returns the number of
    segments that ran."""
    th = (C.c_float * len(thresholds))(*thresholds)
    lib, n_active = model.lib, batch.field("n_active")
    for e in range(len(thresholds)):
        ee.check(lib.ee_decode_segment(model.h, kv.h, batch.h, th, len(thresholds), e, _stream()))
        if e + 1 < len(thresholds) and int(n_active.item()) == 0:
            break
    ee.check(lib.ee_decode_finish(model.h, kv.h, batch.h, e, _stream()))
    return e + 1


def _i32_device(a):
    if isinstance(a, torch.Tensor):
        assert a.is_cuda and a.dtype == torch.int32 and a.is_contiguous()
        return a
    return torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def prefill(model, kv, batch, tok, pos, seq):
    """One ee_prefill call: entry i is token tok[i] at position pos[i] of cache row seq[i]
    (int32 arrays of equal length, numpy or device tensors)."""
    t, p, q = _i32_device(tok), _i32_device(pos), _i32_device(seq)
    assert t.numel() == p.numel() == q.numel()
    return model.lib.ee_prefill(model.h, kv.h, batch.h, _ptr(t), _ptr(p), _ptr(q), int(t.numel()), _stream())


def prefill_chunks(contexts, rows_per_call):
    """Splits contexts {cache row: token ids} into the argument lists of successive ee_prefill
    calls of at most rows_per_call entries: cache rows in the order given, positions rising, a
    context that does not fit the call continues in the next one.  Yields (tok, pos, seq)."""
    tok, pos, seq = [], [], []
    for row, toks in contexts.items():
        done = 0
        while done < len(toks):
            take = min(len(toks) - done, rows_per_call - len(tok))
            tok.extend(int(x) for x in toks[done:done + take])
            pos.extend(range(done, done + take))
            seq.extend([int(row)] * take)
            done += take
            if len(tok) == rows_per_call:
                yield (np.array(tok, np.int32), np.array(pos, np.int32), np.array(seq, np.int32))
                tok, pos, seq = [], [], []
    if tok:
        yield (np.array(tok, np.int32), np.array(pos, np.int32), np.array(seq, np.int32))


class HiddenStore:
    """The exit hidden state of every cached token (fp32 [positions][d_model], laid out like the
    cache rows): what the keys and values of layers loaded later are computed from."""

    def __init__(self, model, kv):
        self.model, self.kv = model, kv
        nbytes = model.lib.ee_hstore_bytes(model.h, kv.h)
        self.buf = torch.zeros(nbytes // 4, dtype=torch.float32, device="cuda")

    def put_step(self, batch):
        return self.model.lib.ee_hstore_put_step(self.model.h, self.kv.h, batch.h, _ptr(self.buf), _stream())

    def put_prefill(self, batch, n):
        return self.model.lib.ee_hstore_put_prefill(self.model.h, self.kv.h, batch.h, int(n), _ptr(self.buf), _stream())


def backfill_kv(model, from_excl, to_incl, kv, batch, store, pos, seq):
    """One ee_backfill_kv call: K, V of layers (from_excl, to_incl] for the cached tokens
    (seq[i], pos[i]) from their states in `store` (a HiddenStore)."""
    p, q = _i32_device(pos), _i32_device(seq)
    assert p.numel() == q.numel()
    return model.lib.ee_backfill_kv(model.h, from_excl, to_incl, kv.h, batch.h, _ptr(store.buf), _ptr(p), _ptr(q),
                                    int(p.numel()), _stream())


class Speculator:
    """Exit-layer self-speculative decoding on one batch: the device buffers a round needs (drafts,
    emitted tokens, the states kept after the draft layers, the batch of B * k entries the verification
    pass runs on) and the call sequence of a round.  Every step is libee's."""

    def __init__(self, model, kv, batch, draft_exit, k, store=None):
        """store: the cache's HiddenStore if the caller keeps one (loading further layers later
        needs it); after a round it holds, for every emitted position, the state after layer R."""
        self.model, self.kv, self.batch, self.draft_exit, self.k = model, kv, batch, draft_exit, k
        B = batch.B
        self.store = store if store is not None else HiddenStore(model, kv)
        self.entries = Batch(model, B * k)
        z = np.zeros(B * k, np.int32)
        self.entries.reset(z, z, None)                 # clears the status word
        self.drafts = torch.zeros((k, B), dtype=torch.int32, device="cuda")
        self.n_emit = torch.zeros(B, dtype=torch.int32, device="cuda")
        self.emit = torch.zeros((B, k), dtype=torch.int32, device="cuda")

    def round(self):
        """k draft steps and one verification; enqueue only.  Afterwards n_emit[r] tokens emit[r, :n]
        are row r's output and the batch stands at its new position."""
        lib, m = self.model.lib, self.model
        for j in range(self.k):
            ee.check(lib.ee_draft_step(m.h, self.kv.h, self.batch.h, self.draft_exit, _ptr(self.drafts[j]), _stream()))
            ee.check(self.store.put_step(self.batch))
        ee.check(lib.ee_verify_drafts(m.h, self.kv.h, self.batch.h, self.entries.h, self.draft_exit, self.k,
                                      _ptr(self.store.buf), _ptr(self.drafts), _ptr(self.n_emit), _ptr(self.emit), _stream()))
        # the draft steps left the states after the draft layers in the store; what a later backfill of
        # newly loaded layers needs is the state after layer R, which the verification pass has for all k positions
        ee.check(self.store.put_prefill(self.entries, self.batch.B * self.k))


class LayerLoader:
    """Brings further layers of a model into HBM while decode steps keep running: the copies from
    pinned host memory and the repacking run on a stream of their own; a layer becomes resident
    (ee_model_set_layer_on, on the caller's current stream) once its event has completed."""

    def __init__(self, model):
        self.model = model
        self.stream = torch.cuda.Stream()
        self.pending = []

    @staticmethod
    def pin(weights):
        """host copies in pinned memory of one layer's tensors (numpy float32 / uint16 bf16 bits, or torch)"""
        out = {}
        for k, a in weights.items():
            if isinstance(a, torch.Tensor):
                t = a.detach().to("cpu")
            else:
                a = np.ascontiguousarray(a)
                t = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16) if a.dtype == np.uint16 else torch.from_numpy(a)
            p = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
            p.copy_(t)
            out[k] = p
        return out

    def start(self, layer, pinned):
        """enqueue the copy and repacking of one layer (dict as for Model.set_layer, pinned host tensors)"""
        m = self.model
        with torch.cuda.stream(self.stream):
            dev = {k: v.to("cuda", non_blocking=True) for k, v in pinned.items()}

            def pack(t, off=0, stride=1, out=None):
                if not m.bf16:
                    return t
                rows = t.shape[0] * stride
                o = out if out is not None else torch.empty((rows, t.shape[1]), dtype=m.tdtype, device="cuda")
                ee.check(m.lib.ee_pack_weight(_ptr(t), t.shape[0], t.shape[1], _ptr(o), off, stride, rows, _stream()))
                return o
            if m.bf16:
                gu = pack(dev["W_gate"], 0, 2)
                pack(dev["W_up"], 1, 2, gu)
            else:
                gu = torch.cat([dev["W_gate"], dev["W_up"]], dim=0).contiguous()
            t = dict(g_attn=dev["g_attn"], w_qkv=pack(dev["W_qkv"]), w_o=pack(dev["W_o"]), g_ffn=dev["g_ffn"],
                     w_gate_up=gu, w_down=pack(dev["W_down"]))
            ev = torch.cuda.Event()
            ev.record(self.stream)
        self.pending.append((layer, t, ev, dev))

    def poll(self, wait=False):
        """makes the layers whose transfer has completed resident, in the order they were started;
        returns their numbers"""
        done = []
        while self.pending and (wait or self.pending[0][2].query()):
            layer, t, ev, dev = self.pending.pop(0)
            if wait:
                ev.synchronize()
            w = ee.ee_layer_weights(_ptr(t["g_attn"]), _ptr(t["w_qkv"]), _ptr(t["w_o"]), _ptr(t["g_ffn"]),
                                    _ptr(t["w_gate_up"]), _ptr(t["w_down"]))
            ee.check(self.model.lib.ee_model_set_layer_on(self.model.h, layer, C.byref(w), _stream()))
            self.model._keep[("layer", layer)] = tuple(t.values())
            done.append(layer)
        return done


class BreachCounter:
    """Device-resident confidence-breach counter (window of the most recent tokens, re-assessment
    when more than cbc_max of them stopped below their threshold)."""
    HEADER_INT32 = 6          # window, cbc_max, head, filled, count, n_triggers
    LOG = 64

    def __init__(self, lib, window=100, cbc_max=50):
        self.lib = lib
        nbytes = lib.ee_cbc_state_bytes(window)
        if nbytes == 0:
            raise ValueError("window out of range")
        self.window = window
        self.state = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        ee.check(lib.ee_cbc_init(C.c_void_p(self.state.data_ptr()), window, cbc_max, _stream()))

    def push(self, flags):
        """flags: uint8 device tensor, one entry per token in stream order"""
        ee.check(self.lib.ee_cbc_push(C.c_void_p(self.state.data_ptr()), C.c_void_p(flags.data_ptr()),
                                        int(flags.numel()), _stream()))

    def push_step(self, batch):
        ee.check(self.lib.ee_cbc_push_step(C.c_void_p(self.state.data_ptr()), batch.h, _stream()))

    def read(self):
        """synchronises; returns dict(count, filled, n_triggers, tokens_seen, trigger_at)"""
        torch.cuda.current_stream().synchronize()
        raw = self.state.cpu().numpy()
        h = raw[:24].view(np.int32)
        seen = int(raw[24:32].view(np.int64)[0])
        log = raw[32:32 + 8 * self.LOG].view(np.int64)
        n = int(h[5])
        return dict(window=int(h[0]), cbc_max=int(h[1]), filled=int(h[3]), count=int(h[4]), n_triggers=n,
                    tokens_seen=seen, trigger_at=[int(v) for v in log[:min(n, self.LOG)]])


class PhtRow:
    """Device-resident row of the Performance History Table: exit profile, breaches and the sum
    of -ln p of the emitted tokens, accumulated after each decode step."""

    def __init__(self, model):
        self.model = model
        self.state = torch.zeros(C.sizeof(ee.ee_pht_row), dtype=torch.uint8, device="cuda")
        ee.check(model.lib.ee_pht_init(C.c_void_p(self.state.data_ptr()), _stream()))

    def reset(self):
        ee.check(self.model.lib.ee_pht_init(C.c_void_p(self.state.data_ptr()), _stream()))

    def push_step(self, batch):
        ee.check(self.model.lib.ee_pht_push_step(C.c_void_p(self.state.data_ptr()), self.model.h, batch.h, _stream()))

    def read(self):
        """synchronises; returns the struct's fields (exits: one count per exit head of the model)"""
        torch.cuda.current_stream().synchronize()
        row = ee.ee_pht_row.from_buffer_copy(self.state.cpu().numpy().tobytes())
        n = self.model.cfg.n_exits
        return dict(tokens=int(row.tokens), breaches=int(row.breaches), exits=[int(row.exits[e]) for e in range(n)],
                    nll=float(row.nll))


def load_or_switch(cost_full_chosen, cost_low_exit_others):
    """The branch of Algorithm 1 taken when the breach counter fires: load the rest of the chosen
    model if its figure (a cost, lower is better) is strictly below that of every other
    candidate's low-exit version, else (a tie included, as the condition is printed) switch to
    the cheapest of those.  Returns ("load", None) or ("switch", candidate)."""
    best = None
    for name in sorted(cost_low_exit_others, key=str):
        if best is None or cost_low_exit_others[name] < cost_low_exit_others[best]:
            best = name
    if best is None or cost_full_chosen < cost_low_exit_others[best]:
        return ("load", None)
    return ("switch", best)


def overhead_of_loading(n_new_layers, layer_bytes, load_bytes_per_s, cached_tokens, backfill_token_layers_per_s):
    """Seconds until the chosen model serves with n_new_layers more layers (Sec. 3.3.3, first
    option): their weights cross from host memory at the measured rate, and every cached token
    gets its keys and values in each of them at the measured backfill rate."""
    return (n_new_layers * layer_bytes / load_bytes_per_s
            + cached_tokens * n_new_layers / backfill_token_layers_per_s)


def overhead_of_switching(cached_tokens, context_tokens_per_s, bytes_to_load=0, load_bytes_per_s=None):
    """Seconds until another candidate's low-exit version serves the same requests (Sec. 3.3.3,
    second option): its resident layers are loaded if they are not in HBM yet, and the cached
    tokens of every request pass through them once (a context pass) to build its cache."""
    t = cached_tokens / context_tokens_per_s
    if bytes_to_load:
        t += bytes_to_load / load_bytes_per_s
    return t


def reassess(load_overhead_s, switch_overheads_s):
    """What the serving loop does when the breach counter fires: Algorithm 1's branch on the two
    measured overheads (the option with the smaller one is taken; a tie switches).  Returns
    (("load", None) | ("switch", candidate), the figures compared)."""
    return load_or_switch(load_overhead_s, switch_overheads_s), dict(load_s=load_overhead_s, switch_s=dict(switch_overheads_s))


class OverheadProbe:
    """Times, on the device, the pieces the two overheads are made of.  Each method runs the real
    calls (a layer load through a LayerLoader, ee_backfill_kv, ee_prefill) once and returns seconds
    of wall time between two synchronisations; nothing is estimated."""

    @staticmethod
    def _timed(fn):
        import time
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    @staticmethod
    def load(loader, pinned_layers):
        """pinned_layers: {layer: dict from LayerLoader.pin}; the layers are resident afterwards"""
        def go():
            for l, p in pinned_layers.items():
                loader.start(l, p)
            loader.poll(wait=True)
        return OverheadProbe._timed(go)

    @staticmethod
    def backfill(model, from_excl, to_incl, kv, batch, store, pos, seq):
        """pos, seq: all cached tokens, passed in calls of at most batch.B entries"""
        p, q = _i32_device(pos), _i32_device(seq)

        def go():
            for lo in range(0, p.numel(), batch.B):
                ee.check(backfill_kv(model, from_excl, to_incl, kv, batch, store, p[lo:lo + batch.B].contiguous(),
                                     q[lo:lo + batch.B].contiguous()))
        return OverheadProbe._timed(go)

    @staticmethod
    def context_pass(model, kv, batch, contexts):
        calls = [tuple(_i32_device(a) for a in c) for c in prefill_chunks(contexts, batch.B)]

        def go():
            for tok, pos, seq in calls:
                ee.check(prefill(model, kv, batch, tok, pos, seq))
        return OverheadProbe._timed(go)


class WindowSwitcher:
    """Host-side routing of one batch between several resident (partially loaded) models in fixed
    windows of decode steps: each model serves one window first, afterwards every window goes to
    the model whose last window had the larger fraction of tokens that left by confidence (not
    forced at its last resident layer); ties go to the earlier model.  Each model keeps its own
    cache, positions and token stream and is frozen while idle.  Policy only: every decode step
    is libee's."""

    def __init__(self, lanes, window):
        """lanes: list of (model, kv, batch, thresholds)"""
        self.lanes = lanes
        self.window = window
        self.last_fraction = [None] * len(lanes)
        self.steps_done = [0] * len(lanes)
        self.history = []

    def choose(self):
        for i, f in enumerate(self.last_fraction):
            if f is None:
                return i
        best = 0
        for i, f in enumerate(self.last_fraction):
            if f > self.last_fraction[best]:
                best = i
        return best

    def run_window(self, scale_for):
        """scale_for(lane index, that lane's step index) -> per-row logit scales"""
        i = self.choose()
        model, kv, batch, th = self.lanes[i]
        before = int(batch.field("breach_count").cpu()[0])
        for _ in range(self.window):
            batch.set_row_scale(scale_for(i, self.steps_done[i]))
            ee.check(decode_step(model, kv, batch, list(th)))
            self.steps_done[i] += 1
        torch.cuda.current_stream().synchronize()
        breaches = int(batch.field("breach_count").cpu()[0]) - before
        tokens = self.window * batch.B
        self.last_fraction[i] = 1.0 - breaches / tokens
        self.history.append((i, self.last_fraction[i]))
        return i, self.last_fraction[i]
