#!/usr/bin/env python3
"""Benchmark of the batched early-exit decode step on one MI355X.

Workload (default): the Llama2-70B-shaped early-exit decoder, 80 resident
layers, exit heads after layers 20/40/60/80 with thresholds 0.9/0.85/0.8/0,
batch 256, per-request context uniform in [512, 2048], 16 decode steps.  All
inputs are seeded and synthetic (random-init weights of that architecture,
random cached context) and already resident in HBM when the timed region
starts.  One "step" is one whole decode step over the batch.

Prints ONE JSON line with the decoded tokens/s, the roofline figures of the
dominant kernel (measured with HIP events on the launch stream) and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes per launch of the gate/up GEMM at batch 256 from the rocprofv3 counter runs summarised in
# profiles/llama2_70b_b256_hbm_traffic.md (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, KiB -> bytes); valid
# only for the kernel source it was measured on.
TRAFFIC_KERNEL_SHA1 = "4865c2d483da2cb324cb0dddd47a355ec085bc27"
TRAFFIC_GATE_UP_BYTES = (943832 + 9366) * 1024


def measured_traffic(batch):
    import hashlib
    src = os.path.join(ROOT, "paper_2504_10724_amd", "csrc", "ee_kernels_bf16.hip")
    try:
        same = hashlib.sha1(open(src, "rb").read()).hexdigest() == TRAFFIC_KERNEL_SHA1
    except OSError:
        same = False
    return TRAFFIC_GATE_UP_BYTES if (same and batch == 256) else None


def build_device_model(s, S, torch, max_pos, seed):
    """random-init weights generated on the device: N(0, 0.02^2) row-major bf16, then
    repacked by the library into the order its kernels stream"""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    model = S.Model.from_shape(s, max_pos=max_pos)

    def mat(n_out, n_in):
        return (torch.randn((n_out, n_in), generator=gen, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)

    d, F, qd = s.d_model, s.d_ffn, s.n_q_heads * s.head_dim
    ones = torch.ones(d, dtype=torch.float32, device="cuda")
    t0 = time.time()
    for l in range(1, s.resident + 1):
        model.set_layer(l, g_attn=ones, W_qkv=mat(s.qkv_rows, d), W_o=mat(d, qd), g_ffn=ones,
                        W_gate=mat(F, d), W_up=mat(F, d), W_down=mat(d, F))
        if l % 20 == 0:
            print(f"[bench] layers 1..{l} resident ({time.time() - t0:.1f} s)", file=sys.stderr, flush=True)
    for e, l in enumerate(s.exit_layers):
        if l <= s.resident:
            model.set_exit(e, g=ones, W=mat(s.vocab, d))
    model.set_embed(mat(s.vocab, d))
    return model


def fill_cache(kv, s, torch):
    """cached context: i.i.d. N(0, (0.02 sqrt(d))^2) in bf16 over the whole pool"""
    std = 0.02 * float(np.sqrt(s.d_model))
    pool = kv.pool.view(torch.bfloat16)
    chunk = 1 << 30
    for i in range(0, pool.numel(), chunk):
        pool[i:i + chunk].normal_(0.0, std)


def cpu_baseline(s, exit_hist, budget_s=10.0, chunk=8):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: one
    70B-shaped layer over rows of the batch (contexts drawn like the workload's), eight
    at a time until about budget_s seconds of layer time are spent or the batch is
    through, then the exit head and the skipped-layer fill for up to 32 of those rows;
    scaled to tokens/s with the exit histogram the GPU run measured."""
    import synth
    from oracle import ee_oracle as orc
    max_rows = int(s.batch)
    one = s.with_(n_layers=1, resident=1, exit_layers=(1,), thresholds=(0.0,), batch=max_rows, steps=1)
    W = synth.layer_weights(one, 1)
    E = synth.exit_weights(one, 0)
    om = orc.OracleModel(n_layers=1, d_model=s.d_model, n_q_heads=s.n_q_heads, n_kv_heads=s.n_kv_heads,
                         head_dim=s.head_dim, d_ffn=s.d_ffn, vocab=s.vocab, dtype=s.dtype, exit_layers=(1,))
    om.set_layer(1, W["g_attn"], W["W_qkv"], W["W_o"], W["g_ffn"], W["W_gate"], W["W_up"], W["W_down"])
    om.set_exit(0, E["g"], E["W"])
    ctx = synth.context_lengths(one)
    cap = int(ctx.max()) + 1
    om.set_rope(s.rope_theta, cap)
    kv = orc.OracleKV(1, max_rows, s.n_kv_heads, cap, s.head_dim)
    h = (np.random.default_rng(0).standard_normal((max_rows, s.d_model)) * 0.02).astype(np.float32)
    n_rows, t_layers = 0, 0.0
    while n_rows < max_rows and t_layers < budget_s:
        rows = range(n_rows, min(n_rows + chunk, max_rows))
        mask = np.zeros(max_rows, np.uint8)
        for b in rows:
            K, V = synth.kv_rows(one, 1, b, int(ctx[b]))
            kv.K[0, b, :, :ctx[b]] = synth.bf16_bits_to_f32(K)
            kv.V[0, b, :, :ctx[b]] = synth.bf16_bits_to_f32(V)
            mask[b] = 1
        t0 = time.perf_counter()
        orc.layer_forward(om, 1, kv, mask, ctx.astype(np.int32), h)
        t_layers += time.perf_counter() - t0
        n_rows = rows[-1] + 1
    t_layer = t_layers / n_rows
    n_small = min(n_rows, 32)
    t0 = time.perf_counter()
    for b in range(n_small):
        orc.exit_head(om, 0, h[b], 1.0)
    t_exit = (time.perf_counter() - t0) / n_small
    t0 = time.perf_counter()
    for b in range(n_small):
        orc.fill_skipped_kv(om, 0, 1, kv, b, int(ctx[b]), h[b])
    t_fill = (time.perf_counter() - t0) / n_small
    # expected time per token under the measured exit histogram
    exits = s.resident_exits
    frac = np.asarray(exit_hist, np.float64)
    frac = frac / frac.sum()
    t_tok = 0.0
    for e, l in enumerate(exits):
        t_tok += frac[e] * (l * t_layer + (e + 1) * t_exit + (s.resident - l) * t_fill)
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    cpu_model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                cpu_model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return dict(value=1.0 / t_tok, unit="tokens/s", cores=cores, kind="oracle (per-row costs of a sample, extrapolated)",
                cpu_model=cpu_model,
                sample=f"1 layer x {n_rows} rows ({t_layers:.1f} s), 1 exit head and 1 skipped-layer KV fill x "
                       f"{n_small} rows, at the workload's shape; per-row costs {t_layer:.3f}/{t_exit:.3f}/{t_fill:.4f} s combined "
                       f"with the measured exit histogram over {s.resident} layers")


def measure_layer_load(s, model, args, torch, S, ee, kv, batch, run, reset):
    """The load-more-layers path at the workload's shape (Sec. 3.3.3), outside the timed region: one
    layer's weights (pinned host memory -> HBM on a stream of their own, repacked there) alone and
    under running decode steps, and the keys/values of new layers for cached tokens."""
    d, F, qd = s.d_model, s.d_ffn, s.n_q_heads * s.head_dim
    gen = torch.Generator(device="cuda")
    gen.manual_seed(s.seed + 7)
    mat = lambda o, i: (torch.randn((o, i), generator=gen, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
    ones = torch.ones(d, dtype=torch.float32)
    pinned = S.LayerLoader.pin(dict(g_attn=ones, W_qkv=mat(s.qkv_rows, d), W_o=mat(d, qd), g_ffn=ones,
                                    W_gate=mat(F, d), W_up=mat(F, d), W_down=mat(d, F)))
    layer_bytes = sum(t.numel() * t.element_size() for t in pinned.values())
    shell = S.Model.from_shape(s, max_pos=model.cfg.max_pos)      # same shape, no weights: the layers land here
    loader = S.LayerLoader(shell)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    loader.start(1, pinned)
    loader.poll(wait=True)
    torch.cuda.synchronize()
    t_alone = time.perf_counter() - t0
    # three more layers while decode steps run on the main stream
    reset()
    torch.cuda.synchronize()
    n_load = 3
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    l0, l1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    l0.record(loader.stream)
    e0.record()
    for l in range(2, 2 + n_load):
        loader.start(l, pinned)
    l1.record(loader.stream)
    run(args.steps, 0)
    e1.record()
    torch.cuda.synchronize()
    loader.poll(wait=True)
    res = dict(layer_bytes=layer_bytes, alone_ms=t_alone * 1e3, alone_gbs=layer_bytes / t_alone / 1e9,
               under_decode_gbs=n_load * layer_bytes / (l0.elapsed_time(l1) * 1e-3) / 1e9,
               decode_ms_per_step_while_loading=e0.elapsed_time(e1) / args.steps)
    # keys and values of layers R-3..R for 256 cached tokens per call from an exit-state store
    store = S.HiddenStore(model, kv)
    store.buf.normal_(0.0, 0.02 * float(np.sqrt(d)), generator=gen)
    R = s.resident
    nl = min(4, R - 1)
    n = min(256, s.batch)
    seq = torch.arange(n, dtype=torch.int32, device="cuda")
    calls = 8
    S.backfill_kv(model, R - nl, R, kv, batch, store, torch.zeros(n, dtype=torch.int32, device="cuda"), seq)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for c in range(calls):
        rc = S.backfill_kv(model, R - nl, R, kv, batch, store, torch.full((n,), 1 + c, dtype=torch.int32, device="cuda"), seq)
        if rc != 0:
            raise ee.EEError(rc, model.lib.ee_last_error().decode())
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    res["backfill"] = dict(tokens_per_call=n, layers=nl, calls=calls, ms_per_call=dt / calls * 1e3,
                           token_layers_per_s=n * nl * calls / dt)
    del store, loader, shell, pinned
    torch.cuda.empty_cache()
    return res


def run_workload(s, model, args, torch, S, ee, synth, C, with_load=False):
    """One batch size: bind cache and batch state, warm up, rewind, time `steps` decode steps."""
    lib = model.lib
    total_steps = args.steps + args.warmup
    ctx = synth.context_lengths(s)
    cap = synth.capacity_for(ctx, max(total_steps, s.steps), 32)
    kv = S.KVCache(model, s.resident, cap)
    fill_cache(kv, s, torch)
    batch = S.Batch(model, s.batch)
    tok0 = synth.first_tokens(s)
    scales = [torch.as_tensor(synth.row_scale(s, t)).cuda() for t in range(total_steps)]
    th = list(s.thresholds)
    torch.cuda.synchronize()
    free, total = torch.cuda.mem_get_info()
    print(f"[bench] {s.name}: B={s.batch} R={s.resident} HBM used {(total - free) / 2**30:.1f} GiB of {total / 2**30:.1f}",
          file=sys.stderr, flush=True)

    def run(n_steps, first_step):
        for t in range(n_steps):
            batch.set_row_scale(scales[first_step + t])
            rc = S.decode_step(model, kv, batch, th)
            if rc != 0:
                raise ee.EEError(rc, lib.ee_last_error().decode())

    def read_classes():
        out = {}
        for k, name in enumerate(ee.KERNEL_CLASSES):
            n, ms = C.c_int(), C.c_float()
            lib.ee_timing_read(k, C.byref(n), C.byref(ms))
            out[name] = dict(launches=n.value, total_ms=round(ms.value, 3))
        return out

    # warmup from the start state, then rewind and time exactly `steps` steps.  Event pairs
    # cost stream time, so the timed region brackets only the dominant kernel (its launch
    # durations feed the roofline; the warm-up steps decide between attention and the gate/up
    # GEMM); the table of all kernel classes comes from a second, untimed pass over the same steps.
    heavy_names = ["attention", "gemm_gate_up"]
    heavy = sum(1 << ee.KERNEL_CLASSES.index(n) for n in heavy_names)
    batch.reset(tok0, ctx.astype(np.int32), None)
    lib.ee_timing_reset()
    lib.ee_timing_enable(heavy)          # the warm-up tells which of the two is the dominant kernel ...
    run(args.warmup, 0)
    torch.cuda.synchronize()
    lib.ee_timing_enable(0)
    dominant_heavy = None
    if args.warmup > 0:
        warm = read_classes()
        dominant_heavy = max(heavy_names, key=lambda n: warm[n]["total_ms"])
        heavy = 1 << ee.KERNEL_CLASSES.index(dominant_heavy)   # ... and only that one is bracketed below
    batch.reset(tok0, ctx.astype(np.int32), None)
    lib.ee_timing_reset()
    lib.ee_timing_enable(heavy)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, 0)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    lib.ee_timing_enable(0)
    timed_kern = read_classes()

    f = batch.field
    assert int(f("status").cpu()[0]) == 0, "device status flag set"
    counts = f("exit_counts").cpu().numpy()[:len(s.resident_exits)].astype(np.int64)
    tokens = s.batch * args.steps
    assert counts.sum() == tokens, (counts, tokens)

    batch.reset(tok0, ctx.astype(np.int32), None)
    lib.ee_timing_reset()
    lib.ee_timing_enable((1 << len(ee.KERNEL_CLASSES)) - 1)
    live_launches = 0          # layer launches that still had a row (the others return at once)
    cbc = S.BreachCounter(lib)  # the device-side confidence-breach counter, fed after every step
    pht = S.PhtRow(model)       # and the Performance History Table row (exit profile, perplexity)
    for t in range(args.steps):
        run(1, t)
        cbc.push_step(batch)
        pht.push_step(batch)
        torch.cuda.synchronize()
        live_launches += int(f("out_layer").max())
    lib.ee_timing_enable(0)
    cbc_state = cbc.read()
    pht_row = pht.read()
    kern = read_classes()
    for name in heavy_names:
        if timed_kern[name]["launches"] > 0:
            kern[name] = timed_kern[name]        # the durations measured inside the timed region

    # rows that ran each layer, from the exit histogram (average per step)
    exits = s.resident_exits
    left_before = np.concatenate([[0], np.cumsum(counts)[:-1]]) / args.steps   # rows gone before segment e
    seg_layers = np.diff(np.concatenate([[0], exits]))
    rows_per_launch = np.repeat(s.batch - left_before, seg_layers)              # avg active rows per layer
    d, F = s.d_model, s.d_ffn
    # gate/up projection with the SwiGLU epilogue: weights streamed once per launch
    gu = kern["gemm_gate_up"]
    gu_bytes = 2 * F * d * 2
    # per-launch durations are per launch with live rows: at small batches the deep layers run empty
    live_frac = live_launches / max(1, gu["launches"])
    rows_live = float(rows_per_launch.sum()) * args.steps / max(1, live_launches)   # average rows of a live launch
    gu_flops = 2.0 * rows_live * d * 2 * F
    gu_t = gu["total_ms"] / max(1, gu["launches"]) / max(live_frac, 1e-9) * 1e-3
    at = kern["attention"]
    kv_bytes_token = 2 * s.n_kv_heads * s.head_dim * 2
    mean_pos = float(ctx.mean()) + (args.steps + 1) / 2.0
    at_bytes = rows_live * mean_pos * kv_bytes_token
    at_t = at["total_ms"] / max(1, at["launches"]) / max(live_frac, 1e-9) * 1e-3
    layer_kernels = ["norm", "gemm_qkv", "rope_append", "attention", "gemm_o", "gemm_gate_up", "gemm_down"]
    dominant = dominant_heavy or max(layer_kernels, key=lambda k: kern[k]["total_ms"])   # the kernel bracketed above
    if dominant == "attention":
        roof = dict(kernel="k_bf16_attn", bound="hbm", achieved=at_bytes / at_t / 1e9, peak=HBM_PEAK_GBS, unit="GB/s",
                    traffic=None)
    else:
        roof = dict(kernel="k_bf16_gemm_dma8<SWIGLU> (gate/up + SwiGLU)", bound="hbm", achieved=gu_bytes / gu_t / 1e9,
                    peak=HBM_PEAK_GBS, unit="GB/s", traffic=measured_traffic(s.batch))
    roof["frac"] = roof["achieved"] / roof["peak"]
    weights_per_layer = s.layer_params() * 2
    res = dict(
        batch=s.batch, tokens_per_s=tokens / dt, ms_per_step=dt / args.steps * 1e3,
        exit_fractions={str(l): float(c) / tokens for l, c in zip(exits, counts)},
        avg_layers_per_token=float((np.asarray(exits) * counts).sum() / tokens),
        avg_active_rows=float(rows_per_launch.mean()), live_layer_launches=live_launches,
        gate_up_gemm=dict(avg_us=gu_t * 1e6, hbm_gbs=gu_bytes / gu_t / 1e9, hbm_frac=gu_bytes / gu_t / 1e9 / HBM_PEAK_GBS,
                          tflops=gu_flops / gu_t / 1e12, mfma_frac=gu_flops / gu_t / 1e12 / MFMA_BF16_PEAK_TFLOPS),
        attention=dict(avg_us=at_t * 1e6, hbm_gbs=at_bytes / at_t / 1e9, hbm_frac=at_bytes / at_t / 1e9 / HBM_PEAK_GBS),
        # all weights of a layer streamed once per launch over the four GEMMs of the layer
        layer_gemms=dict(avg_us=sum(kern[k]["total_ms"] for k in ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down")) /
                         max(1, live_launches) * 1e3,
                         hbm_gbs=weights_per_layer / (sum(kern[k]["total_ms"] for k in ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down")) /
                                                      max(1, live_launches) * 1e-3) / 1e9),
        exit_head_plus_compaction_us_per_step=(kern["exit_gemm"]["total_ms"] + kern["exit_decide"]["total_ms"] +
                                               kern["compact"]["total_ms"]) * 1e3 / args.steps,
        kernels_ms=kern, roofline=roof, counts=counts.tolist(),
        breach_counter=dict(update_us_per_step=kern["cbc"]["total_ms"] * 1e3 / args.steps,
                            reassessments=cbc_state["n_triggers"], tokens=cbc_state["tokens_seen"]),
        pht_row=dict(update_us_per_step=kern["pht"]["total_ms"] * 1e3 / args.steps, tokens=pht_row["tokens"],
                     exits=pht_row["exits"][:len(exits)], breaches=pht_row["breaches"],
                     perplexity=float(np.exp(pht_row["nll"] / max(1, pht_row["tokens"])))))
    res["layer_gemms"]["hbm_frac"] = res["layer_gemms"]["hbm_gbs"] / HBM_PEAK_GBS
    if s.batch <= 16:
        # few requests: the same steps run segment by segment, the host looking at n_active after every exit
        # and ending the step once no row is left (the layers nobody reaches are never launched)
        batch.reset(tok0, ctx.astype(np.int32), None)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        segs = 0
        for t in range(args.steps):
            batch.set_row_scale(scales[t])
            segs += S.decode_step_checked(model, kv, batch, th)
        torch.cuda.synchronize()
        dt_c = time.perf_counter() - t0
        assert f("exit_counts").cpu().numpy()[:len(exits)].astype(np.int64).tolist() == counts.tolist()
        res["step_in_segments"] = dict(tokens_per_s=tokens / dt_c, ms_per_step=dt_c / args.steps * 1e3,
                                       segments_run_per_step=segs / args.steps, segments=len(exits))
    if with_load:
        # the same kernel with every row still in the stack in every launch (no row may leave before the
        # last layer): the large-batch figure, priced against the bf16 MFMA peak
        batch.reset(tok0, ctx.astype(np.int32), None)
        lib.ee_timing_reset()
        lib.ee_timing_enable(1 << ee.KERNEL_CLASSES.index("gemm_gate_up"))
        for t in range(2):
            batch.set_row_scale(scales[t])
            rc = S.decode_step(model, kv, batch, [2.0] * len(exits))
            if rc != 0:
                raise ee.EEError(rc, lib.ee_last_error().decode())
        torch.cuda.synchronize()
        lib.ee_timing_enable(0)
        full = read_classes()["gemm_gate_up"]
        t_full = full["total_ms"] / max(1, full["launches"]) * 1e-3
        fl = 2.0 * s.batch * d * 2 * F
        roof["at_full_rows"] = dict(rows=s.batch, avg_us=t_full * 1e6, bound="mfma", achieved=fl / t_full / 1e12,
                                    peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s", frac=fl / t_full / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                                    hbm_frac=gu_bytes / t_full / 1e9 / HBM_PEAK_GBS)
    if with_load:
        res["layer_load"] = measure_layer_load(s, model, args, torch, S, ee, kv, batch, run,
                                               lambda: batch.reset(tok0, ctx.astype(np.int32), None))
    del batch, kv
    torch.cuda.empty_cache()
    return res


def run_context_pass(s, model, torch, S, ee, synth, C, entries_per_call, n_ctx=8, ctx_len=1024):
    """Context pass (ee_prefill) over n_ctx contexts of ctx_len tokens on the resident layers, in calls of
    entries_per_call entries: tokens/s with the token, position and cache-row arrays resident in HBM.
    Outside the timed decode region; reported in `detail` only."""
    lib = model.lib
    ctx_len = min(ctx_len, model.cfg.max_pos // 32 * 32)
    kv = S.KVCache(model, s.resident, np.full(n_ctx, ctx_len, np.int32))
    pb = S.Batch(model, entries_per_call)
    zero = np.zeros(entries_per_call, np.int32)
    pb.reset(zero, zero, None)
    contexts = {r: synth.context_tokens(s, r, ctx_len) for r in range(n_ctx)}
    calls = [tuple(torch.as_tensor(a).cuda() for a in c) for c in S.prefill_chunks(contexts, entries_per_call)]

    def run():
        for tok, pos, seq in calls:
            rc = S.prefill(model, kv, pb, tok, pos, seq)
            if rc != 0:
                raise ee.EEError(rc, lib.ee_last_error().decode())
    run()                                  # warm-up: the same pass once
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert int(pb.field("status").cpu()[0]) == 0, "device status flag set"
    # per-class kernel times from a further pass of its own (event pairs cost stream time)
    lib.ee_timing_reset()
    lib.ee_timing_enable((1 << len(ee.KERNEL_CLASSES)) - 1)
    run()
    torch.cuda.synchronize()
    lib.ee_timing_enable(0)
    kern = {}
    for k, name in enumerate(ee.KERNEL_CLASSES):
        n, ms = C.c_int(), C.c_float()
        lib.ee_timing_read(k, C.byref(n), C.byref(ms))
        if n.value:
            kern[name] = dict(launches=n.value, total_ms=round(ms.value, 3))
    tokens = n_ctx * ctx_len
    flops = 2.0 * tokens * s.resident * s.layer_params()      # the four products of each layer; attention not counted
    res = dict(entries_per_call=entries_per_call, contexts=n_ctx, tokens_per_context=ctx_len, calls=len(calls),
               ms=dt * 1e3, tokens_per_s=tokens / dt, gemm_tflops=flops / dt / 1e12,
               mfma_frac=flops / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS, kernels_ms=kern)
    del pb, kv
    torch.cuda.empty_cache()
    return res


def run_self_speculative(s, model, torch, S, ee, synth, batch=64, k=4, rounds=4):
    """Exit-layer self-speculative decoding (ee_draft_step, ee_verify_drafts) at the workload's shape,
    outside the timed decode region: the first exit drafts k tokens per row, the remaining layers verify
    all k positions of all rows in one pass.  Random-init heads never agree, so every round emits one
    token per row; the round time against the time of a full-depth step gives the number of tokens a
    round must emit on average to break even."""
    lib = model.lib
    sb = s.with_(batch=batch)
    ctx = synth.context_lengths(sb)
    cap = synth.capacity_for(ctx, (rounds + 2) * k + rounds + 2, 32)
    kv = S.KVCache(model, s.resident, cap)
    fill_cache(kv, sb, torch)
    b = S.Batch(model, batch)
    b.reset(synth.first_tokens(sb), ctx.astype(np.int32), None)
    sp = S.Speculator(model, kv, b, 0, k)
    never = [2.0] * len(s.resident_exits)            # no row leaves before the last resident layer

    def timed(fn, n):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    def full_step():
        rc = S.decode_step(model, kv, b, never)
        if rc != 0:
            raise ee.EEError(rc, lib.ee_last_error().decode())
    t_full = timed(full_step, rounds)
    b.reset(synth.first_tokens(sb), ctx.astype(np.int32), None)
    t_round = timed(sp.round, rounds)
    emitted = float(sp.n_emit.float().mean())
    assert int(b.field("status").cpu()[0]) == 0 and int(sp.entries.field("status").cpu()[0]) == 0
    res = dict(batch=batch, drafts_per_round=k, draft_layers=s.resident_exits[0], verify_layers=s.resident - s.resident_exits[0],
               round_ms=t_round * 1e3, full_depth_step_ms=t_full * 1e3, tokens_per_round_measured=emitted,
               tokens_per_round_to_break_even=t_round / t_full,
               tokens_per_s_if_all_accepted=batch * k / t_round, tokens_per_s_full_depth=batch / t_full)
    del sp, b, kv
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama2_70b")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--layers", type=int, default=None, help="debug: fewer resident layers (not a valid result)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the smaller batch sizes of the sweep")
    ap.add_argument("--no-layer-load", action="store_true", help="skip the layer-load and backfill measurement")
    ap.add_argument("--no-context-pass", action="store_true", help="skip the context-pass (ee_prefill) measurement")
    ap.add_argument("--no-speculative", action="store_true", help="skip the self-speculative decoding measurement")
    ap.add_argument("--context-pass-only", type=int, nargs="*", default=None, metavar="ENTRIES",
                    help="only time the context pass (ee_prefill) with these numbers of entries per call")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy 4 times (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU; nothing shards across GPUs (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    from paper_2504_10724_amd import capi as ee
    from paper_2504_10724_amd import session as S
    import ctypes as C

    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps(dict(copy_bytes=int(src.numel() * 4), copies=4)))
        return
    s = synth.CONFIGS[args.workload]
    if args.batch:
        s = s.with_(batch=args.batch)
    valid = True
    if args.layers:
        keep = tuple(l for l in s.exit_layers if l <= args.layers)
        s = s.with_(resident=args.layers, thresholds=s.thresholds[:len(keep)])
        valid = False
    total_steps = args.steps + args.warmup
    max_cap = int(synth.capacity_for(np.array([s.ctx_hi]), max(total_steps, s.steps), 32)[0])
    model = build_device_model(s, S, torch, max_cap, s.seed)
    if args.context_pass_only is not None:
        for n in (args.context_pass_only or [1024]):
            print(json.dumps(run_context_pass(s, model, torch, S, ee, synth, C, n)), flush=True)
        return
    head = run_workload(s, model, args, torch, S, ee, synth, C, with_load=not args.no_layer_load)
    sweep = {}
    if not args.no_sweep and not args.batch:
        for b in (64, 16, 1):
            r = run_workload(s.with_(batch=b), model, args, torch, S, ee, synth, C)
            sweep[str(b)] = {k: r[k] for k in ("tokens_per_s", "ms_per_step", "exit_fractions", "avg_layers_per_token",
                                               "gate_up_gemm", "attention", "layer_gemms",
                                               "exit_head_plus_compaction_us_per_step", "step_in_segments") if k in r}
    context_pass = None if args.no_context_pass else run_context_pass(s, model, torch, S, ee, synth, C, 1024)
    exits = s.resident_exits
    out = dict(metric="decoded tokens/s/GPU at Llama2-70B shape", value=head["tokens_per_s"], unit="tokens/s", n_gpus=1,
               steps=args.steps, warmup=args.warmup, ms_per_step=head["ms_per_step"], higher_is_better=True,
               scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
               config=dict(workload=f"{s.name}: L={s.n_layers} R={s.resident} d={s.d_model} Hq/Hkv={s.n_q_heads}/{s.n_kv_heads} "
                                    f"F={s.d_ffn} V={s.vocab} exits={list(exits)} th={list(s.thresholds)}",
                           batch=s.batch, ctx=[s.ctx_lo, s.ctx_hi], valid_config=valid),
               exit_fractions=head["exit_fractions"], roofline=head["roofline"],
               detail={k: head[k] for k in ("avg_layers_per_token", "avg_active_rows", "live_layer_launches", "gate_up_gemm", "attention",
                                            "layer_gemms", "exit_head_plus_compaction_us_per_step", "breach_counter", "pht_row", "kernels_ms")},
               batch_sweep=sweep)
    out["detail"]["context_pass"] = context_pass
    out["detail"]["self_speculative"] = (None if args.no_speculative or len(s.resident_exits) < 2 else
                                         run_self_speculative(s, model, torch, S, ee, synth))
    out["detail"]["layer_load"] = head.get("layer_load")
    ll = head.get("layer_load")
    if ll and context_pass and len(exits) > 1:
        # Algorithm 1's branch on these measurements (Sec. 3.3.3): this model loaded up to its first exit
        # and serving the batch's cached tokens, against a candidate of the same shape whose low-exit
        # version (as deep) is not in HBM yet; rates as measured above, the context pass scaled to that depth
        ctx_mean = (s.ctx_lo + s.ctx_hi) / 2.0
        cached = s.batch * ctx_mean
        r0 = exits[0]
        load_s = S.overhead_of_loading(s.n_layers - r0, ll["layer_bytes"], ll["under_decode_gbs"] * 1e9, cached,
                                       ll["backfill"]["token_layers_per_s"])
        switch_s = S.overhead_of_switching(cached, context_pass["tokens_per_s"] * s.resident / r0,
                                           bytes_to_load=r0 * ll["layer_bytes"], load_bytes_per_s=ll["under_decode_gbs"] * 1e9)
        decision, figures = S.reassess(load_s, {"same_shape_low_exit": switch_s})
        out["detail"]["load_or_switch"] = dict(resident_layers=r0, cached_tokens=cached, load_overhead_s=load_s,
                                               switch_overhead_s=switch_s, decision=list(decision))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(s, head["counts"])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
