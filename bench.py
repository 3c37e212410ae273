#!/usr/bin/env python3
"""Benchmark of the fill-job hot path on one MI355X.

A step is one emulated main-job iteration (for the explicit-bubble workload: one bubble cycle):
the stage's idle windows are derived, the fill job's chain is profiled on the device and partitioned
onto the windows (Algorithm 1), and the Executor loop runs the planned chunks inside the windows
while the main stage is emulated on the timeline.  The headline value is

    fill tokens/s in bubbles = tokens of fill sequences that completed the whole chain
                               / summed duration of the windows offered

Workloads (--workload):
  cfg5 (default)  real main-job stage (3 layers d=8192, fwd+bwd on its own stream) under emulated
                  1F1B p=16 m=32 with measured t_f/t_b, the cfg3 job (24-layer d=2048 decoder, weights
                  streamed from pinned host memory) filling its bubbles: the largest configuration that
                  fits one GPU and the only one on which the main-stage slowdown is defined.  A step is
                  one main-job iteration with filling; the same iterations without filling are run
                  outside the timed region for the slowdown.  --main-offload adds the main job's
                  optimizer phase (gradient synchronisation of --sync-ms, Adam update) and offloads
                  optimizer state to pinned host memory around it; the windows gain the offloaded bytes.
  cfg2            12-layer bf16 encoder inference fill job, weights resident, 1F1B p=8 m=16
                  t_f=15 ms t_b=30 ms, 24 GiB free; the steps are shared evenly by the 8 stages.
                  --schedule gpipe fills the two contiguous windows of a GPipe main job instead.
  probe           the doubling probe of Sec. 4.2 against the real d=8192 main stage (small pipeline), next
                  to the closed-form windows; not a throughput line.
  cfg3            24-layer d=2048 causal decoder inference, weights streamed from pinned host memory,
                  explicit 40 ms bubbles separated by 20 ms, 8 GiB cap; g microbatches per layer
                  visit chosen by the planner.
  cfg4            12-layer d=1024 causal decoder TRAINING fill job (fwd + recompute/bwd + Adam,
                  accumulation across bubbles), 1F1B p=16 m=32, 16 GiB free.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# The run keeps more than four streams alive (fill, main, the contexts' copy streams, the offload and deadline
# streams); HIP's default of four hardware queues per process would make some of them share a queue, and a weight
# copy then waits behind the kernels it is meant to overlap.  Read when the HIP runtime is loaded (before torch is imported).
if int(os.environ.get("GPU_MAX_HW_QUEUES", "4") or 4) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"

BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E peak
GIB = 1 << 30


def gemm_flops(M, N, K):
    return 2.0 * M * N * K


def layer_fwd_flops(shape):
    T, d, f = shape.tokens, shape.d_model, shape.d_ff
    att = 4.0 * shape.batch * shape.seq_len ** 2 * d * (0.5 if shape.causal else 1.0)
    return gemm_flops(T, 3 * d, d) + gemm_flops(T, d, d) + 2 * gemm_flops(T, f, d) + att


def cpu_baseline(shape, params, ids, n_seq):
    """The CPU checker as it stands, timed on a bounded sample: n_seq sequences of the workload's
    batch through the whole model (embedding, all layers, final LayerNorm)."""
    from oracle import transformer as ot
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    P = ot.cast_params(params)
    sample = ids[:n_seq]
    t0 = time.perf_counter()
    ot.model_forward(sample, P, shape.n_heads, shape.causal, shape.eps)
    dt = time.perf_counter() - t0
    return {"value": sample.size / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n_seq} of {shape.batch} sequences (seq {shape.seq_len}) through all "
                      f"{shape.n_layers} layers in float64, {dt:.1f} s"}


def _oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline_layer(shape, synth, n_seq, n_lay=3):
    """The CPU checker on a bounded slice of a large inference job: n_seq sequences through n_lay layers (a layer's
    cost is the same for every layer and linear in the number of sequences), scaled to the whole stack."""
    from oracle import transformer as ot
    P = ot.cast_params({"layers": [synth.make_layer_params(shape, 0, seed=300)]})["layers"][0]
    x = synth.make_hidden(shape, seed=301, batch=n_seq).astype("float64")
    t0 = time.perf_counter()
    for _ in range(n_lay):
        x = ot.layer_forward(x, P, shape.n_heads, shape.causal, shape.eps)
    dt = time.perf_counter() - t0
    return {"value": n_seq * shape.seq_len / (dt / n_lay * shape.n_layers), "unit": "tokens/s", "cores": _oracle_threads(),
            "kind": "oracle",
            "sample": f"{n_seq} of {shape.batch} sequences (seq {shape.seq_len}) through {n_lay} of the {shape.n_layers} "
                      f"layers in float64, {dt:.1f} s, scaled to {shape.n_layers} layers (embedding and final LayerNorm "
                      f"left out: under 0.1 % of the work)"}


def cpu_baseline_train(shape, params, ids, n_seq):
    """The CPU checker's training microbatch (forward, loss, backward of every parameter) on n_seq sequences."""
    from oracle import transformer as ot
    P = ot.cast_params(params)
    sample = ids[:n_seq]
    t0 = time.perf_counter()
    ot.model_loss_and_grads(sample, P, shape.n_heads, shape.causal, shape.eps)
    dt = time.perf_counter() - t0
    return {"value": sample.size / dt, "unit": "tokens/s", "cores": _oracle_threads(), "kind": "oracle",
            "sample": f"{n_seq} of {shape.batch} sequences (seq {shape.seq_len}): forward, loss and all gradients through "
                      f"all {shape.n_layers} layers in float64 (no recompute, no Adam), {dt:.1f} s"}


def stage_stepper(pf, model, stages, args, p, m, tf, tb, fill, main_s):
    """Step i of K runs one iteration of stage (i * p) // K (i % p when K < p): each of the p stages
    gets K / p consecutive iterations, like p Executors that each sit on one device.  A stage starts
    with a new fill job planned from its first bubble; when a job completes inside the stage's
    iterations the library plans the next one from the following bubble."""
    state = {"stage": -1, "cursor": C.c_int32(0)}

    def reset():
        state["stage"] = -1

    def run(i):
        s = (i * p) // args.steps if args.steps >= p else i % p
        st = stages[s]
        if s != state["stage"]:
            state["stage"] = s
            state["cursor"] = C.c_int32(0)
            model.ctx.pf_ctx_set_replan(True, args.fill_ppm, args.switch_ns)
        if st.get("explicit"):     # windows with their own start times (GPipe): the library's explicit cycle
            return pf.pf_timeline_run(model.ctx, None, None, 0, 0, 0, 0, 0, st["windows"], st["plan"], st["n_plan"],
                                      model.chain, state["cursor"], fill.cuda_stream, main_s.cuda_stream)
        return pf.pf_timeline_run(model.ctx, None, None, p, m, st["stage"], tf, tb, st["windows"], st["plan"],
                                  st["n_plan"], model.chain, state["cursor"], fill.cuda_stream, main_s.cuda_stream)

    run.reset = reset
    return run


def kernel_rates(ctx, pf, shape):
    """Per-kernel-class rates from the HIP events the library recorded on the fill stream."""
    T, d, f = shape.tokens, shape.d_model, shape.d_ff
    att = 4.0 * shape.batch * shape.seq_len ** 2 * d * (0.5 if shape.causal else 1.0)
    esz = 2
    classes = [
        ("gemm_qkv", pf.PF_K_GEMM_QKV, "mfma", gemm_flops(T, 3 * d, d)),
        ("gemm_out", pf.PF_K_GEMM_OUT, "mfma", gemm_flops(T, d, d)),
        ("gemm_ffn1", pf.PF_K_GEMM_FFN1, "mfma", gemm_flops(T, f, d)),
        ("gemm_ffn2", pf.PF_K_GEMM_FFN2, "mfma", gemm_flops(T, d, f)),
        ("attention", pf.PF_K_ATTENTION, "mfma", att),
        ("layernorm", pf.PF_K_LAYERNORM, "hbm", 2.0 * T * d * esz),       # read x, write y
        ("embed", pf.PF_K_EMBED, "hbm", 2.0 * T * d * esz + T * 4),        # gather row, write row, ids
    ]
    out = {}
    for name, cls, bound, work in classes:
        n, ns = ctx.pf_ctx_kernel_stats(cls)
        if n == 0:
            continue
        avg_s = ns * 1e-9 / n
        if bound == "mfma":
            out[name] = {"bound": "mfma", "achieved": work / avg_s * 1e-12, "peak": BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": work / avg_s * 1e-12 / BF16_PEAK_TFLOPS, "launches": n,
                         "avg_us": avg_s * 1e6}
        else:
            out[name] = {"bound": "hbm", "achieved": work / avg_s * 1e-9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": work / avg_s * 1e-9 / HBM_PEAK_GBS, "launches": n, "avg_us": avg_s * 1e6}
    return out


def measured_traffic(key):
    """HBM bytes per launch of a roofline kernel as the profiler measured them: the committed summary of two
    rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, each scaled by what the same counter reads for a plain copy of
    known size) carries one line `traffic_bytes_per_launch[<key>]: <bytes>` per kernel.  None when no summary
    holds the key (a profiler run is needed to produce one; this program cannot read the counters itself)."""
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*hbm_traffic*.md"))):
        with open(path) as fh:
            m = re.search(r"traffic_bytes_per_launch\[%s\]:\s*(\d+)" % re.escape(key), fh.read())
        if m:
            return int(m.group(1))
    return None


def ffn1_roofline(kernels, shape, key):
    dom = kernels["gemm_ffn1"]
    return {"bound": "mfma", "achieved": dom["achieved"], "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": dom["frac"], "traffic": measured_traffic(key),
            "kernel": "gemm_bf16_nt_w4_kernel<bf16_t,bias+GELU> (FFN1: M=%d N=%d K=%d)" %
                      (shape.tokens, shape.d_ff, shape.d_model),
            "launches": dom["launches"], "avg_us": dom["avg_us"]}


AGG_KEYS = ("offered_ns", "idle_ns", "fill_busy_ns", "overrun_ns", "replicas_done", "chunks_run", "iter_ns",
            "main_busy_ns")


def base_line(args, metric_value, wall, extra):
    out = {"metric": "fill tokens/s in bubbles", "value": metric_value, "unit": "tokens/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall / max(1, args.steps) * 1e3,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic"}
    out.update(extra)
    return out


def fill_stats(agg, copy_wait_ns=0):
    """pct_bubble_filled counts the time the fill stream had kernels to run: the span from a window's first chunk
    start to its last chunk end (HIP events), less the time the stream sat waiting inside it for a streamed layer's
    host-to-HBM copy (copy_wait_ns, bracketed by events of its own)."""
    off = max(1, agg["offered_ns"])
    busy = agg["fill_busy_ns"] - copy_wait_ns
    return {"pct_bubble_filled": 100.0 * busy / off,
            "pct_idle_filled": 100.0 * busy / max(1, agg["idle_ns"]),
            "pct_bubble_spanned": 100.0 * agg["fill_busy_ns"] / off,
            "copy_wait_pct_of_offered": 100.0 * copy_wait_ns / off,
            "overrun_pct_of_offered": 100.0 * agg["overrun_ns"] / off,
            "replicas_done": agg["replicas_done"], "chunks_run": agg["chunks_run"]}


# ---------------------------------------------------------------------------------------------- cfg2
def run_cfg2(args, np, torch, pf, dev, synth):
    name = "cfg2"
    shape = synth.WORKLOADS[name]
    p, m, tf, tb, free = synth.SCHEDULES[name]
    params = synth.make_model_params(shape, seed=100)
    n_ring = 4
    ids = np.stack([synth.make_token_ids(shape, seed=101 + 1000 * i) for i in range(n_ring)])
    model = dev.DeviceModel(shape, params)
    d_in = dev.to_device(ids.astype(np.int32))
    d_out = dev.empty_storage((2, 1, shape.batch, shape.seq_len, shape.d_model), model.md)
    model.set_io(d_in, n_ring, d_out, 2)
    fill, main_s = torch.cuda.Stream(), torch.cuda.Stream()
    model.ctx.pf_profile_chain(model.chain, 3, 7, fill.cuda_stream)
    chain_ns = sum(n.dur_ns for n in model.chain)
    stages, t_plan = [], 0.0
    for s in range(p):
        if args.schedule == "gpipe":
            windows = pf.pf_schedule_gpipe(p, m, s, tf, tb, free)
        else:
            windows = pf.pf_schedule_1f1b(p, m, s, tf, tb, free, not args.paper_mode, 2 * max(n.dur_ns for n in model.chain))
        t0 = time.perf_counter()
        plan, n_plan, k = pf.pf_plan_bubbles(windows, model.chain, args.fill_ppm, args.switch_ns, 0, raw=True)
        t_plan += time.perf_counter() - t0
        stages.append(dict(stage=s, windows=windows, plan=plan, n_plan=n_plan, cursor=C.c_int32(0),
                           explicit=args.schedule == "gpipe"))

    run_step = stage_stepper(pf, model, stages, args, p, m, tf, tb, fill, main_s)

    for i in range(args.warmup):
        run_step(0)
    run_step.reset()
    # only the roofline kernel is bracketed by events during the timed steps (every pair costs a few
    # microseconds on the fill stream); the other classes are measured in two extra steps afterwards
    model.ctx.pf_ctx_kernel_timing(1 << pf.PF_K_GEMM_FFN1)
    model.ctx.pf_ctx_kernel_timing_every(8)     # one FFN1 launch in eight: an event pair costs ~10 us of stream time
    torch.cuda.synchronize()
    agg = dict.fromkeys(AGG_KEYS, 0)
    t0 = time.perf_counter()
    for i in range(args.steps):
        s = run_step(i)
        for k_ in agg:
            agg[k_] += s[k_]
        if args.verbose:
            print(f"step {i}: " + " ".join(f"{k_}={s[k_]}" for k_ in AGG_KEYS), file=sys.stderr)
        model.ctx.pf_ctx_kernel_stats(pf.PF_K_GEMM_FFN1)      # folds this step's event pairs into the totals
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    tokens = agg["replicas_done"] * shape.tokens
    dominant = kernel_rates(model.ctx, pf, shape)
    model.ctx.pf_ctx_kernel_timing(0x7f)
    model.ctx.pf_ctx_kernel_timing_every(1)
    run_step.reset()
    for i in range(2):
        run_step(0)
        model.ctx.pf_ctx_kernel_stats(pf.PF_K_GEMM_FFN1)
    kernels = kernel_rates(model.ctx, pf, shape)
    kernels["gemm_ffn1"] = dominant["gemm_ffn1"]
    out = base_line(args, tokens / (agg["offered_ns"] * 1e-9), wall, {
        "config": {"workload": f"{name}: 12-layer bf16 encoder inference fill job d=768 h=12 ff=3072 seq=512 "
                               f"batch=32, weights resident, {'GPipe' if args.schedule == 'gpipe' else '1F1B'} p={p} m={m} "
                               f"t_f=15ms t_b=30ms, 24 GiB free, "
                               f"all {p} stages, {max(1, args.steps // p)} consecutive iteration(s) each",
                   "fill_ppm": args.fill_ppm, "switch_ns": args.switch_ns,
                   "windows": "contiguous only" if args.paper_mode else "all idle windows"},
        **fill_stats(agg), "main_slowdown_pct": None,
        "fill_tflops_in_bubbles": agg["replicas_done"] * shape.n_layers * layer_fwd_flops(shape) /
        (agg["offered_ns"] * 1e-9) * 1e-12,
        "chain_ms": chain_ns * 1e-6, "planner_ms_all_stages": t_plan * 1e3,
        # the same job with the GPU to itself (profiled chain, back to back): what a bubble-second is worth against it
        "exclusive_tokens_per_s": shape.tokens / (chain_ns * 1e-9),
        "fill_vs_exclusive": (tokens / (agg["offered_ns"] * 1e-9)) / (shape.tokens / (chain_ns * 1e-9)),
        "roofline": ffn1_roofline(kernels, shape, "cfg2_ffn1"), "kernels": kernels})
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, params, ids[0], args.cpu_seqs or 24)
    model.close()
    return out


# ---------------------------------------------------------------------------------------------- cfg3
def make_cfg3_models(torch, pf, dev, synth, gs=(1, 2, 4), slot_counts=(3,), resident=False, batches=(16,)):
    """The candidate configurations of the 24-layer decoder fill job (Sec. 4.3: batch size x execution technique):
    sequences per microbatch x g microbatches per layer visit x {weights streamed from pinned host memory through n
    HBM slots for n in slot_counts, and, if `resident`, all weights kept in HBM}.  One context per candidate; the
    pinned blobs (and the device copies for the resident candidates) are shared."""
    import dataclasses
    shape = synth.WORKLOADS["cfg3"]
    md = pf.model_desc(shape)
    blobs = [dev.random_layer_blob(md, 300 + l, pinned=True) for l in range(shape.n_layers)]
    dev_blobs = [b.cuda() for b in blobs] if resident else None
    gen = torch.Generator(device="cuda")
    gen.manual_seed(299)
    mk = lambda *s: (torch.randn(*s, device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
    tok, pos = mk(shape.vocab, shape.d_model), mk(shape.seq_len, shape.d_model)
    lnf_g, lnf_b = mk(shape.d_model) + 1.0, mk(shape.d_model)
    models = []
    techniques = [("streamed", n) for n in slot_counts] + ([("resident", 0)] if resident else [])
    for tech, n_slots in techniques:
        for batch in batches:
            sh = dataclasses.replace(shape, batch=batch)
            for g in gs:
                if tech == "streamed":
                    mdl = dev.RawModel(sh, blobs, tok, pos, lnf_g, lnf_b, g=g, streamed=True, n_slots=n_slots)
                else:
                    mdl = dev.RawModel(sh, dev_blobs, tok, pos, lnf_g, lnf_b, g=g)
                mdl.label = f"{tech}{n_slots if n_slots else ''}/g={g}" + (f"/batch={batch}" if len(batches) > 1 else "")
                n_ring = 2
                ids = torch.randint(0, sh.vocab, (n_ring, g, batch, sh.seq_len), dtype=torch.int32, device="cuda",
                                    generator=gen)
                out = dev.empty_storage((1, g, batch, sh.seq_len, sh.d_model), mdl.md)
                mdl.set_io(ids, n_ring, out, 1)
                models.append(mdl)
    return shape, models


def choose_streamed_config(pf, windows, models, shape, fill_ppm, switch_ns):
    """Configuration (microbatches per layer visit) of the streamed job: the library compares the candidates on a
    run of back-to-back batches that covers eight bubble cycles (the same job follows itself).  Returns (best index
    or -1, per candidate: batches in the run, cycles the run takes)."""
    cfgs = [dict(F=[(n.dur_ns, n.mem_bytes, n.op, n.layer, n.mb_first, n.mb_count) for n in m_.chain],
                 samples=m_.cfg.g * m_.shape.batch) for m_ in models]
    best, runs, cyc, _ = pf.pf_select_config_stream(windows, cfgs, fill_ppm, switch_ns, 0, 8)
    return best, runs, cyc


def timed_fill_run(ctx, pf, torch, run_step, steps, verbose=False):
    """The timed region: `steps` calls of run_step() with only the roofline kernel (FFN1) and the copy waits
    bracketed by events.  Returns (aggregated statistics, list of per-step statistics, wall seconds, FFN1 rates
    source = the context's totals, copy wait ns)."""
    ctx.pf_ctx_kernel_timing((1 << pf.PF_K_GEMM_FFN1) | (1 << pf.PF_K_COPY_WAIT))
    torch.cuda.synchronize()
    agg = dict.fromkeys(AGG_KEYS, 0)
    per_step = []
    t0 = time.perf_counter()
    for i in range(steps):
        s = run_step()
        per_step.append(s)
        for k_ in agg:
            agg[k_] += s[k_]
        ctx.pf_ctx_kernel_stats(pf.PF_K_GEMM_FFN1)      # folds this step's event pairs into the totals
        if verbose:
            print(f"step {i}: " + " ".join(f"{k_}={s[k_]}" for k_ in AGG_KEYS), file=sys.stderr)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    _, wait_ns = ctx.pf_ctx_kernel_stats(pf.PF_K_COPY_WAIT)
    return agg, per_step, wall, wait_ns


def candidates_report(models, runs, cyc):
    return {m_.label: {"batches_in_run": runs[i], "cycles_of_run": cyc[i],
                       "chain_ms": sum(n.dur_ns for n in m_.chain) * 1e-6,
                       "mem_gib": max(n.mem_bytes for n in m_.chain) / GIB} for i, m_ in enumerate(models)}


def run_cfg3(args, np, torch, pf, dev, synth):
    if args.candidates == "all":
        shape, models = make_cfg3_models(torch, pf, dev, synth, gs=(1, 4), slot_counts=(2, 3), resident=True,
                                         batches=(16, 4, 1))
    else:
        shape, models = make_cfg3_models(torch, pf, dev, synth)
    fill, main_s = torch.cuda.Stream(), torch.cuda.Stream()
    bubble_ns, cap = int(args.bubble_ms * 1e6), int(args.cap_gib * GIB)
    windows = [dict(start=bubble_ns // 2, dur=bubble_ns, free=cap, kind=pf.PF_BUBBLE_EXPLICIT, fillable=1)]
    for mdl in models:
        mdl.ctx.pf_profile_chain(mdl.chain, 1, 3, fill.cuda_stream)
    best, runs, cyc = choose_streamed_config(pf, windows, models, shape, args.fill_ppm, args.switch_ns)
    if best < 0:
        raise RuntimeError(f"no configuration of the streamed job fits the {args.bubble_ms} ms / {args.cap_gib} GiB bubbles")
    mdl = models[best]
    shape = mdl.shape                    # the chosen candidate's sequences per microbatch
    plan, n_plan, k = pf.pf_plan_bubbles(windows, mdl.chain, args.fill_ppm, args.switch_ns, 0, raw=True)
    cursor = C.c_int32(0)
    mdl.ctx.pf_ctx_set_replan(True, args.fill_ppm, args.switch_ns)

    def run_step():
        return pf.pf_timeline_run(mdl.ctx, None, None, 0, 0, 0, 0, 0, windows, plan, n_plan, mdl.chain, cursor,
                                  fill.cuda_stream, main_s.cuda_stream)

    for _ in range(args.warmup):
        run_step()
    agg, _, wall, wait_ns = timed_fill_run(mdl.ctx, pf, torch, run_step, args.steps)
    g = mdl.cfg.g
    tokens = agg["replicas_done"] * g * shape.tokens
    dominant = kernel_rates(mdl.ctx, pf, shape)
    mdl.ctx.pf_ctx_kernel_timing(0x7f)
    for _ in range(4):
        run_step()
        mdl.ctx.pf_ctx_kernel_stats(pf.PF_K_GEMM_FFN1)
    kernels = kernel_rates(mdl.ctx, pf, shape)
    kernels["gemm_ffn1"] = dominant["gemm_ffn1"]
    blob_bytes = pf.pf_layer_blob_layout(mdl.md)[0]
    layer_visits = sum(1 for n in mdl.chain if n.op == pf.PF_OP_LAYER_FWD) * agg["replicas_done"]
    out = base_line(args, tokens / (agg["offered_ns"] * 1e-9), wall, {
        "config": {"workload": "cfg3: 24-layer bf16 causal decoder inference fill job d=2048 h=16 ff=8192 seq=1024 "
                               + ("batch=16, weights streamed per layer from pinned host memory (3 HBM slots), "
                                  if args.candidates == "streamed" else
                                  "batch 16, 4 or 1, weights streamed from pinned host memory (2 or 3 HBM slots) or resident "
                                  "in HBM, 1 or 4 microbatches per layer visit, whichever the planner picks under the cap, ") +
                               f"explicit {args.bubble_ms:g} ms bubbles separated by {args.bubble_ms / 2:g} ms, "
                               f"{args.cap_gib:g} GiB cap",
                   "fill_ppm": args.fill_ppm, "switch_ns": args.switch_ns,
                   "microbatches_per_layer_visit": g, "chosen": mdl.label,
                   "candidates": candidates_report(models, runs, cyc)},
        **fill_stats(agg, wait_ns), "main_slowdown_pct": None,
        "fill_tflops_in_bubbles": agg["replicas_done"] * g * shape.n_layers * layer_fwd_flops(shape) /
        (agg["offered_ns"] * 1e-9) * 1e-12,
        "host_to_hbm_gbs_in_bubbles": (layer_visits * blob_bytes if mdl.cfg.streamed else 0) / (agg["offered_ns"] * 1e-9) * 1e-9,
        "roofline": ffn1_roofline(kernels, shape, "cfg3_ffn1" if shape.batch == 16 else "cfg3_ffn1_small_batch"),
        "kernels": kernels})
    for m_ in models:
        m_.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_layer(synth.WORKLOADS["cfg3"], synth, args.cpu_seqs or 16)
    return out


# ---------------------------------------------------------------------------------------------- cfg4
def run_cfg4(args, np, torch, pf, dev, synth):
    name = "cfg4"
    shape = synth.WORKLOADS[name]
    p, m, tf, tb, free = synth.SCHEDULES[name]
    params = synth.make_model_params(shape, seed=300)
    adam = pf.pf_adam(1e-4, 0.9, 0.999, 1e-8, 4)
    model = dev.DeviceModel(shape, params, training=True, adam=adam)
    n_ring = 4
    ids = np.stack([synth.make_token_ids(shape, seed=301 + 1000 * i)[None] for i in range(n_ring)])
    d_in = dev.to_device(ids.astype(np.int32))
    model.set_io(d_in, n_ring, None, 0)
    fill, main_s = torch.cuda.Stream(), torch.cuda.Stream()
    model.ctx.pf_profile_chain(model.chain, 1, 3, fill.cuda_stream)
    chain_ns = sum(n.dur_ns for n in model.chain)
    stages = []
    for s in range(p):
        windows = pf.pf_schedule_1f1b(p, m, s, tf, tb, free, True, 2 * max(n.dur_ns for n in model.chain))
        plan, n_plan, k = pf.pf_plan_bubbles(windows, model.chain, args.fill_ppm, args.switch_ns, 0, raw=True)
        stages.append(dict(stage=s, windows=windows, plan=plan, n_plan=n_plan, cursor=C.c_int32(0)))

    run_step = stage_stepper(pf, model, stages, args, p, m, tf, tb, fill, main_s)

    for i in range(args.warmup):
        run_step(0)
    run_step.reset()
    _, steps0 = model.ctx.pf_ctx_train_state()
    it = iter(range(args.steps))
    agg, _, wall, _ = timed_fill_run(model.ctx, pf, torch, lambda: run_step(next(it)), args.steps)
    loss, steps1 = model.ctx.pf_ctx_train_state()
    tokens = agg["replicas_done"] * shape.tokens
    kernels = kernel_rates(model.ctx, pf, shape)       # the forward visits' FFN1 (M=8192 N=4096 K=1024), timed in situ
    # forward + recompute + backward (2x forward) = 4x the layer forward, plus the head's three T x V x d GEMMs
    step_flops = 4 * shape.n_layers * layer_fwd_flops(shape) + 3 * gemm_flops(shape.tokens, shape.vocab, shape.d_model)
    L = shape.n_layers
    out = base_line(args, tokens / (agg["offered_ns"] * 1e-9), wall, {
        "config": {"workload": f"{name}: 12-layer bf16 causal decoder TRAINING fill job d=1024 h=16 ff=4096 seq=1024 "
                               f"microbatch=8, fwd + recompute/bwd + Adam every 4 microbatches, gradients accumulated "
                               f"across bubbles, 1F1B p={p} m={m} t_f=15ms t_b=30ms, 16 GiB free, all {p} stages, {max(1, args.steps // p)} consecutive iteration(s) each",
                   "fill_ppm": args.fill_ppm, "switch_ns": args.switch_ns},
        **fill_stats(agg), "main_slowdown_pct": None,
        "fill_tflops_in_bubbles": agg["replicas_done"] * step_flops / (agg["offered_ns"] * 1e-9) * 1e-12,
        "chain_ms": chain_ns * 1e-6, "optimizer_steps": steps1 - steps0, "mean_loss": loss,
        "exclusive_tokens_per_s": shape.tokens / (chain_ns * 1e-9),
        "fill_vs_exclusive": (tokens / (agg["offered_ns"] * 1e-9)) / (shape.tokens / (chain_ns * 1e-9)),
        "arena_gib": model.arena_bytes / GIB,
        "node_ms": {"layer_fwd": model.chain[1].dur_ns * 1e-6, "head_loss": model.chain[L + 2].dur_ns * 1e-6,
                    "layer_bwd": model.chain[L + 3].dur_ns * 1e-6, "opt": model.chain[len(model.chain) - 1].dur_ns * 1e-6},
        "roofline": ffn1_roofline(kernels, shape, "cfg4_ffn1")})
    model.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_train(shape, params, ids[0, 0], args.cpu_seqs or 1)
    return out


# ---------------------------------------------------------------------------------------------- cfg5
def run_cfg5(args, np, torch, pf, dev, synth):
    shape5 = synth.WORKLOADS["cfg5"]
    p, m = 16, 32
    stage = args.stage
    in_flight = min(p - stage, m)
    md5 = pf.model_desc(shape5)
    blobs5 = [dev.random_layer_blob(md5, 500 + l) for l in range(shape5.n_layers)]
    main = dev.RawModel(shape5, blobs5, None, None, None, None, g=in_flight, training=True)
    del blobs5
    main.blobs = []          # the context copied the parameters into its arena
    torch.cuda.empty_cache()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    x = torch.randn(shape5.batch, shape5.seq_len, shape5.d_model, device="cuda", generator=gen).to(torch.bfloat16)
    fill, main_s = torch.cuda.Stream(), torch.cuda.Stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

    def time_main(reps):
        tfs, tbs = [], []
        for r in range(reps):
            ev[0].record(main_s)
            main.ctx.pf_main_stage_step(pf.PF_INSTR_FWD, 0, x.data_ptr(), main_s.cuda_stream)
            ev[1].record(main_s)
            main.ctx.pf_main_stage_step(pf.PF_INSTR_BWD, 0, x.data_ptr(), main_s.cuda_stream)
            ev[2].record(main_s)
            torch.cuda.synchronize()
            tfs.append(ev[0].elapsed_time(ev[1]))
            tbs.append(ev[1].elapsed_time(ev[2]))
        return sorted(tfs)[len(tfs) // 2], sorted(tbs)[len(tbs) // 2]

    time_main(1)
    tf_ms, tb_ms = time_main(3)
    tf, tb = int(tf_ms * 1e6), int(tb_ms * 1e6)

    shape3, models = make_cfg3_models(torch, pf, dev, synth, gs=(1, 2, 4))
    for mdl in models:
        mdl.ctx.pf_profile_chain(mdl.chain, 1, 3, fill.cuda_stream)
    cap = int(args.cap_gib * GIB)
    min_gap = 2 * max(n.dur_ns for mdl in models for n in mdl.chain if mdl.cfg.g == 1)
    windows = pf.pf_schedule_1f1b(p, m, stage, tf, tb, cap, True, min_gap)
    offload = None
    if args.main_offload:
        # measured copy rates (1 GiB, pinned host memory), planned at 85 % of them
        hbuf = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
        dbuf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        rates = []
        for dst, src in ((hbuf, dbuf), (dbuf, hbuf)):
            ts = []
            for _ in range(4):
                ev[0].record(main_s)
                with torch.cuda.stream(main_s):
                    dst.copy_(src, non_blocking=True)
                ev[1].record(main_s)
                torch.cuda.synchronize()
                ts.append(ev[0].elapsed_time(ev[1]))
            rates.append(int((1 << 30) / (sorted(ts[1:])[1] * 1e-3)))
        del hbuf, dbuf
        d2h, h2d = (int(0.85 * r) for r in rates)
        sync_ns = int(args.sync_ms * 1e6)
        state = main.ctx.pf_main_opt_state_bytes()
        slices, extra = pf.pf_offload_plan(p, m, stage, tf, sync_ns, state, d2h, h2d)
        host = torch.empty(max(256, sum(slices)), dtype=torch.uint8, pin_memory=True)
        offload = dict(state=state, slices=slices, extra=extra, host=host, sync_ns=sync_ns, rates=rates)
        for w, e in zip(windows, extra):
            w["free"] += e
    best, runs, cyc = choose_streamed_config(pf, windows, models, shape3, args.fill_ppm, args.switch_ns)
    if best < 0:
        raise RuntimeError(f"no configuration of the fill job fits the stage's bubbles with {args.cap_gib} GiB free")
    fm = models[best]
    plan, n_plan, k = pf.pf_plan_bubbles(windows, fm.chain, args.fill_ppm, args.switch_ns, 0, raw=True)
    cursor = C.c_int32(0)
    fm.ctx.pf_ctx_set_replan(True, args.fill_ppm, args.switch_ns)

    def set_offload(on):
        if offload:
            main.ctx.pf_ctx_set_main_offload(offload["sync_ns"], host.data_ptr(), host.numel(),
                                             offload["slices"] if on else [])

    def run_iter(with_fill):
        return pf.pf_timeline_run(fm.ctx if with_fill else None, main.ctx, x.data_ptr(), p, m, stage, tf, tb, windows,
                                  plan, n_plan, fm.chain, cursor, fill.cuda_stream, main_s.cuda_stream)

    set_offload(True)
    for _ in range(args.warmup):
        run_iter(True)
    # the same iterations with nothing offloaded and nothing filled, outside the timed region: half of them before
    # the filled iterations and half after, so that a drift of the device's clock does not read as a slowdown
    n_base = max(2, min(args.steps, 8))
    set_offload(False)
    base = [run_iter(False) for _ in range((n_base + 1) // 2)]
    set_offload(True)
    off_only = [run_iter(False) for _ in range(min(args.steps, 3))] if offload else []
    agg, filled, wall, wait_ns = timed_fill_run(fm.ctx, pf, torch, lambda: run_iter(True), args.steps)
    dominant = kernel_rates(fm.ctx, pf, shape3)
    set_offload(False)
    base += [run_iter(False) for _ in range(n_base // 2)]
    set_offload(True)
    fm.ctx.pf_ctx_kernel_timing(0x7f)
    run_iter(True)                                        # one more filled iteration with every kernel class bracketed
    kernels = kernel_rates(fm.ctx, pf, shape3)
    kernels["gemm_ffn1"] = dominant["gemm_ffn1"]
    t_base = sum(s["iter_ns"] for s in base) / len(base)
    t_fill = sum(s["iter_ns"] for s in filled) / len(filled)
    mb_base = sum(s["main_busy_ns"] for s in base) / len(base)
    mb_fill = sum(s["main_busy_ns"] for s in filled) / len(filled)
    g = fm.cfg.g
    tokens = agg["replicas_done"] * g * shape3.tokens
    blob_bytes = pf.pf_layer_blob_layout(fm.md)[0]
    layer_visits = sum(1 for n in fm.chain if n.op == pf.PF_OP_LAYER_FWD) * agg["replicas_done"]
    out = base_line(args, tokens / (agg["offered_ns"] * 1e-9), wall, {
        "config": {"workload": f"cfg5: main-job stage of 3 layers d=8192 h=64 ff=32768 seq=2048 microbatch=1 bf16 fwd+bwd "
                               f"(recomputing backward) on its own stream, emulated 1F1B p={p} m={m} stage {stage} with "
                               f"measured t_f={tf_ms:.1f} ms t_b={tb_ms:.1f} ms; fill = cfg3 job (24-layer d=2048 causal "
                               f"decoder inference, seq 1024, batch 16, weights streamed from pinned host memory, "
                               f"{g} microbatches per layer visit), {args.cap_gib:g} GiB free" + (
                                   f"; main job ends the iteration with a {args.sync_ms:g} ms gradient synchronisation and an "
                                   f"Adam update, and offloads {sum(offload['slices']) / GIB:.2f} of its "
                                   f"{offload['state'] / GIB:.2f} GiB of optimizer state" if offload else ""),
                   "fill_ppm": args.fill_ppm, "switch_ns": args.switch_ns,
                   "chosen": fm.label, "microbatches_per_layer_visit": g,
                   "candidates": candidates_report(models, runs, cyc),
                   "iterations_without_fill": len(base)},
        **fill_stats(agg, wait_ns),
        **({"main_offload": {
            "d2h_gb_per_s": offload["rates"][0] * 1e-9, "h2d_gb_per_s": offload["rates"][1] * 1e-9,
            "slice_mib": offload["slices"][0] / (1 << 20), "slices_used": sum(1 for c in offload["slices"] if c),
            "extra_free_gib_per_window": sorted({round(e / GIB, 3) for e in offload["extra"]}),
            "slowdown_pct_offload_alone": 100.0 * (sum(s_["iter_ns"] for s_ in off_only) / len(off_only) - t_base) / t_base,
            "offload_wait_ms_per_iter": sum(s_["offload_wait_ns"] for s_ in filled) / len(filled) * 1e-6,
            "offloaded_gib_per_iter": filled[-1]["offloaded_bytes"] / GIB}} if offload else {}),
        "main_slowdown_pct": 100.0 * (t_fill - t_base) / t_base,
        "main_iter_ms_without_fill": t_base * 1e-6, "main_iter_ms_with_fill": t_fill * 1e-6,
        "main_busy_ms_without_fill": mb_base * 1e-6, "main_busy_ms_with_fill": mb_fill * 1e-6,
        "main_stage_tflops": (4 * shape5.n_layers * layer_fwd_flops(shape5) * m) / (mb_base * 1e-9) * 1e-12,
        "fill_tflops_in_bubbles": agg["replicas_done"] * g * shape3.n_layers * layer_fwd_flops(shape3) /
        (agg["offered_ns"] * 1e-9) * 1e-12,
        "host_to_hbm_gbs_in_bubbles": layer_visits * blob_bytes / (agg["offered_ns"] * 1e-9) * 1e-9,
        "roofline": ffn1_roofline(kernels, shape3, "cfg3_ffn1"), "kernels": kernels})
    for m_ in models:
        m_.close()
    main.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_layer(shape3, synth, args.cpu_seqs or 16)
    return out


# --------------------------------------------------------------------------------------------- probe
def run_probe(args, np, torch, pf, dev, synth):
    """Bubble characterisation (Sec. 4.2) of the real d=8192 main stage: the doubling probe with the stage's kernels
    running and the other stages simulated from the measured t_f / t_b, next to the closed-form windows and to the
    host simulation of the same probe.  A small pipeline (p=4, m=8 by default) keeps the probe to about a minute;
    not a throughput measurement: `value` is the number of windows probed."""
    shape5 = synth.WORKLOADS["cfg5"]
    p, m, stage = args.probe_p, args.probe_m, args.stage if args.stage < args.probe_p else 1
    md5 = pf.model_desc(shape5)
    blobs5 = [dev.random_layer_blob(md5, 500 + l) for l in range(shape5.n_layers)]
    main = dev.RawModel(shape5, blobs5, None, None, None, None, g=min(p - stage, m), training=True)
    del blobs5
    main.blobs = []
    torch.cuda.empty_cache()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    x = torch.randn(shape5.batch, shape5.seq_len, shape5.d_model, device="cuda", generator=gen).to(torch.bfloat16)
    st = torch.cuda.Stream()
    tfs, tbs = [], []
    for _ in range(4):      # an instruction as the probe sees it: launch to the end of a host synchronisation
        torch.cuda.synchronize()
        t0 = time.perf_counter_ns()
        main.ctx.pf_main_stage_step(pf.PF_INSTR_FWD, 0, x.data_ptr(), st.cuda_stream)
        st.synchronize()
        t1 = time.perf_counter_ns()
        main.ctx.pf_main_stage_step(pf.PF_INSTR_BWD, 0, x.data_ptr(), st.cuda_stream)
        st.synchronize()
        t2 = time.perf_counter_ns()
        tfs.append(t1 - t0)
        tbs.append(t2 - t1)
    tf, tb = sorted(tfs[1:])[1], sorted(tbs[1:])[1]
    first, tol = int(args.probe_first_ms * 1e6), args.probe_tol_ppm
    t0 = time.perf_counter()
    est, base = pf.pf_probe_bubbles_live(main.ctx, x.data_ptr(), p, m, stage, tf, tb, first, tol, st.cuda_stream)
    wall = time.perf_counter() - t0
    windows = pf.pf_schedule_1f1b(p, m, stage, tf, tb, 0, True, 0)
    host = pf.pf_probe_bubbles(p, m, stage, tf, tb, first, tol)
    main.close()
    return {"metric": "bubble windows probed", "value": len(est), "unit": "windows", "n_gpus": 1, "steps": 1, "warmup": 0,
            "ms_per_step": wall * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
            "data": "synthetic",
            "config": {"workload": f"probe: doubling probe of the d=8192 main stage (3 layers, seq 2048), 1F1B p={p} m={m} "
                                   f"stage {stage}, first wait {args.probe_first_ms:g} ms, tolerance {tol} ppm"},
            "t_f_ms": tf * 1e-6, "t_b_ms": tb * 1e-6, "undisturbed_period_ms": base * 1e-6,
            "schedule_iteration_ms": (m + p - 1) * (tf + tb) * 1e-6,
            "windows_ms": [w["dur"] * 1e-6 for w in windows], "window_kinds": [w["kind"] for w in windows],
            "estimates_ms": [e * 1e-6 for e in est], "host_simulation_estimates_ms": [e * 1e-6 for e in host],
            "roofline": None}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg5", choices=["cfg2", "cfg3", "cfg4", "cfg5", "probe"])
    ap.add_argument("--fill-ppm", type=int, default=None,
                    help="fraction of each bubble the plan may use (default 0.95 for cfg5, whose chunks never overran their window\n"
                         "up to 0.98 in the sweep, 0.90 for the others)")
    ap.add_argument("--switch-ns", type=int, default=100_000, help="fixed per-bubble cost subtracted before packing")
    ap.add_argument("--paper-mode", action="store_true", help="fill only the contiguous bubbles (cfg2)")
    ap.add_argument("--schedule", default="1f1b", choices=["1f1b", "gpipe"],
                    help="cfg2: main-job schedule whose idle windows are filled (Sec. 4.5; GPipe has two contiguous windows per stage)")
    ap.add_argument("--stage", type=int, default=7, help="pipeline stage emulated by cfg5")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=0,
                    help="sequences of the CPU baseline's sample (0: 24 for cfg2, 16 for cfg3/cfg5, 1 for cfg4)")
    ap.add_argument("--verbose", action="store_true", help="per-step statistics on stderr (cfg2)")
    ap.add_argument("--bubble-ms", type=float, default=40.0, help="cfg3: duration of the explicit bubbles")
    ap.add_argument("--cap-gib", type=float, default=8.0, help="cfg3, cfg5: free memory inside the bubbles")
    ap.add_argument("--main-offload", action="store_true",
                    help="cfg5: the main stage ends each iteration with a gradient synchronisation and an optimizer "
                         "update, and offloads optimizer state to pinned host memory around them")
    ap.add_argument("--sync-ms", type=float, default=100.0, help="cfg5 --main-offload: gradient synchronisation time")
    ap.add_argument("--candidates", default="streamed", choices=["streamed", "all"],
                    help="cfg3: configurations offered to the planner: the workload's own (weights streamed through 3 "
                         "slots, 1/2/4 microbatches per layer visit) or also 2 slots and weights resident in HBM")
    ap.add_argument("--probe-p", type=int, default=4)
    ap.add_argument("--probe-m", type=int, default=8)
    ap.add_argument("--probe-first-ms", type=float, default=5.0, help="probe: first wait tried at a bubble instruction")
    ap.add_argument("--probe-tol-ppm", type=int, default=20_000, help="probe: slowdown of the period that counts as none")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device-to-device copy 10 times (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the fill path has no cross-GPU step "
              "(one independent Executor per device). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)
    defaults = {"cfg2": (16, 2), "cfg3": (50, 3), "cfg4": (16, 1), "cfg5": (6, 1), "probe": (1, 0)}
    if args.fill_ppm is None:
        args.fill_ppm = 950_000 if args.workload == "cfg5" else 900_000
    if args.steps is None:
        args.steps = defaults[args.workload][0]
    if args.warmup is None:
        args.warmup = defaults[args.workload][1]

    import numpy as np
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback for the product path", file=sys.stderr)
        sys.exit(3)
    from paper_2410_07192_amd import binding as pf
    from paper_2410_07192_amd import device as dev
    from paper_2410_07192_amd import synth

    if args.copy_calibration:
        n = 256 << 20
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_copy": n, "bytes_written_per_copy": n, "copies": 10}))
        return
    run = {"cfg2": run_cfg2, "cfg3": run_cfg3, "cfg4": run_cfg4, "cfg5": run_cfg5, "probe": run_probe}[args.workload]
    out = run(args, np, torch, pf, dev, synth)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
