"""GPU parity at the benchmark's full shapes, on sampled outputs the CPU checker can compute one by one
(attention couples tokens only inside a sequence, so one whole sequence of the batch is checked), in
the launch configuration bench.py uses; plus the explicit-bubble timeline."""
import ctypes as C
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import planner as op               # noqa: E402
from oracle import transformer as ot           # noqa: E402
from paper_2410_07192_amd import synth         # noqa: E402


def _mods():
    from paper_2410_07192_amd import binding as pf
    from paper_2410_07192_amd import device as dev
    return pf, dev


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def test_cfg2_full_batch_sampled_sequences():
    """12-layer bf16 encoder at d=768, seq 512, batch 32: the whole chain on the GPU, two sequences of
    the batch against the checker (end to end through 12 layers, not teacher-forced)."""
    pf, dev = _mods()
    shape = synth.WORKLOADS["cfg2"]
    params = synth.make_model_params(shape, seed=100)
    ids = synth.make_token_ids(shape, seed=101)
    m = dev.DeviceModel(shape, params)
    try:
        d_in = dev.to_device(ids[None].astype(np.int32))
        d_out = dev.empty_storage((1, 1, shape.batch, shape.seq_len, shape.d_model), m.md)
        m.set_io(d_in, 1, d_out, 1)
        st = torch.cuda.Stream()
        nF = len(m.chain)
        for a, b in ((0, 5), (5, 6), (6, nF)):
            m.ctx.pf_fill_chunk_fwd(m.chunk(a, b), m.chain, stream=st.cuda_stream)
            m.ctx.pf_ctx_sync()
        got = dev.read_storage(d_out, m.md)[0, 0]
        P = ot.cast_params(params)
        for b in (0, 19):
            ref = ot.model_forward(ids[b:b + 1], P, shape.n_heads, shape.causal, shape.eps)
            assert rel_err(got[b], ref[0]) < 2e-2, b
        assert np.isfinite(got).all()
    finally:
        m.close()


def test_cfg3_shaped_layer_streamed_teacher_forced():
    """One layer of the d=2048 / 16-head / FFN-8192 causal decoder at seq 1024 (d_head 128), weights
    streamed from pinned host memory through 3 slots, g = 2 microbatches per visit."""
    pf, dev = _mods()
    shape = synth.ModelShape(2, 2048, 16, 8192, 1024, 2, 0, True, "bf16")
    params = synth.make_model_params(shape, seed=200)
    g = 2
    x = np.stack([synth.make_hidden(shape, seed=210 + i) for i in range(g)])
    m = dev.DeviceModel(shape, params, g=g, streamed=True, n_slots=3)
    try:
        d_in = dev.storage_tensor(x, m.md)
        d_mid = dev.empty_storage(x.shape, m.md)
        st = torch.cuda.Stream()
        m.ctx.pf_fill_chunk_fwd(m.chunk(0, 1), m.chain, act_in=d_in.data_ptr(), act_out=d_mid.data_ptr(),
                                stream=st.cuda_stream)
        m.ctx.pf_ctx_sync()
        got = dev.read_storage(d_mid, m.md)
        P = ot.cast_params(params)["layers"][0]
        ref = ot.layer_forward(x[1, 1:2].astype(np.float64), P, shape.n_heads, True, shape.eps)
        assert rel_err(got[1, 1], ref[0]) < 2e-2
        # second layer from the GPU's own intermediate (teacher-forced), other microbatch
        d_out = dev.empty_storage(x.shape, m.md)
        m.ctx.pf_fill_chunk_fwd(m.chunk(1, 2), m.chain, act_in=d_mid.data_ptr(), act_out=d_out.data_ptr(),
                                stream=st.cuda_stream)
        m.ctx.pf_ctx_sync()
        P1 = ot.cast_params(params)["layers"][1]
        ref1 = ot.layer_forward(got[0, 0:1].astype(np.float64), P1, shape.n_heads, True, shape.eps)
        assert rel_err(dev.read_storage(d_out, m.md)[0, 0], ref1[0]) < 2e-2
    finally:
        m.close()


@pytest.mark.parametrize("M,N,K", [(2048, 8192, 8192), (2048, 4096, 32768), (8192, 50304, 1024)])
def test_large_gemm_sampled_rows(M, N, K):
    """GEMM shapes of the d=8192 main stage and of the tied head: sampled output rows against float64."""
    pf, dev = _mods()
    md = pf.pf_model_desc()
    md.dtype = pf.PF_DTYPE_BF16
    gen = torch.Generator(device="cuda")
    gen.manual_seed(M + N + K)
    X = torch.randn(M, K, device="cuda", generator=gen).to(torch.bfloat16)
    W = (torch.randn(N, K, device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
    b = torch.randn(N, device="cuda", generator=gen).to(torch.bfloat16)
    Cm = torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
    pf.pf_op_gemm(pf.PF_DTYPE_BF16, X.data_ptr(), W.data_ptr(), Cm.data_ptr(), M, N, K, bias=b.data_ptr())
    torch.cuda.synchronize()
    rows = [0, 1, M // 2 + 3, M - 1]
    Xh = X[rows].float().cpu().numpy().astype(np.float64)
    Wh = W.float().cpu().numpy().astype(np.float64)
    ref = Xh @ Wh.T + b.float().cpu().numpy().astype(np.float64)
    got = Cm[rows].float().cpu().numpy()
    assert rel_err(got, ref) < 1e-2


@pytest.mark.parametrize("M,N,K", [(4096, 1024, 8192), (1024, 4096, 8192), (3072, 1024, 8192), (50304, 1024, 8192)])
def test_weight_gradient_gemm_full_shapes(M, N, K):
    """The weight-gradient shapes of the training workload (and of its tied head) on the k-major kernel, with the
    bias gradient: sampled output rows and the whole column sum against float64."""
    pf, dev = _mods()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(M + 3 * N + K)
    A = torch.randn(K, M, device="cuda", generator=gen).to(torch.bfloat16)
    Bm = (torch.randn(K, N, device="cuda", generator=gen) * 0.1).to(torch.bfloat16)
    Cm = torch.zeros(M, N, device="cuda", dtype=torch.float32)
    cs = torch.zeros(M, device="cuda", dtype=torch.float32)
    pf.pf_op_gemm_tn(pf.PF_DTYPE_BF16, A.data_ptr(), Bm.data_ptr(), Cm.data_ptr(), M, N, K, cs.data_ptr())
    torch.cuda.synchronize()
    rows = [0, 1, 127, 128, M // 2 + 5, M - 1]
    Ah = A[:, rows].float().cpu().numpy().astype(np.float64)
    Bh = Bm.float().cpu().numpy().astype(np.float64)
    ref = Ah.T @ Bh
    got = Cm[rows].cpu().numpy().astype(np.float64)
    scale = (np.abs(Ah).T @ np.abs(Bh)).max()
    assert np.abs(got - ref).max() <= 5e-5 * scale
    cref = A.double().sum(dim=0).cpu().numpy()          # exact enough: float64 sum of bf16 values
    assert np.abs(cs.cpu().numpy() - cref).max() <= 5e-5 * float(A.double().abs().sum(dim=0).max())


@pytest.mark.parametrize("B,S,h,dh", [(8, 1024, 16, 64), (16, 1024, 16, 128), (1, 2048, 64, 128)])
def test_attention_full_shapes_sampled_heads(B, S, h, dh):
    """Causal attention forward and backward at the shapes of the training fill job, of the streamed decoder and of
    the d=8192 main stage: three (sequence, head) pairs, all their rows, against float64."""
    pf, dev = _mods()
    d = h * dh
    gen = torch.Generator(device="cuda")
    gen.manual_seed(S + h + dh)
    qkv = torch.randn(B, S, 3 * d, device="cuda", generator=gen).to(torch.bfloat16)
    dout = torch.randn(B, S, d, device="cuda", generator=gen).to(torch.bfloat16)
    out = torch.empty(B, S, d, device="cuda", dtype=torch.bfloat16)
    dqkv = torch.empty_like(qkv)
    lse = torch.empty(B, h, S, device="cuda", dtype=torch.float32)
    dsum = torch.empty_like(lse)
    pf.pf_op_attention(pf.PF_DTYPE_BF16, qkv.data_ptr(), out.data_ptr(), B, S, h, dh, True, lse.data_ptr())
    pf.pf_op_attention_bwd(pf.PF_DTYPE_BF16, qkv.data_ptr(), out.data_ptr(), dout.data_ptr(), lse.data_ptr(),
                           dsum.data_ptr(), dqkv.data_ptr(), B, S, h, dh, True)
    torch.cuda.synchronize()
    for bi, hi in {(0, 0), (B // 2, h // 2 + 1), (B - 1, h - 1)}:
        sl = lambda t, part: t[bi, :, part * d + hi * dh:part * d + (hi + 1) * dh].float().cpu().numpy().astype(np.float64)
        q, k, v = (sl(qkv, i)[None, None] for i in range(3))
        do = dout[bi, :, hi * dh:(hi + 1) * dh].float().cpu().numpy().astype(np.float64)[None, None]
        A = ot.attention_probs(q, k, True)
        assert rel_err(out[bi, :, hi * dh:(hi + 1) * dh].float().cpu().numpy(), (A @ v)[0, 0]) < 1e-2
        dA = do @ v.transpose(0, 1, 3, 2)
        ds = A * (dA - (dA * A).sum(-1, keepdims=True))
        refs = (ds @ k / np.sqrt(dh), ds.transpose(0, 1, 3, 2) @ q / np.sqrt(dh), A.transpose(0, 1, 3, 2) @ do)
        for i, ref in enumerate(refs):
            assert rel_err(sl(dqkv, i), ref[0, 0]) < 2e-2, (bi, hi, "qkv"[i])


def test_explicit_bubble_cycle_timeline():
    """Explicit windows (p = 0): chunks run only inside the given windows, plans are cyclic, results of
    completed replicas match the checker, and the configuration choice agrees with the checker."""
    pf, dev = _mods()
    shape = synth.ModelShape(6, 128, 2, 256, 128, 2, 300, True, "bf16")
    params = synth.make_model_params(shape, seed=12)
    n_rep = 3
    models, cfgs = [], []
    ids_all = {}
    st, main = torch.cuda.Stream(), torch.cuda.Stream()
    try:
        for g in (1, 2):
            m = dev.DeviceModel(shape, params, g=g, streamed=True, n_slots=2)
            ids = np.stack([np.stack([synth.make_token_ids(shape, seed=500 + 10 * r + j) for j in range(g)])
                            for r in range(n_rep)])
            d_in = dev.to_device(ids.astype(np.int32))
            d_out = dev.empty_storage((n_rep, g, shape.batch, shape.seq_len, shape.d_model), m.md)
            m.set_io(d_in, n_rep, d_out, n_rep)
            m.ctx.pf_profile_chain(m.chain, 1, 3, st.cuda_stream)
            models.append((m, d_in, d_out))
            ids_all[g] = ids
            cfgs.append(dict(F=m.chain, samples=g * shape.batch))
        chain_ns = sum(n.dur_ns for n in models[0][0].chain)
        windows = [dict(start=300_000, dur=max(2 * chain_ns // 3, 400_000), free=1 << 30, kind=3, fillable=1),
                   dict(start=300_000 + 2 * chain_ns, dur=max(chain_ns // 2, 400_000), free=1 << 30, kind=3, fillable=1)]
        windows[1]["start"] = windows[0]["start"] + windows[0]["dur"] + 200_000
        best, rep, cyc, chk = pf.pf_select_config(windows, cfgs, 900_000, 0, 0)
        want_best, plans = op.choose_configuration(
            windows, [dict(F=[(n.dur_ns, n.mem_bytes) for n in c["F"]], samples=c["samples"]) for c in cfgs], 900_000, 0, 0)
        assert best == want_best and best >= 0
        m, d_in, d_out = models[best]
        g = m.cfg.g
        plan, n_plan, k = pf.pf_plan_bubbles(windows, m.chain, 900_000, 0, 0, raw=True)
        cursor = C.c_int32(0)
        done = 0
        for _ in range(8):
            s = pf.pf_timeline_run(m.ctx, None, None, 0, 0, 0, 0, 0, windows, plan, n_plan, m.chain, cursor,
                                   st.cuda_stream, main.cuda_stream)
            assert s["offered_ns"] == windows[0]["dur"] + windows[1]["dur"]
            assert s["iter_ns"] >= windows[1]["start"] + windows[1]["dur"]
            done += s["replicas_done"]
            if done >= 2:
                break
        assert done >= 1
        got = dev.read_storage(d_out, m.md)
        for r in range(min(done, n_rep)):
            for j in range(g):
                ref = ot.model_forward(ids_all[g][r, j], ot.cast_params(params), shape.n_heads, True, shape.eps)
                assert rel_err(got[r, j], ref) < 2e-2, (r, j)
        with pytest.raises(pf.PipeFillError) as e:
            bad = [dict(start=0, dur=10, free=1, kind=3, fillable=1), dict(start=5, dur=10, free=1, kind=3, fillable=1)]
            pf.pf_timeline_run(m.ctx, None, None, 0, 0, 0, 0, 0, bad, plan, n_plan, m.chain, C.c_int32(0),
                               st.cuda_stream, main.cuda_stream)
        assert e.value.code == pf.PF_ERR_ARG
    finally:
        for m, _, _ in models:
            m.close()


def _simulate_jobs(windows, F, ppm, sw, iters):
    """Chunks and completed replicas per iteration when every completed fill job is followed at once by a new
    one: partitioned (by the checker) from the window that took the last chunk, whose first visit is shortened
    by the share already planned in it."""
    fill_idx = [i for i, w in enumerate(windows) if w["fillable"]]
    chunks, _ = op.partition_fill_job(windows, F, ppm, 0, sw)
    cur, out = 0, []
    for _ in range(iters):
        c = r = 0
        for wi, w in enumerate(windows):
            if not w["fillable"] or chunks[cur]["bubble"] != wi:
                continue
            planned = 0
            while True:
                ch = chunks[cur]
                if ch["node_end"] > ch["node_begin"]:
                    c += 1
                    r += sum(1 for j in range(ch["node_begin"], ch["node_end"]) if j % len(F) == len(F) - 1)
                planned += ch["dur"]
                cur += 1
                if cur < len(chunks):
                    break
                cur = 0
                left = max(w["dur"] - (-(-planned * 1_000_000 // ppm)), 0)
                chunks, _ = op.partition_fill_job(windows, F, ppm, fill_idx.index(wi), sw, first_dur=left)
        out.append((c, r))
    return out


def test_next_job_starts_where_the_last_one_ended():
    """A plan that ends in the middle of a cycle: with re-planning on, the next job starts in what is left of
    the same window (chunk and replica counts per iteration equal the checker's simulation, and the outputs
    stay right); with it off, the rest of the cycle stays empty."""
    pf, dev = _mods()
    shape = synth.ModelShape(3, 128, 2, 256, 64, 2, 300, False, "bf16")
    params = synth.make_model_params(shape, seed=31)
    n_ring = 3
    ids = np.stack([synth.make_token_ids(shape, seed=900 + r)[None] for r in range(n_ring)])
    st, main = torch.cuda.Stream(), torch.cuda.Stream()
    m = dev.DeviceModel(shape, params)
    try:
        d_in = dev.to_device(ids.astype(np.int32))
        d_out = dev.empty_storage((n_ring, 1, shape.batch, shape.seq_len, shape.d_model), m.md)
        m.set_io(d_in, n_ring, d_out, n_ring)
        for n in m.chain:                      # planning durations set by hand (well above the real ones)
            n.dur_ns = 400_000
        nF = len(m.chain)                      # embed, 3 layers, final LN: 5 nodes, 2 ms a replica
        gap = 100_000
        durs, fillable = [1_700_000, 700_000, 1_300_000, 1_900_000], [1, 1, 0, 1]
        windows, t = [], gap
        for d, f in zip(durs, fillable):
            windows.append(dict(start=t, dur=d, free=1 << 30, kind=3, fillable=f))
            t += d + gap
        F = [(n.dur_ns, n.mem_bytes) for n in m.chain]
        iters = 6
        want = _simulate_jobs(windows, F, 1_000_000, 0, iters)
        plan, n_plan, k = pf.pf_plan_bubbles(windows, m.chain, 1_000_000, 0, 0, raw=True)
        assert n_plan % 3 != 0                 # the plan ends inside a cycle
        m.ctx.pf_ctx_set_replan(True, 1_000_000, 0)
        cursor = C.c_int32(0)
        got = []
        for _ in range(iters):
            s = pf.pf_timeline_run(m.ctx, None, None, 0, 0, 0, 0, 0, windows, plan, n_plan, m.chain, cursor,
                                   st.cuda_stream, main.cuda_stream)
            assert s["overrun_ns"] == 0
            got.append((s["chunks_run"], s["replicas_done"]))
        assert got == want
        assert sum(r for _, r in got) >= n_ring
        out = dev.read_storage(d_out, m.md)
        for r in range(n_ring):
            ref = ot.model_forward(ids[r, 0], ot.cast_params(params), shape.n_heads, False, shape.eps)
            assert rel_err(out[r, 0], ref) < 2e-2, r
        # without re-planning the plan restarts only at its first bubble
        m.ctx.pf_ctx_set_replan(False)
        cursor = C.c_int32(0)
        chunks_off = 0
        for _ in range(iters):
            s = pf.pf_timeline_run(m.ctx, None, None, 0, 0, 0, 0, 0, windows, plan, n_plan, m.chain, cursor,
                                   st.cuda_stream, main.cuda_stream)
            chunks_off += s["chunks_run"]
        assert chunks_off < sum(c for c, _ in want)
        with pytest.raises(pf.PipeFillError):
            m.ctx.pf_ctx_set_replan(True, 2_000_000, 0)
    finally:
        m.close()


def test_bench_line_contract():
    """bench.py prints exactly one JSON line with the fields the harness reads, the roofline of the dominant kernel
    measured in the same run, and the CPU oracle timed beside it."""
    import json
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "2", "--warmup", "1", "--cpu-seqs", "1"],
                         capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr[-2000:]
    lines = [l for l in out.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["dtype"] == "bf16" and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9 and 0.1 < r["frac"] < 1.0
    assert r["traffic"] is None or r["traffic"] > 0
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1 and c["sample"]
    assert d["value"] > 1e5 and d["pct_bubble_filled"] > 50.0
    # the default workload is the one the whole metric is defined on: real main-stage kernels, so a slowdown exists
    assert d["config"]["workload"].startswith("cfg5") and d["main_slowdown_pct"] is not None
    assert abs(d["main_slowdown_pct"]) < 10.0 and d["pct_bubble_spanned"] >= d["pct_bubble_filled"]


_BLOB_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


def _blob_to_params(pf, md, blob):
    """Device blob in the library's layout (bf16, matrices [out][in]) -> float64 arrays in the checker's layout
    ([in][out] matrices).  Byte plumbing only."""
    _, off = pf.pf_layer_blob_layout(md)
    d, f = md.d_model, md.d_ff
    shapes = {"ln1_g": (d,), "ln1_b": (d,), "w_qkv": (3 * d, d), "b_qkv": (3 * d,), "w_o": (d, d), "b_o": (d,),
              "ln2_g": (d,), "ln2_b": (d,), "w_1": (f, d), "b_1": (f,), "w_2": (d, f), "b_2": (d,)}
    out = {}
    for i, name in enumerate(_BLOB_NAMES):
        n = int(np.prod(shapes[name]))
        a = blob[off[i]:off[i] + 2 * n].view(torch.bfloat16).reshape(shapes[name]).double().cpu().numpy()
        out[name] = a.T if a.ndim == 2 else a        # a view: the matrix products take either layout
    return out


def test_main_stage_layer_full_shape_forward_and_backward():
    """One layer of the d=8192 / 64-head / FFN-32768 main-job stage on a whole sequence of 2048 tokens: forward
    output, input gradient and EVERY parameter gradient against the float64 checker.  At this size the bf16 weight
    gradients take the transposes + accumulating NT GEMM path (results of 8192 x 8192 and more), which no smaller
    layer reaches."""
    pf, dev = _mods()
    shape = synth.ModelShape(1, 8192, 64, 32768, 2048, 1, 0, True, "bf16")
    md = pf.model_desc(shape)
    blob = dev.random_layer_blob(md, 900)
    P = _blob_to_params(pf, md, blob)
    m = dev.RawModel(shape, [blob], None, None, None, None, g=1, training=True)
    try:
        gen = torch.Generator(device="cuda")
        gen.manual_seed(901)
        x = torch.randn(1, shape.seq_len, shape.d_model, device="cuda", generator=gen).to(torch.bfloat16)
        dy = torch.randn(1, shape.seq_len, shape.d_model, device="cuda", generator=gen).to(torch.bfloat16)
        st = torch.cuda.Stream()
        m.ctx.pf_main_stage_step(pf.PF_INSTR_FWD, 0, x.data_ptr(), st.cuda_stream)
        y = torch.empty_like(x)
        m.ctx.pf_main_stage_read(0, 0, y.data_ptr(), y.numel() * 2, st.cuda_stream)
        m.ctx.pf_main_stage_step(pf.PF_INSTR_BWD, 0, dy.data_ptr(), st.cuda_stream)
        dx = torch.empty_like(x)
        m.ctx.pf_main_stage_read(1, 0, dx.data_ptr(), dx.numel() * 2, st.cuda_stream)
        m.ctx.pf_ctx_sync()
        # the checker, on the same bf16 values widened to float64
        yr, cache = ot.layer_forward(x.double().cpu().numpy(), P, shape.n_heads, True, shape.eps, keep=True)
        assert rel_err(y.float().cpu().numpy(), yr) < 2e-2
        dxr, G = ot.layer_backward(dy.double().cpu().numpy(), cache, P, shape.n_heads)
        del cache
        assert rel_err(dx.float().cpu().numpy(), dxr) < 2e-2
        md32 = pf.pf_model_desc.from_buffer_copy(m.md)
        md32.dtype = pf.PF_DTYPE_F32
        size, _ = pf.pf_layer_blob_layout(md32)
        buf = torch.empty(size, dtype=torch.uint8, device="cuda")
        m.ctx.pf_ctx_read_params(0, 0, buf.data_ptr(), size)
        m.ctx.pf_ctx_sync()
        got = pf.unpack_layer_blob_f32(m.md, buf.cpu().numpy())[0]
        for k, ref in G.items():
            assert rel_err(got[k], ref) < 2e-2, k
    finally:
        m.close()


def test_training_head_loss_and_adam_at_the_full_vocabulary():
    """The training fill job's head at its real size (d=1024, 8 x 1024 tokens, vocabulary 50257, padded to 50304
    inside the library): loss and every gradient of one microbatch through one layer against the float64 checker,
    then the Adam step at full size (51.5 M embedding and 12.6 M layer parameters) against the checker's update
    rule applied to the gradients the device produced."""
    from test_gpu_training import read_emb, read_layer
    pf, dev = _mods()
    s4 = synth.WORKLOADS["cfg4"]
    shape = synth.ModelShape(1, s4.d_model, s4.n_heads, s4.d_ff, s4.seq_len, s4.batch, s4.vocab, True, "bf16")
    params = synth.make_model_params(shape, seed=310)
    Pr = ot.cast_params(params)
    lr = 1e-3
    m = dev.DeviceModel(shape, params, training=True, adam=pf.pf_adam(lr, 0.9, 0.999, 1e-8, 2))
    try:
        ids = synth.make_token_ids(shape, seed=311)
        m.set_io(dev.to_device(ids[None, None].astype(np.int32)), 1, None, 0)
        st = torch.cuda.Stream()
        nF = len(m.chain)
        m.ctx.pf_fill_chunk(pf.pf_chunk(0, 0, 0, nF, 0, 0), m.chain, stream=st.cuda_stream)   # accumulates, no step yet
        m.ctx.pf_ctx_sync()
        loss_ref, G = ot.model_loss_and_grads(ids, Pr, shape.n_heads, True, shape.eps)
        g_layer, g_emb = read_layer(m, 0, 0), read_emb(m, 0)
        for k, ref in G["layers"][0].items():
            assert rel_err(g_layer[k], ref) < 2e-2, k
        for k in ("tok_emb", "pos_emb", "lnf_g", "lnf_b"):
            assert rel_err(g_emb[k], G[k]) < 2e-2, k
        # rows of the vocabulary that no token and no target touches still get the softmax's (small) gradient:
        # compared on their own scale
        untouched = np.setdiff1d(np.arange(shape.vocab), ids.reshape(-1))
        assert len(untouched) > 1000
        assert rel_err(g_emb["tok_emb"][untouched], G["tok_emb"][untouched]) < 2e-2
        # the same microbatch again completes the accumulation of two: Adam on the mean gradient = that gradient
        m.ctx.pf_fill_chunk(pf.pf_chunk(0, 0, nF, 2 * nF, 0, 0), m.chain, stream=st.cuda_stream)
        m.ctx.pf_ctx_sync()
        loss, steps = m.ctx.pf_ctx_train_state()
        assert steps == 1 and abs(loss - loss_ref) < 2e-3 * loss_ref
        for name, g_dev, th0, got in (("tok_emb", g_emb["tok_emb"], Pr["tok_emb"], read_emb(m, 1)["tok_emb"]),
                                      ("w_1", g_layer["w_1"], Pr["layers"][0]["w_1"], read_layer(m, 1, 0)["w_1"])):
            g64 = g_dev.astype(np.float64)                     # two equal microbatches: the mean is the gradient itself
            th1, m1, v1 = ot.adam_step(th0, 0.0, 0.0, g64, 1, lr=lr)
            # fp32 arithmetic on an update of size lr: the error is a few ulps of theta, far below the update
            assert np.abs(got.astype(np.float64) - th1).max() < 1e-3 * lr + 4e-7 * np.abs(th0).max(), name
        mom = read_emb(m, 2)["tok_emb"].astype(np.float64)
        assert np.abs(mom - 0.1 * g_emb["tok_emb"]).max() <= 1e-6 * np.abs(mom).max() + 1e-12
        assert not np.any(read_emb(m, 0)["tok_emb"])         # accumulators cleared by the step
    finally:
        m.close()


def test_one_point_of_the_free_memory_sweep():
    """One point of the sweep over the memory free inside the bubbles (Sec. 6.4): with 0.75 GiB neither the candidates
    that keep the 2.6 GB of weights resident nor those with 16 sequences per microbatch fit a bubble, so the planner
    streams the weights and takes 4 sequences per microbatch."""
    import json
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-m", "paper_2410_07192_amd.sweeps", "--which", "memory", "--caps", "0.75"],
                         capture_output=True, text=True, timeout=300, cwd=root)
    assert out.returncode == 0, out.stderr[-2000:]
    rec = json.loads(out.stdout.strip().splitlines()[-1])
    assert rec["sweep"] == "free_memory" and rec["cap_gib"] == 0.75 and "error" not in rec, rec
    assert rec["chosen"].startswith("streamed") and rec["chosen"].endswith("batch=4"), rec
    assert rec["value"] > 1e5 and rec["pct_bubble_filled"] > 50.0
