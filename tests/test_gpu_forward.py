"""GPU parity: HIP kernels and forward chunks against the CPU checker, through the C ABI.

Tolerances (max |gpu - ref| / max |ref| per output tensor): 2e-2 for bf16 storage, 1e-4 for fp32.
The checker is fed the bf16-rounded inputs widened to float64, so the difference is compute and
output-rounding error only."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import transformer as ot          # noqa: E402
from paper_2410_07192_amd import synth        # noqa: E402

TOL = {"bf16": 2e-2, "f32": 1e-4}


def _mods():
    from paper_2410_07192_amd import binding as pf
    from paper_2410_07192_amd import device as dev
    return pf, dev


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def _md(dtype):
    pf, _ = _mods()
    md = pf.pf_model_desc()
    md.dtype = pf.PF_DTYPE_BF16 if dtype == "bf16" else pf.PF_DTYPE_F32
    return md


def _rand(rng, shape, dtype, scale=1.0):
    a = (rng.standard_normal(shape) * scale).astype(np.float32)
    return synth.round_to_bf16(a) if dtype == "bf16" else a


GEMM_SHAPES = [(512, 768, 256), (300, 200, 72), (1, 8, 8), (257, 129, 520), (1024, 2304, 768), (130, 3072, 64)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_plain_and_epilogues(dtype, M, N, K):
    pf, dev = _mods()
    md = _md(dtype)
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    X, W = _rand(rng, (M, K), dtype), _rand(rng, (N, K), dtype, 0.05)
    bias, R = _rand(rng, (N,), dtype), _rand(rng, (M, N), dtype)
    dX, dW, dB, dR = (dev.storage_tensor(a, md) for a in (X, W, bias, R))
    ref0 = X.astype(np.float64) @ W.astype(np.float64).T
    out = dev.empty_storage((M, N), md)
    pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), out.data_ptr(), M, N, K)
    torch.cuda.synchronize()
    assert rel_err(dev.read_storage(out, md), ref0) < TOL[dtype] / 2
    # bias + GELU
    pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), out.data_ptr(), M, N, K, bias=dB.data_ptr(), gelu=1)
    torch.cuda.synchronize()
    assert rel_err(dev.read_storage(out, md), ot.gelu(ref0 + bias)) < TOL[dtype] / 2
    # bias + residual
    pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), out.data_ptr(), M, N, K, bias=dB.data_ptr(),
                  resid=dR.data_ptr())
    torch.cuda.synchronize()
    assert rel_err(dev.read_storage(out, md), ref0 + bias + R) < TOL[dtype] / 2
    # fp32 output, accumulated twice
    acc = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    for _ in range(2):
        pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), acc.data_ptr(), M, N, K, out_f32=1, accumulate=1)
    torch.cuda.synchronize()
    assert rel_err(acc.cpu().numpy(), 2 * ref0) < 1e-4


# Shapes that make the tile chooser take the 256x192 and the 256x256 tile with ragged last tiles along M and N
# (8292 = 32 * 256 + 100), with N a multiple of 8 (16-byte row-contiguous stores) and not (8- and 2-byte stores).
# K = 64, 128, 192 and 320 are one to five K steps: the 256x256 kernel's prologue alone, its two tail steps, and its
# steady-state loop (a stage read, the next written, the one after loaded) run once and three times.
@pytest.mark.parametrize("M,N,K", [(8292, 2368, 128), (8292, 3112, 128), (8292, 2370, 64), (4196, 6150, 64),
                                   (8292, 3112, 192), (4196, 6152, 320)])
def test_gemm_large_tiles_with_ragged_edges(M, N, K):
    pf, dev = _mods()
    md = _md("bf16")
    rng = np.random.default_rng(M + N + K)
    X, W = _rand(rng, (M, K), "bf16"), _rand(rng, (N, K), "bf16", 0.05)
    bias, R = _rand(rng, (N,), "bf16"), _rand(rng, (M, N), "bf16")
    dX, dW, dB, dR = (dev.storage_tensor(a, md) for a in (X, W, bias, R))
    ref0 = X.astype(np.float64) @ W.astype(np.float64).T
    out = dev.empty_storage((M, N), md)
    guard = dev.empty_storage((M + 1, N), md)          # one extra row behind C: must stay untouched
    guard.zero_()
    pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), guard.data_ptr(), M, N, K, bias=dB.data_ptr())
    torch.cuda.synchronize()
    g = dev.read_storage(guard, md)
    assert rel_err(g[:M], ref0 + bias) < TOL["bf16"] / 2 and not g[M].any()
    pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), out.data_ptr(), M, N, K, bias=dB.data_ptr(), gelu=1)
    torch.cuda.synchronize()
    assert rel_err(dev.read_storage(out, md), ot.gelu(ref0 + bias)) < TOL["bf16"] / 2
    pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), out.data_ptr(), M, N, K, bias=dB.data_ptr(),
                  resid=dR.data_ptr())
    torch.cuda.synchronize()
    assert rel_err(dev.read_storage(out, md), ref0 + bias + R) < TOL["bf16"] / 2
    acc = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    for _ in range(2):
        pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), acc.data_ptr(), M, N, K, out_f32=1, accumulate=1)
    torch.cuda.synchronize()
    assert rel_err(acc.cpu().numpy(), 2 * ref0) < 1e-4


# The two epilogues of the training backward, on whole 256-wide tiles (both tile shapes), with ragged edges
# along M and N, with N not a multiple of 8, and on a shape that only the generic kernel takes.
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("M,N,K", [(512, 512, 128), (768, 384, 64), (8292, 2368, 128), (4196, 3112, 64), (1030, 522, 64),
                                   (300, 200, 24)])
def test_gemm_training_epilogues(dtype, M, N, K):
    pf, dev = _mods()
    md = _md(dtype)
    if dtype == "f32" and M > 1100:
        pytest.skip("the fp32 kernel has one code path; the small shapes cover it")
    rng = np.random.default_rng(M * 7 + N + K)
    X, W = _rand(rng, (M, K), dtype), _rand(rng, (N, K), dtype, 0.1)
    bias, U = _rand(rng, (N,), dtype), _rand(rng, (M, N), dtype, 1.5)
    dX, dW, dB, dU = (dev.storage_tensor(a, md) for a in (X, W, bias, U))
    ref0 = X.astype(np.float64) @ W.astype(np.float64).T
    tol = TOL[dtype] / 2
    # forward of the first FFN matrix keeping the pre-activation: two outputs, rows behind both stay untouched
    out = dev.empty_storage((M + 1, N), md)
    pre = dev.empty_storage((M + 1, N), md)
    out.zero_()
    pre.zero_()
    pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), out.data_ptr(), M, N, K, bias=dB.data_ptr(), gelu=1,
                  preact_out=pre.data_ptr())
    torch.cuda.synchronize()
    o, p_ = dev.read_storage(out, md), dev.read_storage(pre, md)
    assert rel_err(p_[:M], ref0 + bias) < tol and not p_[M].any()
    assert rel_err(o[:M], ot.gelu(ref0 + bias)) < tol and not o[M].any()
    # backward through the activation: (X W^T) * GELU'(U)
    out.zero_()
    pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), out.data_ptr(), M, N, K, dact_in=dU.data_ptr())
    torch.cuda.synchronize()
    o = dev.read_storage(out, md)
    assert rel_err(o[:M], ref0 * ot.gelu_grad(U.astype(np.float64))) < tol and not o[M].any()
    for bad in (dict(bias=dB.data_ptr()), dict(gelu=1), dict(resid=dU.data_ptr()), dict(preact_out=pre.data_ptr())):
        with pytest.raises(pf.PipeFillError):
            pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), out.data_ptr(), M, N, K, dact_in=dU.data_ptr(), **bad)


# Weight-gradient shapes: small result, K = all tokens; C holds an earlier gradient that must be kept.
@pytest.mark.parametrize("M,N,K", [(1024, 1024, 8192), (3072, 1024, 8192), (1000, 520, 4096), (256, 256, 2048)])
def test_gemm_accumulate_long_k(M, N, K):
    pf, dev = _mods()
    md = _md("bf16")
    rng = np.random.default_rng(M + N + K)
    X, W = _rand(rng, (M, K), "bf16"), _rand(rng, (N, K), "bf16", 0.05)
    dX, dW = dev.storage_tensor(X, md), dev.storage_tensor(W, md)
    ref0 = X.astype(np.float64) @ W.astype(np.float64).T
    before = rng.standard_normal((M, N)).astype(np.float32)
    acc = torch.from_numpy(before).cuda()
    for _ in range(2):
        pf.pf_op_gemm(md.dtype, dX.data_ptr(), dW.data_ptr(), acc.data_ptr(), M, N, K, out_f32=1, accumulate=1)
    torch.cuda.synchronize()
    assert rel_err(acc.cpu().numpy(), before + 2 * ref0) < 1e-4


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("rows,d", [(5, 8), (1000, 768), (37, 2048), (9, 8192), (130, 1000)])
def test_layernorm(dtype, rows, d):
    pf, dev = _mods()
    md = _md(dtype)
    rng = np.random.default_rng(rows + d)
    x = _rand(rng, (rows, d), dtype, 3.0) + (1.5 if dtype == "f32" else 0)
    x = synth.round_to_bf16(x) if dtype == "bf16" else x
    g, b = _rand(rng, (d,), dtype), _rand(rng, (d,), dtype)
    dx, dg, db = (dev.storage_tensor(a, md) for a in (x, g, b))
    y = dev.empty_storage((rows, d), md)
    mean = torch.empty(rows, dtype=torch.float32, device="cuda")
    rstd = torch.empty(rows, dtype=torch.float32, device="cuda")
    pf.pf_op_layernorm(md.dtype, dx.data_ptr(), dg.data_ptr(), db.data_ptr(), y.data_ptr(), rows, d, 1e-5,
                       mean.data_ptr(), rstd.data_ptr())
    torch.cuda.synchronize()
    ref, _, rr = ot.layer_norm(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64), 1e-5)
    assert rel_err(dev.read_storage(y, md), ref) < TOL[dtype] / 2
    assert rel_err(mean.cpu().numpy(), x.astype(np.float64).mean(-1)) < 1e-5
    assert rel_err(rstd.cpu().numpy(), rr[:, 0]) < 1e-5


@pytest.mark.parametrize("offset,nbytes", [(0, 0), (0, 15), (0, 16), (2, 40), (6, 1 << 20), (0, 8 << 20), (16, (8 << 20) - 16)])
def test_layernorm_with_a_range_to_warm(offset, nbytes):
    """The side job of the LayerNorm kernel (reading a byte range and dropping it) changes nothing in its
    result, whatever the alignment and length of the range: more pieces than threads, fewer, none, a
    ragged head and tail.  The range lies inside an 8 MiB buffer."""
    pf, dev = _mods()
    md = _md("bf16")
    rows, d = 300, 768
    rng = np.random.default_rng(17)
    x = synth.round_to_bf16(_rand(rng, (rows, d), "bf16", 2.0))
    g, b = _rand(rng, (d,), "bf16"), _rand(rng, (d,), "bf16")
    dx, dg, db = (dev.storage_tensor(a, md) for a in (x, g, b))
    buf = torch.full((8 << 20,), 7, dtype=torch.uint8, device="cuda")
    ys = []
    for warm in (False, True):
        y = dev.empty_storage((rows, d), md)
        pf.pf_op_layernorm(md.dtype, dx.data_ptr(), dg.data_ptr(), db.data_ptr(), y.data_ptr(), rows, d, 1e-5,
                           warm=buf.data_ptr() + offset if warm else None, warm_bytes=nbytes if warm else 0)
        torch.cuda.synchronize()
        ys.append(dev.to_host(y, np.uint16))
    assert np.array_equal(ys[0], ys[1])
    assert bool((buf == 7).all())
    ref, _, _ = ot.layer_norm(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64), 1e-5)
    assert rel_err(dev.read_storage(dev.to_device(ys[1]), md), ref) < TOL["bf16"] / 2


ATT_CASES = [("bf16", 2, 200, 3, 64), ("bf16", 1, 513, 2, 128), ("bf16", 3, 64, 2, 64), ("bf16", 2, 50, 2, 16),
             ("f32", 2, 128, 4, 64), ("f32", 2, 77, 2, 8), ("f32", 1, 130, 1, 128), ("bf16", 1, 1, 1, 64),
             ("bf16", 2, 65, 1, 64), ("bf16", 1, 129, 1, 128)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype,B,S,h,dh", ATT_CASES)
def test_attention(dtype, B, S, h, dh, causal):
    pf, dev = _mods()
    md = _md(dtype)
    d = h * dh
    rng = np.random.default_rng(B * 1000 + S + dh)
    qkv = _rand(rng, (B, S, 3 * d), dtype, 1.5)
    dq = dev.storage_tensor(qkv, md)
    out = dev.empty_storage((B, S, d), md)
    lse = torch.empty((B, h, S), dtype=torch.float32, device="cuda")
    pf.pf_op_attention(md.dtype, dq.data_ptr(), out.data_ptr(), B, S, h, dh, causal, lse.data_ptr())
    torch.cuda.synchronize()
    q64 = qkv.astype(np.float64)
    q, k, v = (ot.split_heads(q64[..., i * d:(i + 1) * d], h) for i in range(3))
    A = ot.attention_probs(q, k, causal)
    ref = ot.merge_heads(A @ v)
    assert rel_err(dev.read_storage(out, md), ref) < TOL[dtype] / 2
    s = q @ k.transpose(0, 1, 3, 2) / np.sqrt(dh)
    if causal:
        s = np.where(np.triu(np.ones((S, S), dtype=bool), 1), -np.inf, s)
    mx = s.max(-1)
    ref_lse = mx + np.log(np.exp(s - mx[..., None]).sum(-1))
    assert np.abs(lse.cpu().numpy() - ref_lse).max() < (2e-2 if dtype == "bf16" else 1e-4)


@pytest.mark.parametrize("B,S,h,dh", [(8, 1024, 16, 128), (3, 900, 22, 128), (8, 1024, 16, 64), (4, 1024, 16, 128)])
def test_attention_where_the_kernel_reorders_causal_blocks(B, S, h, dh):
    # Causal attention at sizes where the kernel hands the query blocks out in an order of its own.  First two cases:
    # d_head 128 on more (batch, head, query block) units than the GPU keeps workgroups resident, so that a workgroup
    # walks several units (in rounds of whole heads, handed out in alternating order; then with a ragged last block
    # and rounds that split heads).  Last two: exactly as many units as resident workgroups, the second half of each
    # XCD's range reversed.  Sec. 5; compared with the plain softmax on every query of a sample of heads.
    pf, dev = _mods()
    md = _md("bf16")
    d = h * dh
    rng = np.random.default_rng(B * 100 + h)
    qkv = _rand(rng, (B, S, 3 * d), "bf16", 1.2)
    dq = dev.storage_tensor(qkv, md)
    out = dev.empty_storage((B, S, d), md)
    lse = torch.empty((B, h, S), dtype=torch.float32, device="cuda")
    pf.pf_op_attention(md.dtype, dq.data_ptr(), out.data_ptr(), B, S, h, dh, True, lse.data_ptr())
    torch.cuda.synchronize()
    got = dev.read_storage(out, md).reshape(B, S, h, dh)
    lse_got = lse.cpu().numpy()
    assert np.isfinite(got).all()
    heads = sorted({(0, 0), (B - 1, h - 1), (B // 2, h // 3), (B - 1, 0), (0, h - 1), (B // 2, h - 2)})
    for b, i in heads:
        q, k, v = (qkv[b, :, j * d + i * dh: j * d + (i + 1) * dh].astype(np.float64) for j in range(3))
        s_ = q @ k.T / np.sqrt(dh)
        s_ = np.where(np.triu(np.ones((S, S), dtype=bool), 1), -np.inf, s_)
        mx = s_.max(-1, keepdims=True)
        e = np.exp(s_ - mx)
        ref = (e / e.sum(-1, keepdims=True)) @ v
        assert rel_err(got[b, :, i, :], ref) < TOL["bf16"] / 2, (b, i)
        assert np.abs(lse_got[b, i] - (mx[:, 0] + np.log(e.sum(-1)))).max() < 2e-2, (b, i)
    # every other head: finite and not all zero (a unit nobody visited would be)
    assert (np.abs(got).reshape(B, S, h, dh).max(axis=(1, 3)) > 0).all()


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("S,h,dh", [(300, 2, 64), (200, 2, 128)])
def test_attention_when_the_softmax_reference_has_to_move(S, h, dh, causal):
    # Keys grow along the sequence (scores of later tiles dwarf the running maximum, so the kernel's reference point
    # has to move tile after tile), then a stretch of strongly negative scores (whose probabilities underflow against
    # it), then small ones again.  Sec. 5 (the transformer fill job's attention); the oracle is the plain softmax.
    pf, dev = _mods()
    md = _md("bf16")
    B, d = 2, h * dh
    rng = np.random.default_rng(S + dh + int(causal))
    qkv = _rand(rng, (B, S, 3 * d), "bf16", 1.5)
    grow = np.concatenate([np.linspace(0.2, 9.0, S // 2), np.full(S // 4, -6.0), np.full(S - S // 2 - S // 4, 0.5)])
    qkv[:, :, d:2 * d] *= grow[None, :, None].astype(qkv.dtype)
    qkv = synth.round_to_bf16(qkv)
    dq = dev.storage_tensor(qkv, md)
    out = dev.empty_storage((B, S, d), md)
    lse = torch.empty((B, h, S), dtype=torch.float32, device="cuda")
    pf.pf_op_attention(md.dtype, dq.data_ptr(), out.data_ptr(), B, S, h, dh, causal, lse.data_ptr())
    torch.cuda.synchronize()
    q64 = qkv.astype(np.float64)
    q, k, v = (ot.split_heads(q64[..., i * d:(i + 1) * d], h) for i in range(3))
    ref = ot.merge_heads(ot.attention_probs(q, k, causal) @ v)
    got = dev.read_storage(out, md)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) < TOL["bf16"] / 2
    s = q @ k.transpose(0, 1, 3, 2) / np.sqrt(dh)
    if causal:
        s = np.where(np.triu(np.ones((S, S), dtype=bool), 1), -np.inf, s)
    mx = s.max(-1)
    ref_lse = mx + np.log(np.exp(s - mx[..., None]).sum(-1))
    assert np.abs(lse.cpu().numpy() - ref_lse).max() < 5e-2


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_embedding(dtype):
    pf, dev = _mods()
    md = _md(dtype)
    rng = np.random.default_rng(3)
    V, S, d, B = 1000, 37, 264, 3
    tok, pos = _rand(rng, (V, d), dtype), _rand(rng, (S, d), dtype)
    ids = rng.integers(0, V, size=(B, S), dtype=np.int32)
    dt, dp = dev.storage_tensor(tok, md), dev.storage_tensor(pos, md)
    di = dev.to_device(ids)
    x = dev.empty_storage((B, S, d), md)
    pf.pf_op_embed(md.dtype, di.data_ptr(), dt.data_ptr(), dp.data_ptr(), x.data_ptr(), B * S, S, d, V)
    torch.cuda.synchronize()
    ref = ot.embed(ids, dict(tok_emb=tok.astype(np.float64), pos_emb=pos.astype(np.float64)))
    assert rel_err(dev.read_storage(x, md), ref) < TOL[dtype] / 2


def _run_model(shape, params, inp, g=1, streamed=False, n_slots=0, cuts=None):
    """Runs the whole chain for one replica, optionally cut into chunks at node indices `cuts`."""
    pf, dev = _mods()
    m = dev.DeviceModel(shape, params, g=g, streamed=streamed, n_slots=n_slots)
    try:
        md = m.md
        if shape.vocab > 0:
            d_in = dev.to_device(inp.astype(np.int32))
        else:
            d_in = dev.storage_tensor(inp, md)
        d_out = dev.empty_storage((g, shape.batch, shape.seq_len, shape.d_model), md)
        m.set_io(d_in, 1, d_out, 1)
        nF = len(m.chain)
        edges = [0] + sorted(cuts or []) + [nF]
        st = torch.cuda.Stream()
        for a, b in zip(edges[:-1], edges[1:]):
            m.ctx.pf_fill_chunk_fwd(m.chunk(a, b), m.chain, stream=st.cuda_stream)
            m.ctx.pf_ctx_sync()          # a bubble boundary: everything drains, state stays in the context
        return dev.read_storage(d_out, md)
    finally:
        m.close()


def _oracle_model(shape, params, inp):
    P = ot.cast_params(params)
    x = inp if shape.vocab > 0 else inp.astype(np.float64)
    return ot.model_forward(x, P, shape.n_heads, shape.causal, shape.eps)


def test_cfg1_layer_fp32_full_size():
    shape = synth.WORKLOADS["cfg1"]
    params = synth.make_model_params(shape, seed=0)
    x = synth.make_hidden(shape, seed=1)
    got = _run_model(shape, params, x[None])
    ref = _oracle_model(shape, params, x)
    assert rel_err(got[0], ref) < TOL["f32"]
    # the layer alone (no final LayerNorm), through act_out of a one-node chunk
    pf, dev = _mods()
    m = dev.DeviceModel(shape, params)
    try:
        d_in = dev.storage_tensor(x, m.md)
        d_out = dev.empty_storage(x.shape, m.md)
        m.ctx.pf_fill_chunk_fwd(m.chunk(0, 1), m.chain, act_in=d_in.data_ptr(), act_out=d_out.data_ptr())
        m.ctx.pf_ctx_sync()
        ref1 = ot.layer_forward(x.astype(np.float64), ot.cast_params(params)["layers"][0], shape.n_heads)
        assert rel_err(dev.read_storage(d_out, m.md), ref1) < TOL["f32"]
    finally:
        m.close()


SMALL = [
    synth.ModelShape(3, 256, 4, 1024, 200, 3, 0, False, "bf16"),       # ragged sequence, encoder
    synth.ModelShape(2, 256, 2, 512, 160, 2, 500, True, "bf16"),       # d_head 128, causal, embedding
    synth.ModelShape(2, 64, 4, 256, 70, 2, 300, True, "f32"),          # d_head 16 generic path
    synth.ModelShape(2, 128, 2, 256, 130, 2, 0, True, "f32"),
]


@pytest.mark.parametrize("shape", SMALL, ids=lambda s: f"{s.dtype}-d{s.d_model}-h{s.n_heads}-S{s.seq_len}")
def test_small_models_whole_and_chunked(shape):
    params = synth.make_model_params(shape, seed=5)
    inp = synth.make_token_ids(shape, seed=6) if shape.vocab > 0 else synth.make_hidden(shape, seed=6)
    whole = _run_model(shape, params, inp[None])
    ref = _oracle_model(shape, params, inp)
    assert rel_err(whole[0], ref) < TOL[shape.dtype]
    nF = shape.n_layers + 1 + (1 if shape.vocab > 0 else 0)
    for cuts in ([1], [1, 2], list(range(1, nF))):
        part = _run_model(shape, params, inp[None], cuts=cuts)
        assert np.array_equal(part, whole), cuts        # inter-bubble context: cutting changes nothing


def test_teacher_forced_chunks_bf16():
    """Each chunk compared on its own: the checker starts from the GPU's chunk input."""
    pf, dev = _mods()
    shape = synth.ModelShape(4, 256, 4, 1024, 192, 2, 0, False, "bf16")
    params = synth.make_model_params(shape, seed=8)
    P = ot.cast_params(params)
    x = synth.make_hidden(shape, seed=9)
    m = dev.DeviceModel(shape, params)
    try:
        cur = dev.storage_tensor(x, m.md)
        for a, b in ((0, 1), (1, 3), (3, 4)):
            nxt = dev.empty_storage(x.shape, m.md)
            m.ctx.pf_fill_chunk_fwd(m.chunk(a, b), m.chain, act_in=cur.data_ptr(), act_out=nxt.data_ptr())
            m.ctx.pf_ctx_sync()
            ref = ot.model_forward(dev.read_storage(cur, m.md).astype(np.float64), P, shape.n_heads, False,
                                   shape.eps, layers=(a, b))
            assert rel_err(dev.read_storage(nxt, m.md), ref) < TOL["bf16"]
            cur = nxt
    finally:
        m.close()


def test_streamed_weights_and_microbatch_groups():
    shape = synth.ModelShape(5, 128, 2, 256, 96, 2, 400, True, "bf16")
    params = synth.make_model_params(shape, seed=10)
    g = 3
    ids = np.stack([synth.make_token_ids(shape, seed=20 + i) for i in range(g)])
    resident = _run_model(shape, params, ids, g=g)
    for n_slots in (2, 3):
        streamed = _run_model(shape, params, ids, g=g, streamed=True, n_slots=n_slots, cuts=[2, 3, 6])
        assert np.array_equal(streamed, resident)
    for i in range(g):
        assert rel_err(resident[i], _oracle_model(shape, params, ids[i])) < TOL["bf16"]


@pytest.mark.parametrize("own_stream", [False, True], ids=["ctx-stream", "caller-stream"])
def test_explicit_layer_loads_match_resident(own_stream):
    """Layers brought in by explicit pf_load_layer_async calls (the context's copy stream, or a stream of the
    caller's) before and between chunks: the streamed chunks find them in their slots and give the resident
    configuration's result bit for bit, also when a caller-stream copy follows an automatic prefetch into the
    same slot."""
    pf, dev = _mods()
    shape = synth.ModelShape(5, 128, 2, 256, 96, 2, 400, True, "bf16")
    params = synth.make_model_params(shape, seed=10)
    g = 2
    ids = np.stack([synth.make_token_ids(shape, seed=20 + i) for i in range(g)])
    resident = _run_model(shape, params, ids, g=g)
    n_slots = 3
    m = dev.DeviceModel(shape, params, g=g, streamed=True, n_slots=n_slots)
    try:
        d_in = dev.to_device(ids.astype(np.int32))
        d_out = dev.empty_storage((g, shape.batch, shape.seq_len, shape.d_model), m.md)
        m.set_io(d_in, 1, d_out, 1)
        st, cs = torch.cuda.Stream(), torch.cuda.Stream()
        copy = cs.cuda_stream if own_stream else None
        # before the first bubble: layers 0 and 1 wait in slots 0 and 1
        m.ctx.pf_load_layer_async(0, 0, copy)
        m.ctx.pf_load_layer_async(1, 1, copy)
        m.ctx.pf_fill_chunk_fwd(m.chunk(0, 3), m.chain, stream=st.cuda_stream)      # embed, layers 0 and 1
        # no synchronisation: the chunk's own prefetches (layers 2, 3) are in flight on the context's stream when
        # the caller replaces what slot 0 will hold next; the copy must queue behind them and behind the kernels
        m.ctx.pf_load_layer_async(4, 0, copy)
        m.ctx.pf_fill_chunk_fwd(m.chunk(3, 5), m.chain, stream=st.cuda_stream)      # layers 2 and 3
        m.ctx.pf_ctx_sync()
        m.ctx.pf_fill_chunk_fwd(m.chunk(5, len(m.chain)), m.chain, stream=st.cuda_stream)   # layer 4, final LN
        m.ctx.pf_ctx_sync()
        assert np.array_equal(dev.read_storage(d_out, m.md), resident)
        with pytest.raises(pf.PipeFillError) as e:
            m.ctx.pf_load_layer_async(5, 0, copy)
        assert e.value.code == pf.PF_ERR_ARG
        with pytest.raises(pf.PipeFillError) as e:
            m.ctx.pf_load_layer_async(0, n_slots, copy)
        assert e.value.code == pf.PF_ERR_ARG
    finally:
        m.close()


def test_chunk_error_paths_on_device():
    pf, dev = _mods()
    shape = SMALL[3]
    params = synth.make_model_params(shape, seed=5)
    m = dev.DeviceModel(shape, params)
    try:
        ch = m.chunk(0, 2)
        ch.mem_bytes = 1 << 40
        with pytest.raises(pf.PipeFillError) as e:
            m.ctx.pf_fill_chunk_fwd(ch, m.chain, cap_bytes=1 << 30)
        assert e.value.code == pf.PF_ERR_NOMEM               # refused before any launch
        with pytest.raises(pf.PipeFillError) as e:
            m.ctx.pf_fill_chunk_fwd(m.chunk(0, 1), m.chain)   # no input ring set
        assert e.value.code == pf.PF_ERR_STATE
        with pytest.raises(pf.PipeFillError) as e:
            m.ctx.pf_load_layer_async(0, 0)
        assert e.value.code == pf.PF_ERR_STATE               # configuration is resident
        with pytest.raises(pf.PipeFillError) as e:
            m.ctx.pf_fill_chunk_fwd(m.chunk(3, 2), m.chain)
        assert e.value.code == pf.PF_ERR_ARG
        small = torch.empty(1024, dtype=torch.uint8, device="cuda")
        with pytest.raises(pf.PipeFillError) as e:
            pf.Context(m.md, m.cfg, [b.data_ptr() for b in m.blobs], None, None, m.lnf_g.data_ptr(),
                       m.lnf_b.data_ptr(), (small.data_ptr() + 255) // 256 * 256, 512)
        assert e.value.code == pf.PF_ERR_NOMEM
    finally:
        m.close()


def test_timeline_small():
    """Emulated 1F1B stage with a placeholder main job: chunks run in their bubbles, results equal
    the unchunked run, accounting adds up."""
    pf, dev = _mods()
    shape = synth.ModelShape(4, 128, 2, 256, 128, 4, 300, False, "bf16")
    params = synth.make_model_params(shape, seed=12)
    n_rep = 4
    ids = np.stack([synth.make_token_ids(shape, seed=40 + i) for i in range(n_rep)])
    m = dev.DeviceModel(shape, params)
    try:
        d_in = dev.to_device(ids.astype(np.int32))
        d_out = dev.empty_storage((n_rep, 1, shape.batch, shape.seq_len, shape.d_model), m.md)
        m.set_io(d_in, n_rep, d_out, n_rep)
        st = torch.cuda.Stream()
        m.ctx.pf_profile_chain(m.chain, 1, 3, st.cuda_stream)
        assert all(n.dur_ns > 0 for n in m.chain)
        p, mm, stage, tf, tb = 3, 4, 1, 1_000_000, 2_000_000
        windows = pf.pf_schedule_1f1b(p, mm, stage, tf, tb, 1 << 30, True, 0)
        plan, n_plan, k = pf.pf_plan_bubbles(windows, m.chain, 800_000, 0, 0, raw=True)
        cursor = C.c_int32(0)
        main = torch.cuda.Stream()
        total_rep = 0
        for it in range(3):
            stats = pf.pf_timeline_run(m.ctx, None, None, p, mm, stage, tf, tb, windows, plan, n_plan, m.chain,
                                       cursor, st.cuda_stream, main.cuda_stream)
            assert stats["idle_ns"] == (p - 1) * (tf + tb)
            # a placeholder stage advances a scheduled clock: its forwards and backwards plus its idle windows
            assert stats["iter_ns"] == (mm + p - 1) * (tf + tb)
            assert 0 < stats["fill_busy_ns"]
            total_rep += stats["replicas_done"]
        assert total_rep >= 1
        got = dev.read_storage(d_out, m.md)
        done = min(total_rep, n_rep)
        for i in range(done):
            ref = _oracle_model(shape, params, ids[i])
            assert rel_err(got[i, 0], ref) < TOL["bf16"]
    finally:
        m.close()
