"""The LayerNorm backward that takes no workspace (its partial sums live in a device array of the library's own),
through the C ABI, against the entry point that takes the workspace from the caller: two calls in a row, the second
smaller than the first, so the second finds the first's partial rows in the array.

dx: bit-identical (same kernel, same per-row arithmetic).  dg / db: bit-identical while every row has a workgroup of
its own (same partial rows, same summation order); with more rows than workgroups the two entry points may use
different workgroup counts, so they are compared within the fp32 tolerance of the gradient tests (1e-4 of the
tensor's maximum), and the widest row shape, whose workgroup count the array bounds at 128, is among the cases."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2410_07192_amd import synth        # noqa: E402


def _mods():
    from paper_2410_07192_amd import binding as pf
    from paper_2410_07192_amd import device as dev
    return pf, dev


def _case(pf, dev, dtype, rows, d, with_resid, seed):
    md = pf.pf_model_desc()
    md.dtype = pf.PF_DTYPE_BF16 if dtype == "bf16" else pf.PF_DTYPE_F32
    rng = np.random.default_rng(seed)
    rnd = lambda *s: (synth.round_to_bf16(rng.standard_normal(s).astype(np.float32)) if dtype == "bf16"
                      else rng.standard_normal(s).astype(np.float32))
    x, dy, res, g = rnd(rows, d), rnd(rows, d), rnd(rows, d), rnd(d)
    dx_, ddy, dres, dg_ = (dev.storage_tensor(a, md) for a in (x, dy, res, g))
    db_ = dev.storage_tensor(np.zeros(d, np.float32), md)
    y = dev.empty_storage((rows, d), md)
    mean = torch.empty(rows, dtype=torch.float32, device="cuda")
    rstd = torch.empty(rows, dtype=torch.float32, device="cuda")
    pf.pf_op_layernorm(md.dtype, dx_.data_ptr(), dg_.data_ptr(), db_.data_ptr(), y.data_ptr(), rows, d, 1e-5,
                       mean.data_ptr(), rstd.data_ptr())
    out = []
    for static in (False, True):
        dxo = dev.empty_storage((rows, d), md)
        acc_g = torch.full((d,), 2.0, dtype=torch.float32, device="cuda")
        acc_b = torch.full((d,), -1.0, dtype=torch.float32, device="cuda")
        args = (md.dtype, ddy.data_ptr(), dx_.data_ptr(), dg_.data_ptr(), mean.data_ptr(), rstd.data_ptr(),
                dres.data_ptr() if with_resid else None, dxo.data_ptr(), acc_g.data_ptr(), acc_b.data_ptr())
        if static:
            pf.pf_op_layernorm_bwd_static(*args, rows, d)
        else:
            partial = torch.empty(512 * 2 * d, dtype=torch.float32, device="cuda")
            pf.pf_op_layernorm_bwd(*args, partial.data_ptr(), rows, d)
        torch.cuda.synchronize()
        out.append((dxo.cpu().numpy().copy(), acc_g.cpu().numpy().copy(), acc_b.cpu().numpy().copy()))
    (dx0, g0, b0), (dx1, g1, b1) = out
    assert np.array_equal(dx0, dx1), (dtype, rows, d)
    blocks_static = min(512, (8 << 20) // (8 * d))
    if rows <= blocks_static:
        assert np.array_equal(g0, g1) and np.array_equal(b0, b1), (dtype, rows, d)
    else:
        for a, b in ((g0, g1), (b0, b1)):
            assert np.abs(a - b).max() <= 1e-4 * np.abs(a).max(), (dtype, rows, d)


# (first call, second smaller call): the second starts with the first's partial rows still in the array
PAIRS = [
    (("bf16", 2000, 1024, True), ("bf16", 300, 256, False)),
    (("f32", 700, 2048, False), ("f32", 129, 520, True)),
    (("bf16", 1030, 8192, True), ("bf16", 100, 8192, False)),      # 128 workgroups at the widest row
]


@pytest.mark.parametrize("first,second", PAIRS, ids=lambda c: f"{c[0]}-{c[1]}x{c[2]}")
def test_layernorm_bwd_without_workspace_matches(first, second):
    pf, dev = _mods()
    _case(pf, dev, *first, seed=1)
    _case(pf, dev, *second, seed=2)


def test_layernorm_bwd_without_workspace_rejects_oversize():
    pf, dev = _mods()
    t = torch.zeros(16384, dtype=torch.float32, device="cuda")
    p = t.data_ptr()
    with pytest.raises(pf.PipeFillError) as e:
        pf.pf_op_layernorm_bwd_static(pf.PF_DTYPE_F32, p, p, p, p, p, None, p, p, p, 1, 8200)
    assert e.value.code == pf.PF_ERR_ARG and "8192" in str(e.value)
    with pytest.raises(pf.PipeFillError) as e:
        pf.pf_op_layernorm_bwd_static(pf.PF_DTYPE_F32, p, p, p, p, p, None, p, p, p, 0, 64)
    assert e.value.code == pf.PF_ERR_ARG
