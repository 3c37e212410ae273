"""Pins for the compute checker: finite differences, an independent autograd cross-check with a
library's double-precision ops, and closed-form special cases."""
import numpy as np
import pytest

from oracle import transformer as ot
from paper_2410_07192_amd import synth

TINY = synth.ModelShape(n_layers=2, d_model=16, n_heads=2, d_ff=32, seq_len=5, batch=2,
                        vocab=11, causal=True, dtype="f32")


def tiny_params(shape=TINY, std=0.3, seed=3):
    return ot.cast_params(synth.make_model_params(shape, seed=seed, std=std))


def test_layernorm_and_gelu_identities():
    g = np.linspace(0.5, 1.5, 8)
    b = np.linspace(-1, 1, 8)
    y, _, _ = ot.layer_norm(np.full((3, 8), 4.2), g, b, 1e-5)
    assert np.allclose(y, b)                                  # constant row -> beta
    x = np.random.default_rng(0).standard_normal((4, 8)) * 3 + 1
    y, xhat, _ = ot.layer_norm(x, np.ones(8), np.zeros(8), 0.0)
    assert np.allclose(y.mean(-1), 0) and np.allclose(y.var(-1), 1)
    u = np.linspace(-6, 6, 101)
    assert ot.gelu(np.zeros(1))[0] == 0.0
    assert np.allclose(ot.gelu(u) - ot.gelu(-u), u)           # x Phi(x) + x Phi(-x)... = x
    assert abs(ot.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15   # Phi(1)
    h = 1e-6
    assert np.allclose((ot.gelu(u + h) - ot.gelu(u - h)) / (2 * h), ot.gelu_grad(u), atol=1e-8)


def test_zero_projections_give_identity():
    P = tiny_params()["layers"][0]
    for k in ("w_o", "b_o", "w_2", "b_2"):
        P[k] = np.zeros_like(P[k])
    x = np.random.default_rng(1).standard_normal((2, 5, 16))
    assert np.array_equal(ot.layer_forward(x, P, 2), x)


@pytest.mark.parametrize("causal", [False, True])
def test_zero_qk_gives_mean_of_values(causal):
    rng = np.random.default_rng(2)
    q = np.zeros((2, 2, 6, 4))
    k = rng.standard_normal((2, 2, 6, 4))
    v = rng.standard_normal((2, 2, 6, 4))
    A = ot.attention_probs(q, k, causal)
    assert np.allclose(A.sum(-1), 1.0)
    out = A @ v
    if causal:
        want = np.cumsum(v, axis=2) / np.arange(1, 7)[None, None, :, None]
    else:
        want = np.broadcast_to(v.mean(axis=2, keepdims=True), v.shape)
    assert np.allclose(out, want)


def test_causal_layer_ignores_the_future_and_encoder_does_not():
    P = tiny_params()["layers"][0]
    x = np.random.default_rng(4).standard_normal((1, 5, 16))
    x2 = x.copy()
    x2[0, 3] += np.linspace(-1.0, 1.0, 16)      # not a constant shift: LayerNorm would remove that
    y, y2 = ot.layer_forward(x, P, 2, causal=True), ot.layer_forward(x2, P, 2, causal=True)
    assert np.array_equal(y[0, :3], y2[0, :3]) and not np.allclose(y[0, 3:], y2[0, 3:])
    y, y2 = ot.layer_forward(x, P, 2, causal=False), ot.layer_forward(x2, P, 2, causal=False)
    assert not np.allclose(y[0, :3], y2[0, :3])


def test_batch_and_head_permutation_equivariance():
    P = tiny_params()["layers"][0]
    x = np.random.default_rng(5).standard_normal((3, 5, 16))
    y = ot.layer_forward(x, P, 2)
    assert np.allclose(ot.layer_forward(x[[2, 0, 1]], P, 2), y[[2, 0, 1]], atol=1e-14)
    # swapping the two heads' columns in W_qkv/b_qkv and rows in W_o leaves the layer unchanged
    perm = np.r_[8:16, 0:8]
    Q = dict(P)
    p3 = np.concatenate([perm, 16 + perm, 32 + perm])
    Q["w_qkv"], Q["b_qkv"], Q["w_o"] = P["w_qkv"][:, p3], P["b_qkv"][p3], P["w_o"][perm, :]
    assert np.allclose(ot.layer_forward(x, Q, 2), y, atol=1e-13)


def _torch_layer(x, P, n_heads, causal, eps):
    import torch
    import torch.nn.functional as F
    d = x.shape[-1]
    a = F.layer_norm(x, (d,), P["ln1_g"], P["ln1_b"], eps)
    qkv = F.linear(a, P["w_qkv"].T, P["b_qkv"])
    q, k, v = qkv.split(d, dim=-1)
    hs = lambda t: t.view(t.shape[0], t.shape[1], n_heads, d // n_heads).transpose(1, 2)
    o = F.scaled_dot_product_attention(hs(q), hs(k), hs(v), is_causal=causal)
    c = o.transpose(1, 2).reshape(x.shape)
    x1 = x + F.linear(c, P["w_o"].T, P["b_o"])
    b = F.layer_norm(x1, (d,), P["ln2_g"], P["ln2_b"], eps)
    return x1 + F.linear(F.gelu(F.linear(b, P["w_1"].T, P["b_1"])), P["w_2"].T, P["b_2"])


@pytest.mark.parametrize("causal", [False, True])
def test_layer_forward_backward_against_library_autograd(causal):
    import torch
    P = tiny_params()["layers"][0]
    rng = np.random.default_rng(6)
    x = rng.standard_normal((2, 5, 16))
    dy = rng.standard_normal((2, 5, 16))
    y, cache = ot.layer_forward(x, P, 2, causal, 1e-5, keep=True)
    dx, G = ot.layer_backward(dy, cache, P, 2)
    tP = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in P.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = _torch_layer(tx, tP, 2, causal, 1e-5)
    ty.backward(torch.tensor(dy))
    assert np.allclose(y, ty.detach().numpy(), atol=1e-12)
    assert np.allclose(dx, tx.grad.numpy(), atol=1e-11)
    for k in P:
        assert np.allclose(G[k], tP[k].grad.numpy(), atol=1e-11), k


def test_layer_gradients_by_central_differences():
    P = tiny_params()["layers"][0]
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 5, 16))
    dy = rng.standard_normal((2, 5, 16))
    y, cache = ot.layer_forward(x, P, 2, True, 1e-5, keep=True)
    dx, G = ot.layer_backward(dy, cache, P, 2)
    f = lambda xx, PP: float((ot.layer_forward(xx, PP, 2, True, 1e-5) * dy).sum())
    h = 1e-5
    for name in list(P) + ["x"]:
        arr = x if name == "x" else P[name]
        grad = dx if name == "x" else G[name]
        idxs = [tuple(rng.integers(0, s) for s in arr.shape) for _ in range(6)]
        for idx in idxs:
            old = arr[idx]
            arr[idx] = old + h
            fp = f(x, P)
            arr[idx] = old - h
            fm = f(x, P)
            arr[idx] = old
            num = (fp - fm) / (2 * h)
            assert abs(num - grad[idx]) < 1e-6 * max(1.0, abs(num)), (name, idx, num, grad[idx])


def test_model_loss_gradients_by_central_differences_and_checkpointing():
    params = tiny_params()
    ids = synth.make_token_ids(TINY, seed=9)
    loss, G = ot.model_loss_and_grads(ids, params, 2, True, 1e-5, checkpoint=False)
    loss2, G2 = ot.model_loss_and_grads(ids, params, 2, True, 1e-5, checkpoint=True)
    assert loss == loss2
    for k in ("tok_emb", "pos_emb", "lnf_g", "lnf_b"):
        assert np.array_equal(G[k], G2[k])
    for l in range(2):
        for k in G["layers"][l]:
            assert np.array_equal(G["layers"][l][k], G2["layers"][l][k])
    # loss of a uniform predictor is log(V): zero the final LN so logits are 0
    z = dict(params)
    z["lnf_g"], z["lnf_b"] = np.zeros(16), np.zeros(16)
    assert abs(ot.model_loss_and_grads(ids, z, 2)[0] - np.log(11)) < 1e-12
    rng = np.random.default_rng(10)
    h = 1e-5
    f = lambda: ot.model_loss_and_grads(ids, params, 2, True, 1e-5)[0]
    targets = [("tok_emb", params["tok_emb"], G["tok_emb"]), ("pos_emb", params["pos_emb"], G["pos_emb"]),
               ("lnf_g", params["lnf_g"], G["lnf_g"]),
               ("l0.w_qkv", params["layers"][0]["w_qkv"], G["layers"][0]["w_qkv"]),
               ("l1.w_2", params["layers"][1]["w_2"], G["layers"][1]["w_2"]),
               ("l0.ln1_b", params["layers"][0]["ln1_b"], G["layers"][0]["ln1_b"])]
    for name, arr, grad in targets:
        for _ in range(5):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            if name == "tok_emb":
                idx = (int(ids.reshape(-1)[rng.integers(0, ids.size)]), idx[1])
            old = arr[idx]
            arr[idx] = old + h; fp = f()
            arr[idx] = old - h; fm = f()
            arr[idx] = old
            num = (fp - fm) / (2 * h)
            assert abs(num - grad[idx]) < 2e-7 * max(1.0, abs(num) * 10), (name, idx, num, grad[idx])


def test_chunked_execution_equals_unchunked():
    shape = synth.ModelShape(4, 16, 2, 32, 5, 2, 0, False, "f32")
    params = ot.cast_params(synth.make_model_params(shape, seed=1, std=0.3))
    x = np.random.default_rng(12).standard_normal((2, 5, 16))
    whole = ot.model_forward(x, params, 2, layers=(0, 4))
    part = ot.model_forward(ot.model_forward(ot.model_forward(x, params, 2, layers=(0, 1)), params, 2,
                                             layers=(1, 3)), params, 2, layers=(3, 4))
    assert np.array_equal(whole, part)


def test_adam_first_step_closed_form_and_decay():
    g = np.array([0.5, -2.0, 1e-3, 0.0])
    th = np.ones(4)
    th1, m1, v1 = ot.adam_step(th, np.zeros(4), np.zeros(4), g, 1, lr=1e-2, eps=1e-8)
    assert np.allclose(th1, th - 1e-2 * g / (np.abs(g) + 1e-8), atol=1e-15)
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)
    # constant gradient: mhat = g and vhat = g^2 at every step
    th, m, v = np.ones(4), np.zeros(4), np.zeros(4)
    for t in range(1, 6):
        th, m, v = ot.adam_step(th, m, v, g, t, lr=1e-2)
    assert np.allclose(th, 1 - 5e-2 * g / (np.abs(g) + 1e-8), atol=1e-12)


def test_lm_loss_hand_worked_next_token_alignment():
    """Tied head, V = 3, S = 3, two sequences, logits chosen as logarithms of small integers so every softmax is a
    ratio of integers (R7: position t predicts token t+1, the last position has no target, mean over B(S-1)).
    Position 0 of sequence 0 holds p = (1/8, 2/8, 5/8) and must be scored on ids[0,1] = 0; a loss aligned with
    ids[0,0] = 2, or one that counts the last position, gives a different number."""
    E = np.eye(3)                                   # tied embedding = identity: logits are the hidden states
    L = np.log
    h = np.array([[[L(1), L(2), L(5)], [L(3), L(1), L(4)], [L(7), L(1), L(1)]],
                  [[L(2), L(1), L(1)], [L(1), L(1), L(2)], [L(1), L(9), L(1)]]])
    ids = np.array([[2, 0, 1], [1, 1, 2]])
    loss, dlogits = ot.lm_loss(h, E, ids)
    # targets: seq 0 -> (0, 1) with p = 1/8, 1/8; seq 1 -> (1, 2) with p = 1/4, 1/2
    assert abs(loss - (L(8) + L(8) + L(4) + L(2)) / 4) < 1e-15
    want = np.array([[[1 / 8 - 1, 2 / 8, 5 / 8], [3 / 8, 1 / 8 - 1, 4 / 8], [0, 0, 0]],
                     [[1 / 2, 1 / 4 - 1, 1 / 4], [1 / 4, 1 / 4, 1 / 2 - 1], [0, 0, 0]]]) / 4
    assert np.allclose(dlogits, want, atol=1e-15)


def test_embed_hand_worked():
    """x[b,t] = E[ids[b,t]] + P[t] (R5) on numbers that name their own row: token v -> (10v, 10v+1), position t ->
    (100t, 200t); the position table is longer than the sequence."""
    tok = np.array([[0., 1.], [10., 11.], [20., 21.], [30., 31.]])
    pos = np.array([[0., 0.], [100., 200.], [200., 400.], [300., 600.]])
    ids = np.array([[2, 0, 3], [1, 1, 0]])
    x = ot.embed(ids, dict(tok_emb=tok, pos_emb=pos))
    want = np.array([[[20., 21.], [100., 201.], [230., 431.]],
                     [[10., 11.], [110., 211.], [200., 401.]]])
    assert np.array_equal(x, want)
