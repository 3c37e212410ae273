"""CPU checker for the fill-job compute: transformer layer forward / backward, the model
around it, the training loss and Adam.  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this file; the
product path never does, and it shares no code with the HIP library.

The paper delegates fill-job execution to an existing framework (Sec. 4.5) and gives no model
internals; what is computed here is the textbook definition of a pre-LayerNorm transformer
written out with NumPy, in float64 unless another dtype is asked for:

    x1 = x  + Attn(LN1(x)) W_o + b_o
    y  = x1 + GELU(LN2(x1) W_1 + b_1) W_2 + b_2

LayerNorm uses the biased variance and eps inside the square root; GELU is the exact erf form;
attention is softmax(Q K^T / sqrt(d_head) [+ causal mask]) V per head; weights are
[in_features, out_features]; Q, K, V are the three column blocks of the fused projection and
head i owns columns i*d_head .. (i+1)*d_head of each block.  A library matmul and erf serve as
steps; there is no blocking, fusion or reordering.

Pins (tests/test_oracle_transformer.py): central finite differences for every gradient, an
independent autograd cross-check with a library's double-precision ops, closed-form special
cases (zero projections -> identity, W_q=W_k=0 -> (prefix) mean of V, causal independence of
the future, LayerNorm of a constant row, GELU identities, first Adam step).  End-to-end
accuracy on real data is parity unpinned: there are no datasets or trained weights here.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

SQRT2 = np.sqrt(2.0)
SQRT2PI = np.sqrt(2.0 * np.pi)


def layer_norm(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * g + b, xhat, rstd


def layer_norm_backward(dy, xhat, rstd, g):
    dxhat = dy * g
    dx = (dxhat - dxhat.mean(axis=-1, keepdims=True)
          - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True)) * rstd
    red = tuple(range(dy.ndim - 1))
    return dx, (dy * xhat).sum(axis=red), dy.sum(axis=red)


def gelu(u):
    return 0.5 * u * (1.0 + erf(u / SQRT2))


def gelu_grad(u):
    return 0.5 * (1.0 + erf(u / SQRT2)) + u * np.exp(-0.5 * u * u) / SQRT2PI


def split_heads(t, n_heads):
    b, s, d = t.shape
    return t.reshape(b, s, n_heads, d // n_heads).transpose(0, 2, 1, 3)


def merge_heads(t):
    b, h, s, dh = t.shape
    return t.transpose(0, 2, 1, 3).reshape(b, s, h * dh)


def attention_probs(q, k, causal):
    """softmax(q k^T / sqrt(d_head)) with max subtraction; causal: key j > query i masked."""
    dh = q.shape[-1]
    s = q @ k.transpose(0, 1, 3, 2) / np.sqrt(dh)
    if causal:
        S = s.shape[-1]
        mask = np.triu(np.ones((S, S), dtype=bool), k=1)
        s = np.where(mask, -np.inf, s)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def layer_forward(x, P, n_heads, causal=False, eps=1e-5, keep=False):
    """One pre-LN layer.  x: [B,S,d].  Returns y, or (y, cache) when keep is set."""
    d = x.shape[-1]
    a, xhat1, rstd1 = layer_norm(x, P["ln1_g"], P["ln1_b"], eps)
    qkv = a @ P["w_qkv"] + P["b_qkv"]
    q, k, v = (split_heads(qkv[..., i * d:(i + 1) * d], n_heads) for i in range(3))
    A = attention_probs(q, k, causal)
    c = merge_heads(A @ v)
    x1 = x + c @ P["w_o"] + P["b_o"]
    bb, xhat2, rstd2 = layer_norm(x1, P["ln2_g"], P["ln2_b"], eps)
    u = bb @ P["w_1"] + P["b_1"]
    gl = gelu(u)
    y = x1 + gl @ P["w_2"] + P["b_2"]
    if not keep:
        return y
    cache = dict(x=x, a=a, xhat1=xhat1, rstd1=rstd1, q=q, k=k, v=v, A=A, c=c, x1=x1,
                 bb=bb, xhat2=xhat2, rstd2=rstd2, u=u, gl=gl)
    return y, cache


def _flat(t):
    return t.reshape(-1, t.shape[-1])


def layer_backward(dy, cache, P, n_heads):
    """Gradients of the layer w.r.t. its input and every parameter, given dL/dy."""
    C = cache
    G = {}
    d = dy.shape[-1]
    dh = d // n_heads
    # y = x1 + gelu(u) W_2 + b_2
    G["w_2"] = _flat(C["gl"]).T @ _flat(dy)
    G["b_2"] = _flat(dy).sum(axis=0)
    du = (dy @ P["w_2"].T) * gelu_grad(C["u"])
    G["w_1"] = _flat(C["bb"]).T @ _flat(du)
    G["b_1"] = _flat(du).sum(axis=0)
    dbb = du @ P["w_1"].T
    dln2, G["ln2_g"], G["ln2_b"] = layer_norm_backward(dbb, C["xhat2"], C["rstd2"], P["ln2_g"])
    dx1 = dy + dln2
    # x1 = x + c W_o + b_o
    G["w_o"] = _flat(C["c"]).T @ _flat(dx1)
    G["b_o"] = _flat(dx1).sum(axis=0)
    do = split_heads(dx1 @ P["w_o"].T, n_heads)
    A, q, k, v = C["A"], C["q"], C["k"], C["v"]
    dA = do @ v.transpose(0, 1, 3, 2)
    dv = A.transpose(0, 1, 3, 2) @ do
    ds = A * (dA - (dA * A).sum(axis=-1, keepdims=True))
    dq = ds @ k / np.sqrt(dh)
    dk = ds.transpose(0, 1, 3, 2) @ q / np.sqrt(dh)
    dqkv = np.concatenate([merge_heads(dq), merge_heads(dk), merge_heads(dv)], axis=-1)
    G["w_qkv"] = _flat(C["a"]).T @ _flat(dqkv)
    G["b_qkv"] = _flat(dqkv).sum(axis=0)
    da = dqkv @ P["w_qkv"].T
    dln1, G["ln1_g"], G["ln1_b"] = layer_norm_backward(da, C["xhat1"], C["rstd1"], P["ln1_g"])
    return dx1 + dln1, G


def cast_params(params, dtype=np.float64):
    out = {}
    for k, v in params.items():
        if k == "layers":
            out[k] = [{n: np.asarray(a, dtype=dtype) for n, a in L.items()} for L in v]
        else:
            out[k] = np.asarray(v, dtype=dtype)
    return out


def embed(ids, params):
    """x[b,t] = E[id[b,t]] + P[t]   (token plus learned position embedding)."""
    S = ids.shape[1]
    return params["tok_emb"][ids] + params["pos_emb"][:S][None, :, :]


def model_forward(inp, params, n_heads, causal=False, eps=1e-5, layers=None):
    """Embedding (if inp holds integer ids) -> layers -> final LayerNorm.  `layers` may give a
    (begin, end) range to run only part of the stack on hidden states (no embed, no final LN)."""
    if layers is not None:
        x = inp
        for l in range(*layers):
            x = layer_forward(x, params["layers"][l], n_heads, causal, eps)
        return x
    x = embed(inp, params) if np.issubdtype(inp.dtype, np.integer) else inp
    for P in params["layers"]:
        x = layer_forward(x, P, n_heads, causal, eps)
    return layer_norm(x, params["lnf_g"], params["lnf_b"], eps)[0]


def lm_loss(h, tok_emb, ids):
    """Mean next-token cross-entropy with the output projection tied to the token embedding:
    logits[b,t] = h[b,t] E^T predicts ids[b,t+1]; the last position of a sequence has no target.
    Returns (loss, dlogits) with dlogits = d loss / d logits (zero rows where there is no target)."""
    Bn, S, _ = h.shape
    logits = h @ tok_emb.T
    z = logits - logits.max(axis=-1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=-1, keepdims=True))
    tgt = ids[:, 1:]
    n = Bn * (S - 1)
    bi, ti = np.meshgrid(np.arange(Bn), np.arange(S - 1), indexing="ij")
    loss = -logp[bi, ti, tgt].sum() / n
    dlogits = np.exp(logp)
    dlogits[bi, ti, tgt] -= 1.0
    dlogits[:, S - 1, :] = 0.0
    return loss, dlogits / n


def model_loss_and_grads(ids, params, n_heads, causal=True, eps=1e-5, checkpoint=False):
    """Forward, loss and the gradient of every parameter for one microbatch of token ids.
    checkpoint=True keeps only each layer's input and recomputes the layer in the backward."""
    x = embed(ids, params)
    saved = []
    for P in params["layers"]:
        if checkpoint:
            saved.append(x)
            x = layer_forward(x, P, n_heads, causal, eps)
        else:
            x, cache = layer_forward(x, P, n_heads, causal, eps, keep=True)
            saved.append(cache)
    h, xhat, rstd = layer_norm(x, params["lnf_g"], params["lnf_b"], eps)
    loss, dlogits = lm_loss(h, params["tok_emb"], ids)
    G = {"layers": [None] * len(params["layers"])}
    G["tok_emb"] = _flat(dlogits).T @ _flat(h)
    dh = dlogits @ params["tok_emb"]
    dx, G["lnf_g"], G["lnf_b"] = layer_norm_backward(dh, xhat, rstd, params["lnf_g"])
    for l in reversed(range(len(params["layers"]))):
        P = params["layers"][l]
        if checkpoint:
            _, cache = layer_forward(saved[l], P, n_heads, causal, eps, keep=True)
        else:
            cache = saved[l]
        dx, G["layers"][l] = layer_backward(dx, cache, P, n_heads)
    np.add.at(G["tok_emb"], ids.reshape(-1), _flat(dx))
    G["pos_emb"] = dx.sum(axis=0)
    return loss, G


def adam_step(theta, m, v, g, t, lr=1e-4, b1=0.9, b2=0.999, eps=1e-8):
    """Adam with bias correction, no weight decay; t is the 1-based step number.
    m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;  theta <- theta - lr * mhat / (sqrt(vhat) + eps)."""
    m = b1 * m + (1.0 - b1) * g
    v = b2 * v + (1.0 - b2) * g * g
    mhat = m / (1.0 - b1 ** t)
    vhat = v / (1.0 - b2 ** t)
    return theta - lr * mhat / (np.sqrt(vhat) + eps), m, v
