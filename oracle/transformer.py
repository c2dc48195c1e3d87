"""CPU oracle for the per-device Transformer training step.  TEST INFRASTRUCTURE.

This file is the slow, plain definition that the HIP library is checked
against.  Only the tests, the smoke check and the benchmark's cpu_baseline leg
may import it; the product never does, and it shares no code with the product.

What it defines (float64 throughout, numpy matmul as the only library step):

  * one pre-LayerNorm decoder block, forward and analytic backward: the
    decoder-only Transformer the paper trains (Fig. 1; Vaswani et al. for the
    attention and feed-forward definitions), with heads as the unit that
    tensor parallelism distributes (Sec. 3.2) -- so H*dh may differ from D and
    the un-reduced partial products are returned beside the outputs;
  * a stack of blocks, and the full model with token + learned position
    embeddings, a final LayerNorm and a tied output projection;
  * mean softmax cross-entropy and its gradient: the "loss" phase that Fig. 4
    separates from the forward and backward passes;
  * the Adam update (Table 1 caption; Kingma & Ba) with decoupled weight
    decay; wd = 0 is plain Adam.

Nothing is tiled, fused or reordered: scores are materialised as S x S
matrices, softmax is the two-pass form, and the backward pass is the chain
rule written out.  Weight matrices are [in, out] and applied as x @ W + b.
The fused QKV projection has columns [Q | K | V], head-major inside each.

Pins (tests, CPU only): central finite differences for every gradient,
float64 PyTorch library routines and autograd as a third party, and the
closed forms and invariants listed in each function's docstring.
"""
import math

import numpy as np

_SQRT_2_OVER_PI = math.sqrt(2.0 / math.pi)
_GELU_K = 0.044715


# --------------------------------------------------------------------------
# LayerNorm
# --------------------------------------------------------------------------
def layernorm_fwd(x, gamma, beta, eps):
    """h = (x - mean) / sqrt(var + eps) * gamma + beta over the last axis.

    Biased variance (divide by D).  With gamma=1, beta=0 each output row has
    mean 0 and variance var/(var+eps).  Returns (h, xhat, rstd).
    """
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * gamma + beta, xhat, rstd


def layernorm_bwd(dh, xhat, rstd, gamma):
    """Gradient of layernorm_fwd.  dx rows are orthogonal to 1 and to xhat."""
    g = dh * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True)
                 - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    D = dh.shape[-1]
    dgamma = (dh * xhat).reshape(-1, D).sum(axis=0)
    dbeta = dh.reshape(-1, D).sum(axis=0)
    return dx, dgamma, dbeta


# --------------------------------------------------------------------------
# GELU, both forms
# --------------------------------------------------------------------------
def _erf(u):
    from scipy.special import erf
    return erf(u)


def gelu(u, form="tanh"):
    """tanh form: u/2 (1 + tanh(c (u + k u^3))); erf form: u Phi(u).
    Both satisfy gelu(u) - gelu(-u) = u."""
    if form == "tanh":
        t = np.tanh(_SQRT_2_OVER_PI * (u + _GELU_K * u ** 3))
        return 0.5 * u * (1.0 + t)
    if form == "erf":
        return 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))
    raise ValueError(form)


def gelu_grad(u, form="tanh"):
    if form == "tanh":
        t = np.tanh(_SQRT_2_OVER_PI * (u + _GELU_K * u ** 3))
        return 0.5 * (1.0 + t) + 0.5 * u * (1.0 - t * t) * _SQRT_2_OVER_PI * (1.0 + 3.0 * _GELU_K * u * u)
    if form == "erf":
        cdf = 0.5 * (1.0 + _erf(u / math.sqrt(2.0)))
        pdf = np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
        return cdf + u * pdf
    raise ValueError(form)


# --------------------------------------------------------------------------
# Causal multi-head attention
# --------------------------------------------------------------------------
def causal_probs(q, k):
    """P[i, j] = softmax_j(q_i . k_j / sqrt(dh)) over j <= i; exactly 0 for j > i.

    q, k: [S, dh].  Two-pass softmax with the row maximum subtracted.
    Also returns the row log-sum-exp of the scaled, masked scores.
    """
    S, dh = q.shape
    s = (q @ k.T) / math.sqrt(dh)
    future = np.triu(np.ones((S, S), dtype=bool), k=1)
    s = np.where(future, -np.inf, s)
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=-1, keepdims=True)
    return e / z, (m + np.log(z))[:, 0]


def split_heads(a, H, dh):
    """[B, S, H*dh] -> [B, H, S, dh]."""
    B, S, _ = a.shape
    return a.reshape(B, S, H, dh).transpose(0, 2, 1, 3)


def merge_heads(a):
    """[B, H, S, dh] -> [B, S, H*dh]."""
    B, H, S, dh = a.shape
    return a.transpose(0, 2, 1, 3).reshape(B, S, H * dh)


def attention_fwd(qkv, H, dh):
    """qkv [B, S, 3*H*dh] -> (ctx [B, S, H*dh], lse [B, H, S])."""
    B, S, _ = qkv.shape
    Hd = H * dh
    q = split_heads(qkv[..., 0:Hd], H, dh)
    k = split_heads(qkv[..., Hd:2 * Hd], H, dh)
    v = split_heads(qkv[..., 2 * Hd:3 * Hd], H, dh)
    o = np.empty_like(q)
    lse = np.empty((B, H, S))
    for b in range(B):
        for h in range(H):
            P, lse[b, h] = causal_probs(q[b, h], k[b, h])
            o[b, h] = P @ v[b, h]
    return merge_heads(o), lse


def attention_bwd(dctx, qkv, H, dh):
    """Gradient of attention_fwd with respect to qkv (same packing)."""
    B, S, _ = qkv.shape
    Hd = H * dh
    q = split_heads(qkv[..., 0:Hd], H, dh)
    k = split_heads(qkv[..., Hd:2 * Hd], H, dh)
    v = split_heads(qkv[..., 2 * Hd:3 * Hd], H, dh)
    do = split_heads(dctx, H, dh)
    dq = np.empty_like(q)
    dk = np.empty_like(k)
    dv = np.empty_like(v)
    scale = 1.0 / math.sqrt(dh)
    for b in range(B):
        for h in range(H):
            P, _ = causal_probs(q[b, h], k[b, h])
            dv[b, h] = P.T @ do[b, h]
            dP = do[b, h] @ v[b, h].T
            dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
            dq[b, h] = (dS @ k[b, h]) * scale
            dk[b, h] = (dS.T @ q[b, h]) * scale
    return np.concatenate([merge_heads(dq), merge_heads(dk), merge_heads(dv)], axis=-1)


# --------------------------------------------------------------------------
# One decoder block
# --------------------------------------------------------------------------
def block_fwd(x, p, H, dh, gelu_form="tanh", eps=1e-5):
    """y = block(x) for x [B, S, D].

    x1 = x + ctx Wo + bo with ctx = causal attention of LN1(x) Wqkv + bqkv;
    y  = x1 + gelu(LN2(x1) W1 + b1) W2 + b2.
    The cache also carries p_attn = ctx Wo and p_mlp = a W2: the partial sums
    a tensor-parallel rank holds before the reduction over the model axis.
    """
    c = {"x": x, "H": H, "dh": dh, "gelu_form": gelu_form}
    c["h1"], c["xhat1"], c["rstd1"] = layernorm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    c["qkv"] = c["h1"] @ p["wqkv"] + p["bqkv"]
    c["ctx"], c["lse"] = attention_fwd(c["qkv"], H, dh)
    c["p_attn"] = c["ctx"] @ p["wo"]
    c["x1"] = x + c["p_attn"] + p["bo"]
    c["h2"], c["xhat2"], c["rstd2"] = layernorm_fwd(c["x1"], p["ln2_g"], p["ln2_b"], eps)
    c["u"] = c["h2"] @ p["w1"] + p["b1"]
    c["a"] = gelu(c["u"], gelu_form)
    c["p_mlp"] = c["a"] @ p["w2"]
    y = c["x1"] + c["p_mlp"] + p["b2"]
    return y, c


def _flat(a):
    return a.reshape(-1, a.shape[-1])


def block_bwd(dy, c, p):
    """Gradients of block_fwd.  Returns (dx, grads, partials).

    partials["dh2"] = du W1^T and partials["dh1"] = dqkv Wqkv^T are the
    input-gradient partial sums a tensor-parallel rank holds before reduction.
    """
    g = {}
    g["b2"] = _flat(dy).sum(axis=0)
    g["w2"] = _flat(c["a"]).T @ _flat(dy)
    da = dy @ p["w2"].T
    du = da * gelu_grad(c["u"], c["gelu_form"])
    g["b1"] = _flat(du).sum(axis=0)
    g["w1"] = _flat(c["h2"]).T @ _flat(du)
    dh2 = du @ p["w1"].T
    dx1_ln, g["ln2_g"], g["ln2_b"] = layernorm_bwd(dh2, c["xhat2"], c["rstd2"], p["ln2_g"])
    dx1 = dy + dx1_ln
    g["bo"] = _flat(dx1).sum(axis=0)
    g["wo"] = _flat(c["ctx"]).T @ _flat(dx1)
    dctx = dx1 @ p["wo"].T
    dqkv = attention_bwd(dctx, c["qkv"], c["H"], c["dh"])
    g["bqkv"] = _flat(dqkv).sum(axis=0)
    g["wqkv"] = _flat(c["h1"]).T @ _flat(dqkv)
    dh1 = dqkv @ p["wqkv"].T
    dx_ln, g["ln1_g"], g["ln1_b"] = layernorm_bwd(dh1, c["xhat1"], c["rstd1"], p["ln1_g"])
    dx = dx1 + dx_ln
    inter = {"dh1": dh1, "dh2": dh2, "da": da, "du": du, "dx1": dx1, "dctx": dctx, "dqkv": dqkv}
    return dx, g, inter


# --------------------------------------------------------------------------
# Stack of blocks
# --------------------------------------------------------------------------
def stack_fwd(x, params, H, dh, gelu_form="tanh", eps=1e-5):
    caches = []
    for p in params:
        x, c = block_fwd(x, p, H, dh, gelu_form, eps)
        caches.append(c)
    return x, caches


def stack_bwd(dy, caches, params):
    grads = [None] * len(params)
    for l in reversed(range(len(params))):
        dy, grads[l], _ = block_bwd(dy, caches[l], params[l])
    return dy, grads


# --------------------------------------------------------------------------
# Loss
# --------------------------------------------------------------------------
def cross_entropy(z, labels):
    """Mean over all N rows of logsumexp(z_n) - z_n[label_n]; dz = (softmax - onehot)/N.

    z [N, V], labels [N].  Each row of dz sums to 0; constant logits give ln V.
    """
    N = z.shape[0]
    m = z.max(axis=-1, keepdims=True)
    e = np.exp(z - m)
    s = e.sum(axis=-1, keepdims=True)
    lse = (m + np.log(s))[:, 0]
    rows = np.arange(N)
    loss = (lse - z[rows, labels]).mean()
    dz = e / s
    dz[rows, labels] -= 1.0
    return loss, dz / N


# --------------------------------------------------------------------------
# Full model: embeddings, blocks, final LayerNorm, tied output projection
# --------------------------------------------------------------------------
def model_fwd(p, tokens, H, dh, gelu_form="tanh", eps=1e-5):
    """logits[b, s] = LN_f(blocks(E[tok] + Ppos[s])) @ E^T.  Returns (z, cache)."""
    B, S = tokens.shape
    x0 = p["tok_emb"][tokens] + p["pos_emb"][:S][None, :, :]
    xL, caches = stack_fwd(x0, p["blocks"], H, dh, gelu_form, eps)
    hf, xhatf, rstdf = layernorm_fwd(xL, p["lnf_g"], p["lnf_b"], eps)
    z = hf @ p["tok_emb"].T
    return z, {"tokens": tokens, "caches": caches, "hf": hf, "xhatf": xhatf, "rstdf": rstdf, "xL": xL}


def model_loss_and_grads(p, tokens, labels, H, dh, gelu_form="tanh", eps=1e-5):
    """Training loss and the gradient of every parameter tensor."""
    B, S = tokens.shape
    D = p["tok_emb"].shape[1]
    z, c = model_fwd(p, tokens, H, dh, gelu_form, eps)
    loss, dz = cross_entropy(_flat(z), labels.reshape(-1))
    dz = dz.reshape(z.shape)
    g = {}
    g["tok_emb"] = _flat(dz).T @ _flat(c["hf"])            # output projection's share
    dhf = dz @ p["tok_emb"]
    dxL, g["lnf_g"], g["lnf_b"] = layernorm_bwd(dhf, c["xhatf"], c["rstdf"], p["lnf_g"])
    dx0, g["blocks"] = stack_bwd(dxL, c["caches"], p["blocks"])
    np.add.at(g["tok_emb"], tokens.reshape(-1), _flat(dx0))  # embedding lookup's share
    g["pos_emb"] = np.zeros_like(p["pos_emb"])
    g["pos_emb"][:S] = dx0.sum(axis=0)
    return loss, g, {"logits": z, "dx0": dx0}


# --------------------------------------------------------------------------
# Adam with decoupled weight decay
# --------------------------------------------------------------------------
def adamw(p, m, v, g, lr, beta1, beta2, eps, wd, t):
    """One update at step t >= 1.  Returns new (p, m, v).

    m' = b1 m + (1-b1) g;  v' = b2 v + (1-b2) g^2;
    p' = p (1 - lr wd) - lr (m'/(1-b1^t)) / (sqrt(v'/(1-b2^t)) + eps).
    At t=1 from zero moments: p' = p (1 - lr wd) - lr g / (|g| + eps).
    """
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    p = p * (1.0 - lr * wd) - lr * mhat / (np.sqrt(vhat) + eps)
    return p, m, v


# --------------------------------------------------------------------------
# Tensor-parallel share: the slice of a block's parameters one rank holds
# --------------------------------------------------------------------------
def tp_share(p, H, dh, rank, ranks):
    """Parameters of rank `rank` when heads and feed-forward columns are
    split `ranks` ways: its heads' columns of each of Q, K, V, the matching
    rows of Wo, and a contiguous slice of the feed-forward width.  LayerNorm
    parameters and the output biases bo, b2 are replicated."""
    Hd = H * dh
    hl = H // ranks
    cols = np.concatenate([np.arange(part * Hd + rank * hl * dh, part * Hd + (rank + 1) * hl * dh)
                           for part in range(3)])
    F = p["w1"].shape[1]
    fl = F // ranks
    fs = slice(rank * fl, (rank + 1) * fl)
    q = dict(p)
    q["wqkv"] = p["wqkv"][:, cols]
    q["bqkv"] = p["bqkv"][cols]
    q["wo"] = p["wo"][rank * hl * dh:(rank + 1) * hl * dh, :]
    q["w1"] = p["w1"][:, fs]
    q["b1"] = p["b1"][fs]
    q["w2"] = p["w2"][fs, :]
    return q, hl, cols, fs
