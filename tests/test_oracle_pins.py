"""Pins for the CPU oracle: what the mathematics fixes, independent of the oracle's own code.

Finite differences, closed forms, invariants, and float64 PyTorch library
routines / autograd as a third party.  A dropped term, a wrong sign or index,
or a transposed operand in the oracle fails at least one of these.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import transformer as orc
from workloads import BlockShape, ModelShape, make_block_inputs, make_model_inputs, get_config

TINY = BlockShape(B=1, S=8, D=16, H=2, dh=8, F=32, dtype="f32", sigma_w=0.3)
CFG1 = get_config("cfg1")


# ---------------------------------------------------------------- LayerNorm
def test_layernorm_zero_mean_unit_variance():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 7, 64)) * 3 + 2
    eps = 1e-5
    h, xhat, rstd = orc.layernorm_fwd(x, np.ones(64), np.zeros(64), eps)
    assert np.abs(h.mean(-1)).max() < 1e-12
    var = x.var(-1)
    assert np.allclose(h.var(-1), var / (var + eps), rtol=0, atol=1e-12)


def test_layernorm_matches_library():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((4, 9, 48)); g = rng.standard_normal(48); b = rng.standard_normal(48)
    h, _, _ = orc.layernorm_fwd(x, g, b, 1e-5)
    ref = TF.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), torch.from_numpy(b), 1e-5).numpy()
    assert np.abs(h - ref).max() < 1e-13


def test_layernorm_bwd_orthogonality_and_autograd():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, 5, 32)); g = rng.standard_normal(32); b = rng.standard_normal(32)
    dh = rng.standard_normal((3, 5, 32))
    # with eps = 0 the normalised row has unit second moment, so dx is exactly
    # orthogonal to both 1 and xhat; with eps > 0 the second holds to O(eps/var)
    _, xhat0, rstd0 = orc.layernorm_fwd(x, g, b, 0.0)
    dx0, _, _ = orc.layernorm_bwd(dh, xhat0, rstd0, g)
    assert np.abs(dx0.sum(-1)).max() < 1e-12
    assert np.abs((dx0 * xhat0).sum(-1)).max() < 1e-12
    _, xhat, rstd = orc.layernorm_fwd(x, g, b, 1e-5)
    dx, dg, db = orc.layernorm_bwd(dh, xhat, rstd, g)
    assert np.abs(dx.sum(-1)).max() < 1e-12
    xt = torch.from_numpy(x).requires_grad_(); gt = torch.from_numpy(g).requires_grad_(); bt = torch.from_numpy(b).requires_grad_()
    TF.layer_norm(xt, (32,), gt, bt, 1e-5).backward(torch.from_numpy(dh))
    assert np.abs(dx - xt.grad.numpy()).max() < 1e-12
    assert np.abs(dg - gt.grad.numpy()).max() < 1e-12
    assert np.abs(db - bt.grad.numpy()).max() < 1e-12


# --------------------------------------------------------------------- GELU
@pytest.mark.parametrize("form", ["tanh", "erf"])
def test_gelu_identities(form):
    u = np.linspace(-8, 8, 4001)
    assert np.abs(orc.gelu(u, form) - orc.gelu(-u, form) - u).max() < 1e-14
    assert orc.gelu(np.zeros(1), form)[0] == 0.0
    assert abs(orc.gelu_grad(np.zeros(1), form)[0] - 0.5) < 1e-15
    h = 1e-6
    fd = (orc.gelu(u + h, form) - orc.gelu(u - h, form)) / (2 * h)
    assert np.abs(fd - orc.gelu_grad(u, form)).max() < 1e-8
    approx = "tanh" if form == "tanh" else "none"
    ref = TF.gelu(torch.from_numpy(u), approximate=approx).numpy()
    assert np.abs(orc.gelu(u, form) - ref).max() < 1e-14


def test_gelu_forms_differ_by_known_gap():
    u = np.linspace(-8, 8, 160001)
    gap = np.abs(orc.gelu(u, "tanh") - orc.gelu(u, "erf")).max()
    assert 4.6e-4 < gap < 4.8e-4


# ---------------------------------------------------------------- attention
def test_softmax_rows_sum_to_one_and_mask_is_exact():
    rng = np.random.default_rng(4)
    q = rng.standard_normal((33, 16)) * 3; k = rng.standard_normal((33, 16)) * 3
    P, lse = orc.causal_probs(q, k)
    assert np.abs(P.sum(-1) - 1).max() < 1e-12
    assert np.all(np.triu(P, 1) == 0.0)
    assert P[0, 0] == 1.0
    s = q @ k.T / 4.0
    for i in (0, 5, 32):
        assert abs(lse[i] - math.log(np.exp(s[i, :i + 1]).sum())) < 1e-12


def test_attention_special_cases():
    rng = np.random.default_rng(5)
    B, S, H, dh = 2, 12, 3, 8
    Hd = H * dh
    qkv = rng.standard_normal((B, S, 3 * Hd))
    ctx, _ = orc.attention_fwd(qkv, H, dh)
    assert np.array_equal(ctx[:, 0], qkv[:, 0, 2 * Hd:])       # first row sees only itself
    one, _ = orc.attention_fwd(qkv[:, :1], H, dh)
    assert np.array_equal(one[:, 0], qkv[:, 0, 2 * Hd:])       # S = 1 is the identity on V
    flat = qkv.copy(); flat[..., Hd:2 * Hd] = 0.0              # all keys 0: uniform weights
    ctx, _ = orc.attention_fwd(flat, H, dh)
    v = flat[..., 2 * Hd:]
    run = np.cumsum(v, axis=1) / np.arange(1, S + 1)[None, :, None]
    assert np.abs(ctx - run).max() < 1e-13


def test_attention_matches_library_with_head_packing():
    rng = np.random.default_rng(6)
    B, S, H, dh = 2, 17, 3, 8
    Hd = H * dh
    qkv = rng.standard_normal((B, S, 3 * Hd))
    ctx, _ = orc.attention_fwd(qkv, H, dh)
    t = torch.from_numpy(qkv)
    q, k, v = [t[..., i * Hd:(i + 1) * Hd].reshape(B, S, H, dh).permute(0, 2, 1, 3) for i in range(3)]
    ref = TF.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3).reshape(B, S, Hd).numpy()
    assert np.abs(ctx - ref).max() < 1e-13


def test_attention_bwd_matches_autograd():
    rng = np.random.default_rng(7)
    B, S, H, dh = 2, 11, 2, 8
    Hd = H * dh
    qkv = rng.standard_normal((B, S, 3 * Hd)); dctx = rng.standard_normal((B, S, Hd))
    t = torch.from_numpy(qkv).requires_grad_()
    q, k, v = [t[..., i * Hd:(i + 1) * Hd].reshape(B, S, H, dh).permute(0, 2, 1, 3) for i in range(3)]
    out = TF.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3).reshape(B, S, Hd)
    out.backward(torch.from_numpy(dctx))
    assert np.abs(orc.attention_bwd(dctx, qkv, H, dh) - t.grad.numpy()).max() < 1e-12


# ------------------------------------------------------------ block: causal
def test_block_causality_forward_and_backward():
    p, x, dy = make_block_inputs(TINY, seed=3, generic=True)
    y, c = orc.block_fwd(x, p, TINY.H, TINY.dh)
    i = 4
    x2 = x.copy(); x2[:, i + 1:] += np.random.default_rng(0).standard_normal(x2[:, i + 1:].shape)
    y2, _ = orc.block_fwd(x2, p, TINY.H, TINY.dh)
    assert np.array_equal(y[:, :i + 1], y2[:, :i + 1])          # bit-identical, not just close
    assert np.abs(y[:, i + 1:] - y2[:, i + 1:]).max() > 1e-3
    d = np.zeros_like(dy); d[:, i] = dy[:, i]
    dx, _, _ = orc.block_bwd(d, c, p)
    assert np.all(dx[:, i + 1:] == 0.0)
    assert np.abs(dx[:, :i + 1]).max() > 1e-3


# ------------------------------------------------- block: finite differences
def _block_loss(x, p, sh, dy, form):
    y, _ = orc.block_fwd(x, p, sh.H, sh.dh, form)
    return float((y * dy).sum())


@pytest.mark.parametrize("sh,form", [(TINY, "tanh"), (TINY, "erf"), (CFG1, "tanh")])
def test_block_gradients_by_central_differences(sh, form):
    p, x, dy = make_block_inputs(sh, seed=0, generic=True)
    y, c = orc.block_fwd(x, p, sh.H, sh.dh, form)
    dx, g, _ = orc.block_bwd(dy, c, p)
    rng = np.random.default_rng(11)
    h = 1e-5
    # directional derivatives along random directions, one tensor at a time
    for name in ["x"] + list(p):
        base = x if name == "x" else p[name]
        d = rng.standard_normal(base.shape)
        def f(s):
            if name == "x":
                return _block_loss(x + s * d, p, sh, dy, form)
            q = dict(p); q[name] = p[name] + s * d
            return _block_loss(x, q, sh, dy, form)
        fd = (f(h) - f(-h)) / (2 * h)
        an = float(((dx if name == "x" else g[name]) * d).sum())
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, fd, an)
    # per-element spot checks
    for name in ["x", "wqkv", "bqkv", "wo", "w1", "w2", "ln1_g", "ln2_b"]:
        base = x if name == "x" else p[name]
        for _ in range(3):
            idx = tuple(int(rng.integers(0, n)) for n in base.shape)
            e = np.zeros(base.shape); e[idx] = 1.0
            def f(s):
                if name == "x":
                    return _block_loss(x + s * e, p, sh, dy, form)
                q = dict(p); q[name] = p[name] + s * e
                return _block_loss(x, q, sh, dy, form)
            fd = (f(h) - f(-h)) / (2 * h)
            an = float((dx if name == "x" else g[name])[idx])
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, idx, fd, an)


def test_key_bias_gradient_is_zero():
    p, x, dy = make_block_inputs(CFG1, seed=0, generic=True)
    _, c = orc.block_fwd(x, p, CFG1.H, CFG1.dh)
    _, g, _ = orc.block_bwd(dy, c, p)
    Hd = CFG1.Hd
    assert np.abs(g["bqkv"][Hd:2 * Hd]).max() <= 1e-12 * np.abs(g["bqkv"]).max()


# ------------------------------------------- block and model: torch autograd
def _torch_block(x, p, H, dh, form):
    B, S, D = x.shape
    Hd = H * dh
    h1 = TF.layer_norm(x, (D,), p["ln1_g"], p["ln1_b"], 1e-5)
    qkv = h1 @ p["wqkv"] + p["bqkv"]
    q, k, v = [qkv[..., i * Hd:(i + 1) * Hd].reshape(B, S, H, dh).permute(0, 2, 1, 3) for i in range(3)]
    ctx = TF.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3).reshape(B, S, Hd)
    x1 = x + ctx @ p["wo"] + p["bo"]
    h2 = TF.layer_norm(x1, (D,), p["ln2_g"], p["ln2_b"], 1e-5)
    a = TF.gelu(h2 @ p["w1"] + p["b1"], approximate="tanh" if form == "tanh" else "none")
    return x1 + a @ p["w2"] + p["b2"]


@pytest.mark.parametrize("form", ["tanh", "erf"])
def test_block_matches_torch_autograd(form):
    sh = CFG1
    p, x, dy = make_block_inputs(sh, seed=0, generic=True)
    y, c = orc.block_fwd(x, p, sh.H, sh.dh, form)
    dx, g, _ = orc.block_bwd(dy, c, p)
    tp = {k: torch.from_numpy(v).requires_grad_() for k, v in p.items()}
    tx = torch.from_numpy(x).requires_grad_()
    ty = _torch_block(tx, tp, sh.H, sh.dh, form)
    ty.backward(torch.from_numpy(dy))
    assert np.abs(y - ty.detach().numpy()).max() < 1e-12
    assert np.abs(dx - tx.grad.numpy()).max() <= 1e-11 * np.abs(dx).max()
    for k in p:
        ref = tp[k].grad.numpy()
        assert np.abs(g[k] - ref).max() <= 1e-11 * max(np.abs(ref).max(), 1e-3), k


def test_wide_share_shape_matches_torch_autograd():
    """H*dh != D: one tensor-parallel rank's local block."""
    sh = BlockShape(B=2, S=16, D=48, H=2, dh=8, F=40, dtype="f32", sigma_w=0.2)
    p, x, dy = make_block_inputs(sh, seed=5, generic=True)
    y, c = orc.block_fwd(x, p, sh.H, sh.dh)
    dx, g, _ = orc.block_bwd(dy, c, p)
    tp = {k: torch.from_numpy(v).requires_grad_() for k, v in p.items()}
    tx = torch.from_numpy(x).requires_grad_()
    ty = _torch_block(tx, tp, sh.H, sh.dh, "tanh")
    ty.backward(torch.from_numpy(dy))
    assert np.abs(y - ty.detach().numpy()).max() < 1e-12
    assert np.abs(dx - tx.grad.numpy()).max() < 1e-11
    for k in p:
        assert np.abs(g[k] - tp[k].grad.numpy()).max() < 1e-11, k


MODEL_TINY = ModelShape(BlockShape(B=2, S=12, D=16, H=2, dh=8, F=32, dtype="f32", sigma_w=0.2, L=2), V=37, S_max=16)


def test_model_loss_and_grads_match_torch_autograd():
    ms = MODEL_TINY; sh = ms.blk
    p, tok, lab = make_model_inputs(ms, seed=1, generic=True)
    loss, g, _ = orc.model_loss_and_grads(p, tok, lab, sh.H, sh.dh)
    tp = {k: torch.from_numpy(v).requires_grad_() for k, v in p.items() if k != "blocks"}
    tb = [{k: torch.from_numpy(v).requires_grad_() for k, v in bp.items()} for bp in p["blocks"]]
    ttok = torch.from_numpy(tok.astype(np.int64))
    x = TF.embedding(ttok, tp["tok_emb"]) + tp["pos_emb"][:sh.S]
    for bp in tb:
        x = _torch_block(x, bp, sh.H, sh.dh, "tanh")
    z = TF.layer_norm(x, (sh.D,), tp["lnf_g"], tp["lnf_b"], 1e-5) @ tp["tok_emb"].T
    tl = TF.cross_entropy(z.reshape(-1, ms.V), torch.from_numpy(lab.astype(np.int64)).reshape(-1))
    tl.backward()
    assert abs(loss - tl.item()) < 1e-12
    for k in tp:
        assert np.abs(g[k] - tp[k].grad.numpy()).max() < 1e-12, k
    for l in range(sh.L):
        for k in tb[l]:
            assert np.abs(g["blocks"][l][k] - tb[l][k].grad.numpy()).max() < 1e-12, (l, k)


def test_model_gradients_by_central_differences():
    ms = MODEL_TINY; sh = ms.blk
    p, tok, lab = make_model_inputs(ms, seed=2, generic=True)
    _, g, _ = orc.model_loss_and_grads(p, tok, lab, sh.H, sh.dh)
    rng = np.random.default_rng(5)
    h = 1e-5
    for name in ["tok_emb", "pos_emb", "lnf_g", "lnf_b"]:
        d = rng.standard_normal(p[name].shape)
        def f(s):
            q = dict(p); q[name] = p[name] + s * d
            z, _ = orc.model_fwd(q, tok, sh.H, sh.dh)
            return orc.cross_entropy(z.reshape(-1, ms.V), lab.reshape(-1))[0]
        # fourth-order central difference: the loss curves sharply along
        # embedding directions (LayerNorm rescales the 0.02-sized rows)
        fd = (8 * (f(h) - f(-h)) - (f(2 * h) - f(-2 * h))) / (12 * h)
        an = float((g[name] * d).sum())
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, fd, an)


# ------------------------------------------------------------ cross-entropy
def test_cross_entropy_invariants_and_library():
    rng = np.random.default_rng(8)
    N, V = 19, 51
    z = rng.standard_normal((N, V)) * 4; y = rng.integers(0, V, N)
    loss, dz = orc.cross_entropy(z, y)
    assert np.abs(dz.sum(-1)).max() < 1e-15
    zt = torch.from_numpy(z).requires_grad_()
    ref = TF.cross_entropy(zt, torch.from_numpy(y)); ref.backward()
    assert abs(loss - ref.item()) < 1e-13
    assert np.abs(dz - zt.grad.numpy()).max() < 1e-15
    V = 51200
    loss, _ = orc.cross_entropy(np.full((3, V), 0.7), np.array([0, 5, V - 1]))
    assert abs(loss - math.log(V)) < 1e-12 and abs(loss - 10.8435) < 1e-4


# -------------------------------------------------------------------- AdamW
def test_adamw_first_step_closed_form():
    rng = np.random.default_rng(9)
    p = rng.standard_normal(1000); g = rng.standard_normal(1000) * 10
    lr, b1, b2, eps, wd = 1e-3, 0.9, 0.999, 1e-8, 0.01
    p1, m1, v1 = orc.adamw(p, np.zeros(1000), np.zeros(1000), g, lr, b1, b2, eps, wd, 1)
    assert np.abs(p1 - (p * (1 - lr * wd) - lr * g / (np.abs(g) + eps))).max() < 1e-15
    assert np.allclose(m1, 0.1 * g, rtol=1e-14) and np.allclose(v1, 0.001 * g * g, rtol=1e-12)


def test_adamw_constant_gradient_has_constant_corrected_moments():
    g = np.array([0.3, -2.0, 5.0]); p = np.zeros(3); m = np.zeros(3); v = np.zeros(3)
    lr = 1e-2
    for t in range(1, 8):
        pn, m, v = orc.adamw(p, m, v, g, lr, 0.9, 0.999, 0.0, 0.0, t)
        assert np.allclose(m / (1 - 0.9 ** t), g, rtol=1e-13)
        assert np.allclose(v / (1 - 0.999 ** t), g * g, rtol=1e-12)
        assert np.allclose(pn - p, -lr * np.sign(g), rtol=1e-12)
        p = pn


def test_adamw_matches_library_over_several_steps():
    rng = np.random.default_rng(10)
    p0 = rng.standard_normal(257); gs = [rng.standard_normal(257) for _ in range(4)]
    tp = torch.from_numpy(p0.copy()).requires_grad_()
    opt = torch.optim.AdamW([tp], lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    p, m, v = p0.copy(), np.zeros(257), np.zeros(257)
    for t, g in enumerate(gs, 1):
        tp.grad = torch.from_numpy(g.copy()); opt.step()
        p, m, v = orc.adamw(p, m, v, g, 1e-3, 0.9, 0.999, 1e-8, 0.01, t)
        assert np.abs(p - tp.detach().numpy()).max() < 1e-14


# -------------------------------------------- tensor-parallel sum identity
@pytest.mark.parametrize("ranks", [2, 4])
def test_rank_partials_sum_to_unsplit_block(ranks):
    sh = CFG1
    p, x, dy = make_block_inputs(sh, seed=0, generic=True)
    y, c = orc.block_fwd(x, p, sh.H, sh.dh)
    dx, g, it = orc.block_bwd(dy, c, p)
    pa = np.zeros_like(x); gw = {k: np.zeros_like(v) for k, v in g.items()}
    for r in range(ranks):
        q, hl, cols, fs = orc.tp_share(p, sh.H, sh.dh, r, ranks)
        h1 = c["h1"]
        qkv = h1 @ q["wqkv"] + q["bqkv"]
        ctx, _ = orc.attention_fwd(qkv, hl, sh.dh)
        pa += ctx @ q["wo"]
        gw["wqkv"][:, cols] = h1.reshape(-1, sh.D).T @ orc.attention_bwd(it["dx1"] @ q["wo"].T, qkv, hl, sh.dh).reshape(-1, 3 * hl * sh.dh)
    assert np.abs(pa - c["p_attn"]).max() < 1e-12
    assert np.abs(gw["wqkv"] - g["wqkv"]).max() < 1e-11
    # MLP half: feed every rank the reduced x1, sum the partial products
    pm = np.zeros_like(x); dh2 = np.zeros_like(x)
    for r in range(ranks):
        q, hl, cols, fs = orc.tp_share(p, sh.H, sh.dh, r, ranks)
        u = c["h2"] @ q["w1"] + q["b1"]
        pm += orc.gelu(u) @ q["w2"]
        du = (dy @ q["w2"].T) * orc.gelu_grad(u)
        dh2 += du @ q["w1"].T
    assert np.abs(pm - c["p_mlp"]).max() < 1e-12
    assert np.abs(dh2 - it["dh2"]).max() < 1e-11
