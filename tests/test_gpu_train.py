"""Parity of fax_train_step (embedding, blocks, final LayerNorm, tied output projection, mean
cross-entropy, all gradients, AdamW) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2204_06514_amd as fax
from oracle import transformer as orc
from workloads import BlockShape, ModelShape, make_model_inputs, PARAM_NAMES
from workloads.configs import ADAMW_DEFAULT
from helpers import DEV, TDTYPE, to_dev, to_np, err, tol, dims_of, adamw_step_report, bqkv_keep

pytestmark = pytest.mark.gpu

TOP = ("tok_emb", "pos_emb", "lnf_g", "lnf_b")


def _dev_params(p, dtype):
    d = {k: to_dev(p[k], dtype) for k in TOP}
    d["blocks"] = [{k: to_dev(bp[k], dtype) for k in PARAM_NAMES} for bp in p["blocks"]]
    return d


def _like(d, fill=None, dtype=torch.float32, src=None):
    def mk(t, s):
        if src is not None:
            return s.to(dtype).clone()
        return torch.full(t.shape, fill, dtype=dtype, device=DEV)
    out = {k: mk(d[k], src[k] if src else None) for k in TOP}
    out["blocks"] = [{k: mk(b[k], src["blocks"][i][k] if src else None) for k in PARAM_NAMES}
                     for i, b in enumerate(d["blocks"])]
    return out


def update_failures(ms, p, g_ref, master, m, v):
    """First AdamW step of every tensor of the model against the oracle's (moments, displacement,
    and that there is one); {} when all agree."""
    sh = ms.blk
    bad = {}
    for name, get in _walk(master):
        keep = bqkv_keep(sh.Hd) if name.endswith("bqkv") else None
        r = adamw_step_report(to_np(get(master)), to_np(get(m)), to_np(get(v)), get(p), get(g_ref), ADAMW_DEFAULT,
                              keep=keep, dtype=sh.dtype)
        if r:
            bad[name] = r
    return bad


def run_train_step(ms, p, tok, lab, update, step=1, flags=0):
    sh = ms.blk
    md = fax.FaxModelDims(dims_of(sh), sh.L, ms.V, ms.S_max, flags | (0 if update else fax.FAX_FLAG_SKIP_UPDATE))
    params = _dev_params(p, sh.dtype)
    if sh.dtype == "f32":
        master = params                       # one fp32 copy, updated in place
    else:
        master = _like(params, src=params)    # fp32 master copies of the bf16 parameters
    m = _like(params, 0.0); v = _like(params, 0.0); grads = _like(params, 7.0)   # 7: must be overwritten
    wsb = fax.fax_train_workspace_bytes(md)
    ws = torch.empty(wsb, dtype=torch.uint8, device=DEV)
    loss = torch.zeros(4, device=DEV)
    hp = fax.FaxAdamW(**ADAMW_DEFAULT)
    fax.fax_train_step(md, params, master, m, v, grads, torch.from_numpy(tok).to(DEV), torch.from_numpy(lab).to(DEV),
                       hp, step, loss, ws, wsb)
    torch.cuda.synchronize()
    return loss[0].item(), params, master, m, v, grads


def _walk(d):
    for k in TOP:
        yield k, (lambda t, k=k: t[k])
    for l in range(len(d["blocks"])):
        for k in PARAM_NAMES:
            yield "blocks[%d].%s" % (l, k), (lambda t, l=l, k=k: t["blocks"][l][k])


CASES = [
    ModelShape(BlockShape(B=2, S=24, D=32, H=2, dh=16, F=64, dtype="f32", sigma_w=0.1, L=2), V=97, S_max=32),
    ModelShape(BlockShape(B=2, S=128, D=128, H=2, dh=64, F=256, dtype="bf16", sigma_w=0.05, L=2), V=512, S_max=128),
    ModelShape(BlockShape(B=1, S=40, D=72, H=3, dh=24, F=100, dtype="bf16", sigma_w=0.05, L=1), V=333, S_max=48),
]


@pytest.mark.parametrize("ms", CASES, ids=lambda m: "%s_D%d_V%d" % (m.blk.dtype, m.blk.D, m.V))
def test_train_step_gradients_then_update(ms):
    sh = ms.blk
    p, tok, lab = make_model_inputs(ms, seed=3, generic=True)
    loss_ref, g_ref, _ = orc.model_loss_and_grads(p, tok, lab, sh.H, sh.dh, sh.gelu, sh.ln_eps)
    # gradients only
    loss, params, _, _, _, grads = run_train_step(ms, p, tok, lab, update=False)
    assert abs(loss - loss_ref) <= (1e-5 if sh.dtype == "f32" else 2e-3) * abs(loss_ref)
    t = tol(sh.dtype)
    bad = {}
    for name, get in _walk(grads):
        e = err(to_np(get(grads)), get(g_ref), sh.dtype)
        if not e <= t:
            bad[name] = e
    assert not bad, bad
    for name, get in _walk(params):   # parameters untouched
        assert np.array_equal(to_np(get(params)), get(p)), name
    # full step: moments, displacement of every element and its presence against the oracle's AdamW
    loss, params, master, m, v, grads = run_train_step(ms, p, tok, lab, update=True)
    bad = update_failures(ms, p, g_ref, master, m, v)
    assert not bad, bad
    if sh.dtype == "bf16":
        for name, get in _walk(master):
            assert torch.equal(get(params), get(master).to(torch.bfloat16)), name


def test_train_step_pos_rows_beyond_sequence_get_zero_gradient():
    ms = CASES[2]
    p, tok, lab = make_model_inputs(ms, seed=5)
    _, _, _, _, _, grads = run_train_step(ms, p, tok, lab, update=False)
    assert torch.all(grads["pos_emb"][ms.blk.S:] == 0)
    assert torch.any(grads["pos_emb"][:ms.blk.S] != 0)


# ---- the validation step and gradient accumulation over micro-batches -------------------------------
@pytest.mark.parametrize("ms", CASES, ids=lambda m: "%s_D%d_V%d" % (m.blk.dtype, m.blk.D, m.V))
def test_eval_step_gives_the_forward_loss_and_touches_nothing(ms):
    sh = ms.blk
    p, tok, lab = make_model_inputs(ms, seed=3, generic=True)
    logits, _ = orc.model_fwd(p, tok, sh.H, sh.dh, sh.gelu, sh.ln_eps)
    loss_ref, _ = orc.cross_entropy(logits.reshape(-1, ms.V), lab.reshape(-1))
    md = fax.FaxModelDims(dims_of(sh), sh.L, ms.V, ms.S_max, 0)
    params = _dev_params(p, sh.dtype)
    wsb = fax.fax_eval_workspace_bytes(md)
    assert wsb < fax.fax_train_workspace_bytes(md)
    ws = torch.empty(wsb, dtype=torch.uint8, device=DEV)
    loss = torch.zeros(4, device=DEV)
    fax.fax_eval_step(md, params, torch.from_numpy(tok).to(DEV), torch.from_numpy(lab).to(DEV), loss, ws, wsb)
    torch.cuda.synchronize()
    assert abs(loss[0].item() - loss_ref) <= (1e-5 if sh.dtype == "f32" else 2e-3) * abs(loss_ref)
    for name, get in _walk(params):
        assert np.array_equal(to_np(get(params)), get(p)), name
    # the training step reports the same number
    loss_t, *_ = run_train_step(ms, p, tok, lab, update=False)
    assert abs(loss[0].item() - loss_t) <= 1e-6 * abs(loss_t)
    with pytest.raises(fax.FaxError):
        fax.fax_eval_step(md, params, torch.from_numpy(tok).to(DEV), torch.from_numpy(lab).to(DEV), loss, ws, wsb - 1)


@pytest.mark.parametrize("ms", CASES[:2], ids=lambda m: "%s_D%d_V%d" % (m.blk.dtype, m.blk.D, m.V))
def test_two_micro_batches_accumulate_to_the_full_batch_step(ms):
    """Batch rows 0 and 1 as two calls (micro_batches = 2; the second adds to the gradients and applies
    the update) against the oracle's gradients and AdamW step for the batch of two."""
    sh = ms.blk
    assert sh.B == 2
    p, tok, lab = make_model_inputs(ms, seed=3, generic=True)
    loss_ref, g_ref, _ = orc.model_loss_and_grads(p, tok, lab, sh.H, sh.dh, sh.gelu, sh.ln_eps)
    half = ms.scaled(B=1)
    params = _dev_params(p, sh.dtype)
    master = params if sh.dtype == "f32" else _like(params, src=params)
    m = _like(params, 0.0); v = _like(params, 0.0); grads = _like(params, 7.0)
    hp = fax.FaxAdamW(**ADAMW_DEFAULT)
    loss = torch.zeros(4, device=DEV)
    losses = []
    for i, flags in enumerate((fax.FAX_FLAG_SKIP_UPDATE, fax.FAX_FLAG_ACCUMULATE | fax.FAX_FLAG_SKIP_UPDATE)):
        md = fax.FaxModelDims(dims_of(half.blk), sh.L, ms.V, ms.S_max, flags, 2)
        wsb = fax.fax_train_workspace_bytes(md)
        ws = torch.empty(wsb, dtype=torch.uint8, device=DEV)
        fax.fax_train_step(md, params, master, m, v, grads, torch.from_numpy(tok[i:i + 1].copy()).to(DEV),
                           torch.from_numpy(lab[i:i + 1].copy()).to(DEV), hp, 1, loss, ws, wsb)
        torch.cuda.synchronize()
        losses.append(loss[0].item())
    assert abs(0.5 * (losses[0] + losses[1]) - loss_ref) <= (1e-5 if sh.dtype == "f32" else 2e-3) * abs(loss_ref)
    t = tol(sh.dtype)
    bad = {}
    for name, get in _walk(grads):
        e = err(to_np(get(grads)), get(g_ref), sh.dtype)
        if not e <= t:
            bad[name] = e
    assert not bad, bad
    # the same two calls on a fresh state, the second one now also applying the update
    params = _dev_params(p, sh.dtype)
    master = params if sh.dtype == "f32" else _like(params, src=params)
    m = _like(params, 0.0); v = _like(params, 0.0); grads = _like(params, 7.0)
    for i, flags in enumerate((fax.FAX_FLAG_SKIP_UPDATE, fax.FAX_FLAG_ACCUMULATE)):
        md = fax.FaxModelDims(dims_of(half.blk), sh.L, ms.V, ms.S_max, flags, 2)
        fax.fax_train_step(md, params, master, m, v, grads, torch.from_numpy(tok[i:i + 1].copy()).to(DEV),
                           torch.from_numpy(lab[i:i + 1].copy()).to(DEV), hp, 1, loss, ws, wsb)
    torch.cuda.synchronize()
    bad = update_failures(ms, p, g_ref, master, m, v)
    assert not bad, bad
