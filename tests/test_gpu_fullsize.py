"""Parity at the benchmark configurations' full sizes, in the launch configurations bench.py times.

Every case is compared with the oracle element by element (per tensor, at the bars of helpers.py).
cfg2, cfg3, cfg4 and the three capacity-table shares run whole.  The two full models are covered
by two cuts each, because the float64 oracle's softmax over batch x sequence x vocabulary logits
is what limits them, not the device: all layers at one batch row (depth: the error that builds
up over twelve layers), and one layer at the full batch (every GEMM, attention and reduction
launch exactly as the full model launches it: the plans depend on the token count, not on the
layer count, which `fax_gemm_plan` confirms in the test).  The full models at full depth and full
batch are then checked through properties that hold at any size.
"""
import math

import numpy as np
import pytest
import torch

import paper_2204_06514_amd as fax
from oracle import transformer as orc
from workloads import get_config, make_block_inputs, make_stack_inputs, make_model_inputs, PARAM_NAMES
from workloads.configs import ADAMW_DEFAULT
from helpers import DEV, TDTYPE, to_dev, to_np, rel_fro, dims_of, run_block, TOL_BF16, adamw_step_report, bqkv_keep
from test_gpu_train import run_train_step, _walk, update_failures

pytestmark = pytest.mark.gpu


def _assert_all(report):
    bad = {k: v for k, v in report.items() if not v <= TOL_BF16}
    assert not bad, (bad, report)


def test_cfg2_two_layer_stack_with_adamw_full_size():
    sh = get_config("cfg2")
    ps, x, dy = make_stack_inputs(sh, seed=0)
    dims = dims_of(sh)
    pd = [{k: to_dev(p[k], "bf16") for k in PARAM_NAMES} for p in ps]
    xs = [to_dev(x, "bf16")] + [torch.empty((sh.B, sh.S, sh.D), dtype=torch.bfloat16, device=DEV) for _ in range(sh.L)]
    dyd = to_dev(dy, "bf16"); dcur = torch.empty_like(dyd)
    lay = fax.fax_block_saved_layout(dims)
    saved = [torch.empty(lay.total, dtype=torch.uint8, device=DEV) for _ in range(sh.L)]
    wsb = fax.fax_block_workspace_bytes(dims); ws = torch.empty(wsb, dtype=torch.uint8, device=DEV)
    gd = [{k: torch.empty(t.shape, dtype=torch.float32, device=DEV) for k, t in p.items()} for p in pd]
    for l in range(sh.L):
        fax.fax_block_fwd(dims, pd[l], xs[l], xs[l + 1], saved[l], None, None, ws, wsb)
    for l in reversed(range(sh.L)):
        fax.fax_block_bwd(dims, pd[l], xs[l], dyd if l == sh.L - 1 else dcur, saved[l], dcur, gd[l], 0, None, None, ws, wsb)
    master = [{k: t.float().clone() for k, t in p.items()} for p in pd]
    hp = fax.FaxAdamW(**ADAMW_DEFAULT)
    ms_, vs_ = [], []
    for l in range(sh.L):   # one launch per block
        m = {k: torch.zeros_like(t) for k, t in master[l].items()}
        v = {k: torch.zeros_like(t) for k, t in master[l].items()}
        fax.fax_adamw_block_step(dims, *(fax.block_tensors(t) for t in (master[l], m, v, gd[l], pd[l])), hp, 1)
        ms_.append(m); vs_.append(v)
    torch.cuda.synchronize()
    y, caches = orc.stack_fwd(x, ps, sh.H, sh.dh)
    dx, g = orc.stack_bwd(dy, caches, ps)
    rep = {"y": rel_fro(to_np(xs[-1]), y), "dx": rel_fro(to_np(dcur), dx)}
    bad = {}
    for l in range(sh.L):
        for k in PARAM_NAMES:
            rep["L%d.d%s" % (l, k)] = rel_fro(to_np(gd[l][k]), g[l][k])
            r = adamw_step_report(to_np(master[l][k]), to_np(ms_[l][k]), to_np(vs_[l][k]), ps[l][k], g[l][k], ADAMW_DEFAULT,
                                  keep=bqkv_keep(sh.Hd) if k == "bqkv" else None)
            if r:
                bad["L%d.%s" % (l, k)] = r
            assert torch.equal(pd[l][k], master[l][k].to(torch.bfloat16)), (l, k)
    _assert_all(rep)
    assert not bad, bad


def test_cfg3_large_block_full_size():
    sh = get_config("cfg3")
    p, x, dy = make_block_inputs(sh, seed=0)
    out = run_block(sh, p, x, dy)
    y, c = orc.block_fwd(x, p, sh.H, sh.dh)
    dx, g, it = orc.block_bwd(dy, c, p)
    flat = lambda a: a.reshape(-1, a.shape[-1])
    rep = {"y": rel_fro(out["y"], y), "dx": rel_fro(out["dx"], dx)}
    for k in PARAM_NAMES:
        rep["d" + k] = rel_fro(out["grads"][k], g[k])
    for k in ("qkv", "ctx", "x1", "a"):
        rep["saved." + k] = rel_fro(out["saved"][k], flat(c[k]))
    rep["saved.dgelu"] = rel_fro(out["saved"]["dgelu"], flat(orc.gelu_grad(c["u"])))
    for k in ("du", "dh2", "dx1", "dctx", "dqkv", "dh1"):
        rep["bwd." + k] = rel_fro(out["bwd"][k], flat(it[k]))
    _assert_all(rep)
    assert np.abs(out["saved"]["lse"] - c["lse"]).max() <= 2e-3


def test_cfg4_tensor_parallel_share():
    """One rank's share of the 12288-wide block at its full batch of 8: local shapes 12 heads x 128,
    QKV 12288x4608, out-proj 1536x12288, FFN 12288x6144 / 6144x12288.  Outputs, the un-reduced
    partial sums of both passes, and every weight and bias gradient (contractions over all 16384
    tokens) against the oracle run on the same full batch."""
    sh = get_config("cfg4")
    p, x, dy = make_block_inputs(sh, seed=0)
    rep, _, _ = _share_report(sh, p, x, dy)
    _assert_all(rep)


def _block_gemm_shapes(sh):
    T, D, Hd, F = sh.T, sh.D, sh.Hd, sh.F
    fwd = [(T, 3 * Hd, D, 0), (T, D, Hd, 0), (T, F, D, 0), (T, D, F, 0)]
    dgrad = [(T, F, D, 0), (T, D, F, 0), (T, Hd, D, 0), (T, D, 3 * Hd, 0)]
    wgrad = [(F, D, T, 1), (D, F, T, 1), (Hd, D, T, 1), (D, 3 * Hd, T, 1)]
    return fwd + dgrad + wgrad


def _model_gemm_shapes(ms):
    sh = ms.blk
    return _block_gemm_shapes(sh) + [(sh.T, ms.V, sh.D, 0), (ms.V, sh.D, sh.T, 1), (sh.T, sh.D, ms.V, 0)]


def _model_parity(ms, seed=0):
    sh = ms.blk
    p, tok, lab = make_model_inputs(ms, seed=seed)
    loss_ref, g_ref, _ = orc.model_loss_and_grads(p, tok, lab, sh.H, sh.dh)
    loss, params, master, m, v, grads = run_train_step(ms, p, tok, lab, update=False)
    assert abs(loss - loss_ref) <= 2e-3 * abs(loss_ref), (loss, loss_ref)
    rep = {name: rel_fro(to_np(get(grads)), get(g_ref)) for name, get in _walk(grads)}
    return rep, p, g_ref


def test_cfg5_all_twelve_layers_one_batch_row():
    """Depth: the 148 gradient tensors of the 12-layer model and its loss, full vocabulary, width and
    sequence, one batch row.  The errors per layer are printed (-s) so that their growth towards
    the input can be read off."""
    ms = get_config("cfg5").scaled(B=1)
    rep, _, _ = _model_parity(ms)
    for l in range(ms.L):
        row = {k.split(".")[1]: v for k, v in rep.items() if k.startswith("blocks[%d]." % l)}
        print("cfg5 layer %2d: worst %.4f (%s)  wqkv %.4f  w2 %.4f" % (l, max(row.values()), max(row, key=row.get),
                                                                      row["wqkv"], row["w2"]))
    _assert_all(rep)


def test_cfg5_one_layer_full_batch_launch_plans_and_update():
    """Breadth: one layer at the full batch of 8 x 2048 tokens.  Every product has the shape, and so
    the tile class, K split and strip decomposition, it has in the 12-layer step; gradients and the
    first AdamW step of every tensor against the oracle."""
    full = get_config("cfg5")
    ms = full.scaled(L=1)
    assert [fax.fax_gemm_plan(*g) for g in _model_gemm_shapes(ms)] == [fax.fax_gemm_plan(*g) for g in _model_gemm_shapes(full)]
    sh = ms.blk
    p, tok, lab = make_model_inputs(ms, seed=0)
    loss_ref, g_ref, _ = orc.model_loss_and_grads(p, tok, lab, sh.H, sh.dh)
    loss, params, master, m, v, grads = run_train_step(ms, p, tok, lab, update=True)
    assert abs(loss - loss_ref) <= 2e-3 * abs(loss_ref), (loss, loss_ref)
    _assert_all({name: rel_fro(to_np(get(grads)), get(g_ref)) for name, get in _walk(grads)})
    bad = update_failures(ms, p, g_ref, master, m, v)
    assert not bad, bad


def test_cfg5_full_size_step_properties():
    """The whole train step at full size: 12 layers, batch 8, vocabulary 51200.  Checked through what
    must hold at any size: the initial loss is ln V plus a small excess, every gradient is finite
    and non-trivial, the first AdamW step moves no parameter by more than lr (1 + wd |p|), and the
    bf16 compute copy is the rounded master."""
    ms = get_config("cfg5")
    sh = ms.blk
    p, tok, lab = make_model_inputs(ms, seed=0)
    loss, params, master, m, v, grads = run_train_step(ms, p, tok, lab, update=True)
    assert math.log(ms.V) - 0.05 <= loss <= math.log(ms.V) + 0.5, loss
    hp = ADAMW_DEFAULT
    for name, get in _walk(grads):
        gt = get(grads)
        assert torch.isfinite(gt).all(), name
        ref = torch.from_numpy(np.ascontiguousarray(get(p), dtype=np.float32)).to(DEV)
        step = (get(master) - ref).abs()
        bound = hp["lr"] * (1.0 + hp["wd"] * ref.abs()) * 1.001 + 1e-7
        assert bool((step <= bound).all()), name
        assert torch.equal(get(params), get(master).to(torch.bfloat16)), name
        if not name.endswith(("bqkv",)) and "pos_emb" not in name:
            assert float(gt.abs().max()) > 0, name
    # positions beyond the sequence do not exist here (S == S_max); token rows never looked up and never
    # predicted still receive the softmax mass of the output projection, so no row of dE is exactly zero
    Hd = sh.Hd
    gb = grads["blocks"][0]["bqkv"]
    assert float(gb[Hd:2 * Hd].abs().max()) <= 2e-2 * float(gb.abs().max())


# ---- capacity-table shares (Table 1 operating point: batch 1, sequence 2048, maximal tensor parallelism) ----
def _share_report(sh, p, x, dy):
    out = run_block(sh, p, x, dy, partial=True)
    y, c = orc.block_fwd(x, p, sh.H, sh.dh)
    dx, g, it = orc.block_bwd(dy, c, p)
    flat = lambda a: a.reshape(-1, a.shape[-1])
    rep = {"y": rel_fro(out["y"], y), "dx": rel_fro(out["dx"], dx), "p_attn": rel_fro(out["p_attn"], c["p_attn"]),
           "p_mlp": rel_fro(out["p_mlp"], c["p_mlp"]), "dh1_partial": rel_fro(out["bwd"]["dh1"], flat(it["dh1"])),
           "dh2_partial": rel_fro(out["bwd"]["dh2"], flat(it["dh2"]))}
    for k in PARAM_NAMES:
        rep["d" + k] = rel_fro(out["grads"][k], g[k])
    return rep, out, y


@pytest.mark.parametrize("name", ["t1_5120", "t1_10240"])
def test_capacity_table_share_full_size(name):
    """2048 tokens against weights of width 5120 / 10240: few, odd-shaped tiles per GEMM (N = 1920,
    K = 640, ...), 5 or 10 heads.  Element by element, every output and gradient."""
    sh = get_config(name)
    p, x, dy = make_block_inputs(sh, seed=0)
    rep, _, _ = _share_report(sh, p, x, dy)
    _assert_all(rep)


def test_capacity_table_share_16384():
    """Width 16384 at the full 2048 positions, element by element like the narrower two."""
    sh = get_config("t1_16384")
    p, x, dy = make_block_inputs(sh, seed=0)
    rep, _, _ = _share_report(sh, p, x, dy)
    _assert_all(rep)


# ---- the model of the per-phase timing figure (Fig. 4): 124M parameters, batch 32, sequence 2048 ----
def test_fig4_model_reduced_depth_and_batch_full_vocabulary():
    """Width 768, 12 heads of 64, vocabulary 50304, sequence 2048, at 2 layers and one batch row:
    loss and every gradient against the oracle."""
    ms = get_config("fig4_124m").scaled(B=1, L=2)
    rep, _, _ = _model_parity(ms)
    _assert_all(rep)


def test_fig4_block_at_the_full_batch_of_65536_tokens():
    """One block of that model at batch 32 x 2048: the four weight-gradient products contract over
    65536 tokens and run as 7 to 25 K ranges plus a fold; all of it element by element."""
    full = get_config("fig4_124m")
    sh = full.blk.scaled(L=1)
    assert [fax.fax_gemm_plan(*g) for g in _block_gemm_shapes(sh)] == [fax.fax_gemm_plan(*g) for g in _block_gemm_shapes(full.blk)]
    assert max(fax.fax_gemm_plan(*g)[3] for g in _block_gemm_shapes(sh)) >= 7
    p, x, dy = make_block_inputs(sh, seed=0)
    rep, _, _ = _share_report(sh, p, x, dy)
    _assert_all(rep)


def test_fig4_one_layer_full_batch_launch_plans():
    """One layer of that model at the full batch of 32 x 2048 tokens: the output projection over the
    50304-entry vocabulary (bulk on 256-wide tiles plus a 128-wide strip; its weight-gradient
    product over 65536 tokens in K ranges) and the loss over 65536 x 50304 logits as the full
    model launches them; loss and every gradient against the oracle."""
    full = get_config("fig4_124m")
    ms = full.scaled(L=1)
    assert [fax.fax_gemm_plan(*g) for g in _model_gemm_shapes(ms)] == [fax.fax_gemm_plan(*g) for g in _model_gemm_shapes(full)]
    rep, _, _ = _model_parity(ms)
    _assert_all(rep)


def test_fig4_model_full_size_step_properties_and_phase_times():
    """All 12 layers at batch 32: what must hold at any size (see the cfg5 test), and the timing
    records of the three phases the paper's figure splits the step into."""
    ms = get_config("fig4_124m")
    sh = ms.blk
    p, tok, lab = make_model_inputs(ms, seed=0)
    fax.fax_timing_enable(1)
    try:
        loss, params, master, m, v, grads = run_train_step(ms, p, tok, lab, update=True)
        rows = {r["name"]: r for r in fax.fax_timing_report(64)}
    finally:
        fax.fax_timing_enable(0)
    assert math.log(ms.V) - 0.05 <= loss <= math.log(ms.V) + 0.5, loss
    hp = ADAMW_DEFAULT
    for name, get in _walk(grads):
        gt = get(grads)
        assert torch.isfinite(gt).all(), name
        ref = torch.from_numpy(np.ascontiguousarray(get(p), dtype=np.float32)).to(DEV)
        step = (get(master) - ref).abs()
        bound = hp["lr"] * (1.0 + hp["wd"] * ref.abs()) * 1.001 + 1e-7
        assert bool((step <= bound).all()), name
        assert torch.equal(get(params), get(master).to(torch.bfloat16)), name
        if not name.endswith(("bqkv",)) and "pos_emb" not in name:
            assert float(gt.abs().max()) > 0, name
    for ph in ("phase_forward", "phase_loss", "phase_backward", "phase_update"):
        assert rows[ph]["launches"] == 1 and rows[ph]["ms"] > 0, ph
    # backward does twice the matrix work of forward; it cannot be faster, nor (here) four times slower
    assert 1.0 <= rows["phase_backward"]["ms"] / rows["phase_forward"]["ms"] <= 4.0
