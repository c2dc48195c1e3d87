"""End-to-end parity of fax_block_fwd / fax_block_bwd against the CPU oracle, through the C ABI.

Bar: fp32 workloads, max-norm relative error <= 1e-5 per tensor; bf16 workloads, Frobenius-norm
relative error <= 2e-2 per output and gradient tensor.  Both sides receive the same seeded inputs,
already rounded to the storage precision.
"""
import numpy as np
import pytest

from oracle import transformer as orc
from workloads import BlockShape, get_config, make_block_inputs, PARAM_NAMES
from helpers import run_block, err, tol, rel_max

pytestmark = pytest.mark.gpu


def _check_block(sh, out, p, x, dy, gelu, partial=False):
    y, c = orc.block_fwd(x, p, sh.H, sh.dh, gelu, sh.ln_eps)
    dx, g, it = orc.block_bwd(dy, c, p)
    t = tol(sh.dtype)
    report = {"y": err(out["y"], y, sh.dtype), "dx": err(out["dx"], dx, sh.dtype)}
    for k in PARAM_NAMES:
        report["d" + k] = err(out["grads"][k], g[k], sh.dtype)
    flat = lambda a: a.reshape(-1, a.shape[-1])
    for k in ("h1", "qkv", "ctx", "x1", "h2", "a"):
        report["saved." + k] = err(out["saved"][k], flat(c[k]), sh.dtype)
    report["saved.dgelu"] = err(out["saved"]["dgelu"], flat(orc.gelu_grad(c["u"], gelu)), sh.dtype)
    for k in ("du", "dh2", "dx1", "dctx", "dqkv", "dh1"):
        report["bwd." + k] = err(out["bwd"][k], flat(it[k]), sh.dtype)
    if partial:
        report["p_attn"] = err(out["p_attn"], c["p_attn"], sh.dtype)
        report["p_mlp"] = err(out["p_mlp"], c["p_mlp"], sh.dtype)
    bad = {k: v for k, v in report.items() if not v <= t}
    assert not bad, (bad, report)
    # the key-bias gradient is analytically zero: a free check on the attention backward
    Hd = sh.Hd
    gb = out["grads"]["bqkv"]
    assert np.abs(gb[Hd:2 * Hd]).max() <= (1e-5 if sh.dtype == "f32" else 2e-2) * np.abs(gb).max()
    return report


@pytest.mark.parametrize("gelu", ["tanh", "erf"])
@pytest.mark.parametrize("generic", [False, True])
def test_cfg1_fp32_block(gelu, generic):
    sh = get_config("cfg1")
    p, x, dy = make_block_inputs(sh, seed=0, generic=generic)
    out = run_block(sh, p, x, dy, gelu=gelu)
    _check_block(sh, out, p, x, dy, gelu)


@pytest.mark.parametrize("generic", [False, True])
def test_cfg1_fp32_block_then_adamw_step(generic):
    """The tiny configuration as it is defined: forward, backward, then one AdamW step (lr 1e-3,
    betas 0.9 / 0.999, eps 1e-8, wd 0.01) on the block's own gradients; updated parameters and both
    moments against the oracle's update of the oracle's gradients."""
    import torch
    import paper_2204_06514_amd as fax
    from workloads.configs import ADAMW_DEFAULT
    from helpers import dims_of, to_dev, to_np, DEV, adamw_step_report, bqkv_keep
    sh = get_config("cfg1")
    p, x, dy = make_block_inputs(sh, seed=0, generic=generic)
    dims = dims_of(sh)
    pd = {k: to_dev(p[k], "f32") for k in PARAM_NAMES}
    xd, dyd = to_dev(x, "f32"), to_dev(dy, "f32")
    saved = torch.empty(fax.fax_block_saved_layout(dims).total, dtype=torch.uint8, device=DEV)
    wsb = fax.fax_block_workspace_bytes(dims)
    ws = torch.empty(wsb, dtype=torch.uint8, device=DEV)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    gd = {k: torch.full(t.shape, 7.0, dtype=torch.float32, device=DEV) for k, t in pd.items()}
    fax.fax_block_fwd(dims, pd, xd, y, saved, None, None, ws, wsb)
    fax.fax_block_bwd(dims, pd, xd, dyd, saved, dx, gd, 0, None, None, ws, wsb)
    m = {k: torch.zeros_like(t) for k, t in pd.items()}
    v = {k: torch.zeros_like(t) for k, t in pd.items()}
    fax.fax_adamw_block_step(dims, *(fax.block_tensors(t) for t in (pd, m, v, gd)), None, fax.FaxAdamW(**ADAMW_DEFAULT), 1)
    torch.cuda.synchronize()
    _, c = orc.block_fwd(x, p, sh.H, sh.dh, "tanh", sh.ln_eps)
    _, g, _ = orc.block_bwd(dy, c, p)
    a = ADAMW_DEFAULT
    bad = {}
    for k in PARAM_NAMES:
        keep = bqkv_keep(sh.Hd) if k == "bqkv" else None
        r = adamw_step_report(to_np(pd[k]), to_np(m[k]), to_np(v[k]), p[k], g[k], a, keep=keep, dtype="f32")
        ref, _, _ = orc.adamw(p[k], 0.0, 0.0, g[k], a["lr"], a["beta1"], a["beta2"], a["eps"], a["wd"], 1)
        got = to_np(pd[k])
        if keep is not None:
            ref, got = ref[keep], got[keep]
        e = rel_max(got, ref)
        if e > 1e-5:
            r["updated_parameters"] = e
        if r:
            bad[k] = r
    assert not bad, bad


def test_fp32_ragged_shapes_and_partial_sums():
    sh = BlockShape(B=3, S=37, D=72, H=3, dh=20, F=100, dtype="f32", sigma_w=0.05)
    p, x, dy = make_block_inputs(sh, seed=4, generic=True)
    out = run_block(sh, p, x, dy, partial=True)
    _check_block(sh, out, p, x, dy, "tanh", partial=True)


def test_gradient_accumulation_flag():
    sh = get_config("cfg1")
    p, x, dy = make_block_inputs(sh, seed=1, generic=True)
    rng = np.random.default_rng(0)
    init = {k: rng.standard_normal(p[k].shape) for k in PARAM_NAMES}
    out = run_block(sh, p, x, dy, accumulate=True, grads_init=init)
    _, c = orc.block_fwd(x, p, sh.H, sh.dh)
    _, g, _ = orc.block_bwd(dy, c, p)
    for k in PARAM_NAMES:
        ref = init[k].astype(np.float32).astype(np.float64) + g[k]
        assert rel_max(out["grads"][k], ref) <= 1e-5, k


BF16_SMALL = [
    # several MFMA tiles in every GEMM
    BlockShape(B=2, S=256, D=256, H=4, dh=64, F=1024, dtype="bf16", sigma_w=0.02),
    # a tensor-parallel share: H*dh != D
    BlockShape(B=1, S=384, D=512, H=2, dh=128, F=256, dtype="bf16", sigma_w=0.02),
    # ragged everything: the scalar fallback kernels
    BlockShape(B=2, S=100, D=136, H=3, dh=24, F=200, dtype="bf16", sigma_w=0.05),
    # many tokens, narrow layers: the weight-gradient products split their contraction over several workgroups per tile
    BlockShape(B=2, S=1024, D=256, H=4, dh=64, F=512, dtype="bf16", sigma_w=0.02),
]


@pytest.mark.parametrize("sh", BF16_SMALL, ids=lambda s: "D%d_S%d_dh%d" % (s.D, s.S, s.dh))
@pytest.mark.parametrize("generic", [False, True])
def test_bf16_small_blocks(sh, generic):
    p, x, dy = make_block_inputs(sh, seed=2, generic=generic)
    out = run_block(sh, p, x, dy, partial=True)
    _check_block(sh, out, p, x, dy, "tanh", partial=True)


def test_bf16_split_contraction_accumulates():
    """Weight gradients whose contraction is split over workgroups, added onto existing values."""
    sh = BF16_SMALL[3]
    p, x, dy = make_block_inputs(sh, seed=5, generic=True)
    rng = np.random.default_rng(1)
    init = {k: rng.standard_normal(p[k].shape) * 0.5 for k in PARAM_NAMES}
    out = run_block(sh, p, x, dy, accumulate=True, grads_init=init)
    base = run_block(sh, p, x, dy)
    for k in PARAM_NAMES:
        ref = init[k].astype(np.float32).astype(np.float64) + base["grads"][k].astype(np.float64)
        assert rel_max(out["grads"][k], ref) <= 1e-6, k
