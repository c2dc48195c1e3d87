"""Shared plumbing for the GPU parity tests: numpy <-> device tensors, error norms, and
drivers that run the C-ABI entry points on inputs from `workloads`."""
import numpy as np
import torch

import paper_2204_06514_amd as fax
from workloads import PARAM_NAMES

DEV = "cuda:0"
TDTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}
CODE = {"f32": fax.FAX_F32, "bf16": fax.FAX_BF16}
GELU = {"tanh": fax.FAX_GELU_TANH, "erf": fax.FAX_GELU_ERF}

# Tolerances of the parity bar: fp32 workloads, max-norm relative error per tensor;
# bf16 workloads, Frobenius-norm relative error per tensor.
TOL_F32 = 1e-5
TOL_BF16 = 2e-2


def to_dev(a, dtype):
    """float64 numpy (already representable in `dtype`) -> device tensor."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(TDTYPE[dtype]).contiguous()


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_max(got, ref):
    d = np.abs(ref).max()
    return np.abs(got - ref).max() / (d if d > 0 else 1.0)


def rel_fro(got, ref):
    d = np.linalg.norm(ref)
    return np.linalg.norm(got - ref) / (d if d > 0 else 1.0)


def err(got, ref, dtype):
    return rel_max(got, ref) if dtype == "f32" else rel_fro(got, ref)


def tol(dtype):
    return TOL_F32 if dtype == "f32" else TOL_BF16


def view_bytes(buf, offset, shape, tdtype):
    """Typed view into a uint8 device buffer."""
    n = int(np.prod(shape))
    return buf[offset:offset + n * torch.empty((), dtype=tdtype).element_size()].view(tdtype).view(*shape)


def dims_of(sh, flags=0, gelu=None):
    return fax.block_dims(sh.B, sh.S, sh.D, sh.H, sh.dh, sh.F, CODE[sh.dtype], GELU[gelu or sh.gelu], sh.ln_eps, flags)


def zeros_like_params(pd, dtype=torch.float32):
    return {k: torch.zeros(v.shape, dtype=dtype, device=DEV) for k, v in pd.items()}


def run_block(sh, p, x, dy, gelu=None, partial=False, accumulate=False, grads_init=None):
    """fax_block_fwd + fax_block_bwd through the C ABI.  Returns everything as float64 numpy."""
    dims = dims_of(sh, fax.FAX_FLAG_TP_PARTIAL if partial else 0, gelu)
    pd = {k: to_dev(p[k], sh.dtype) for k in PARAM_NAMES}
    xd, dyd = to_dev(x, sh.dtype), to_dev(dy, sh.dtype)
    td = TDTYPE[sh.dtype]
    lay = fax.fax_block_saved_layout(dims)
    saved = torch.empty(lay.total, dtype=torch.uint8, device=DEV)
    wsb = fax.fax_block_workspace_bytes(dims)
    ws = torch.empty(wsb, dtype=torch.uint8, device=DEV)
    y = torch.empty_like(xd)
    pa = torch.empty_like(xd) if partial else None
    pm = torch.empty_like(xd) if partial else None
    fax.fax_block_fwd(dims, pd, xd, y, saved, pa, pm, ws, wsb)
    gd = zeros_like_params(pd)
    if grads_init is not None:
        for k in gd:
            gd[k].copy_(torch.from_numpy(grads_init[k].astype(np.float32)))
    dx = torch.empty_like(xd)
    # a tensor-parallel rank asks for the two input-gradient partial sums in buffers of its own;
    # otherwise they stay in the workspace, at the offsets of fax_block_bwd_layout()
    d1 = torch.empty_like(xd) if partial else None
    d2 = torch.empty_like(xd) if partial else None
    fax.fax_block_bwd(dims, pd, xd, dyd, saved, dx, gd, accumulate, d1, d2, ws, wsb)
    torch.cuda.synchronize()
    T, Hd = sh.T, sh.Hd
    out = {"y": to_np(y).reshape(x.shape), "dx": to_np(dx).reshape(x.shape),
           "grads": {k: to_np(v) for k, v in gd.items()}}
    sv = {"h1": (lay.h1, (T, sh.D), td), "qkv": (lay.qkv, (T, 3 * Hd), td), "ctx": (lay.ctx, (T, Hd), td),
          "lse": (lay.lse, (sh.B, sh.H, sh.S), torch.float32), "x1": (lay.x1, (T, sh.D), td),
          "h2": (lay.h2, (T, sh.D), td), "dgelu": (lay.dgelu, (T, sh.F), td), "a": (lay.a, (T, sh.F), td)}
    out["saved"] = {k: to_np(view_bytes(saved, o, s, t)) for k, (o, s, t) in sv.items()}
    bl = fax.fax_block_bwd_layout(dims)
    bw = {"du": (bl.du, (T, sh.F)), "dh2": (bl.dh2, (T, sh.D)), "dx1": (bl.dx1, (T, sh.D)),
          "dctx": (bl.dctx, (T, Hd)), "dqkv": (bl.dqkv, (T, 3 * Hd)), "dh1": (bl.dh1, (T, sh.D))}
    if partial:   # delivered to the caller's buffers; their workspace slots are not written
        del bw["dh1"], bw["dh2"]
    out["bwd"] = {k: to_np(view_bytes(ws, o, s, td)) for k, (o, s) in bw.items()}
    if partial:
        out["bwd"]["dh1"] = to_np(d1).reshape(T, sh.D)
        out["bwd"]["dh2"] = to_np(d2).reshape(T, sh.D)
        out["p_attn"] = to_np(pa).reshape(x.shape)
        out["p_mlp"] = to_np(pm).reshape(x.shape)
    return out


# ---- the first AdamW step, end to end ------------------------------------------------------------------
# At step 1 from zero moments the update is lr g / (|g| + eps): every element moves by about lr in
# the direction of -g, whatever |g| is.  Comparing updated parameters at a bar of a few lr would
# therefore pass an update that does nothing (error lr) or goes the wrong way (2 lr).  What is
# compared instead: the moments (linear and quadratic in g, so the gradient bar carries over), the
# displacement master - p0 element by element against the oracle's (an element either agrees to
# rounding or, where the gradient is within the kernels' noise of zero, has the other sign: a
# small fraction), and that the displacement is there at all.
def adamw_step_report(got_master, got_m, got_v, p0, g_ref, hp, keep=None, dtype="bf16", step=1):
    """Failures (name -> value) of one tensor's first update.  All arguments float64 numpy;
    `keep`: optional boolean mask of the elements that count (the key third of bqkv does not:
    its gradient is analytically zero, so its first step is rounding noise times 1/eps)."""
    from oracle import transformer as orc
    ref_p, ref_m, ref_v = orc.adamw(p0, 0.0, 0.0, g_ref, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["wd"], step)
    sel = (lambda a: a[keep]) if keep is not None else (lambda a: a.reshape(-1))
    gm, gv, gp, p0s = sel(got_m), sel(got_v), sel(got_master), sel(p0)
    rm, rv, rp = sel(ref_m), sel(ref_v), sel(ref_p)
    bad = {}
    if dtype == "f32":
        if rel_max(gm, rm) > 1e-5: bad["m"] = rel_max(gm, rm)
        if rel_max(gv, rv) > 2e-5: bad["v"] = rel_max(gv, rv)
        if np.abs(gp - rp).max() > 2.5e-3 * hp["lr"]: bad["p"] = np.abs(gp - rp).max()
    else:
        if rel_fro(gm, rm) > 2e-2: bad["m"] = rel_fro(gm, rm)
        if rel_fro(gv, rv) > 4e-2: bad["v"] = rel_fro(gv, rv)
        # An element whose gradient lies within the kernels' error of zero may come out with the
        # other sign (a displacement of 2 lr).  The gradient bar bounds that error by 2e-2 of the
        # tensor's rms, so: no element with |g| above five times that may differ, and of the rest
        # at most 1 % of the tensor (two elements of a tensor smaller than 200).
        off = np.abs((gp - p0s) - (rp - p0s)) > 0.1 * hp["lr"]
        gr = sel(np.broadcast_to(g_ref, p0.shape))
        rms = np.sqrt(np.mean(gr * gr)) if gr.size else 0.0
        clear = np.abs(gr) > 0.1 * rms
        if (off & clear).any(): bad["displaced_elsewhere_clear_gradient"] = int((off & clear).sum())
        if off.sum() > max(0.01 * off.size, 2): bad["displaced_elsewhere"] = off.mean()
    moved = np.abs(gp - p0s).max() if gp.size else 0.0
    want = np.abs(rp - p0s).max() if rp.size else 0.0
    if want > 0 and moved < 0.5 * want: bad["not_moved"] = moved
    return bad


def bqkv_keep(Hd):
    """Mask of bqkv's query and value thirds."""
    k = np.ones(3 * Hd, dtype=bool)
    k[Hd:2 * Hd] = False
    return k
