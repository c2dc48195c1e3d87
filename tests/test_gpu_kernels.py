"""Per-kernel parity on the GPU against the CPU oracle (or, for a bare GEMM, the float64 product
that the oracle's own matmul step is), through the C ABI."""
import math

import numpy as np
import pytest
import torch

import paper_2204_06514_amd as fax
from oracle import transformer as orc
from workloads import round_to_bf16
from helpers import DEV, TDTYPE, CODE, to_dev, to_np, err, tol, rel_max, rel_fro

pytestmark = pytest.mark.gpu


def _store(a, dtype):
    return round_to_bf16(a) if dtype == "bf16" else a.astype(np.float32).astype(np.float64)


# ------------------------------------------------------------------------------ GEMM
GEMM_CASES = [
    # dtype, path, ta, tb, M, N, K
    ("f32", fax.PATH_SCALAR, 0, 0, 128, 384, 128),
    ("f32", fax.PATH_SCALAR, 0, 1, 70, 33, 19),
    ("f32", fax.PATH_SCALAR, 1, 0, 65, 130, 257),
    ("f32", fax.PATH_SCALAR, 1, 1, 5, 7, 3),
    ("bf16", fax.PATH_SCALAR, 0, 0, 100, 72, 40),
    ("bf16", fax.PATH_SCALAR, 1, 0, 96, 40, 200),
    ("bf16", fax.PATH_MFMA, 0, 0, 256, 384, 192),     # 128-tiles, forward form
    ("bf16", fax.PATH_MFMA, 0, 1, 384, 128, 256),     # input-gradient form
    ("bf16", fax.PATH_MFMA, 1, 0, 128, 256, 320),     # weight-gradient form
    ("bf16", fax.PATH_MFMA, 1, 1, 128, 128, 64),
    ("bf16", fax.PATH_MFMA, 0, 0, 2048, 4096, 256),   # 256-tiles
    ("bf16", fax.PATH_MFMA, 0, 1, 4096, 2048, 128),
    ("bf16", fax.PATH_MFMA, 1, 0, 2048, 4096, 192),
    ("bf16", fax.PATH_MFMA, 1, 1, 4096, 2048, 64),
    # more 256-tiles than CUs and not a multiple of either 8 or the CU count: some workgroups of the
    # persistent kernel do two tiles, some one; K of one, two and three slabs
    ("bf16", fax.PATH_MFMA, 0, 0, 4352, 4352, 64),
    ("bf16", fax.PATH_MFMA, 0, 1, 4352, 4352, 128),
    ("bf16", fax.PATH_MFMA, 1, 0, 4352, 4352, 192),
    # one dimension an odd multiple of 128: 256-tiles for the bulk, 128-tiles for the last strip
    ("bf16", fax.PATH_MFMA, 0, 0, 4224, 2048, 128),
    ("bf16", fax.PATH_MFMA, 0, 1, 2048, 4224, 64),
    ("bf16", fax.PATH_MFMA, 1, 0, 4224, 2048, 192),
    ("bf16", fax.PATH_MFMA, 1, 1, 2048, 4224, 128),
    # too few 256^2 tiles for the chip, more than one round of 128^2 tiles: the 256 x 128 tile class
    ("bf16", fax.PATH_MFMA, 0, 0, 2048, 2560, 320),
    ("bf16", fax.PATH_MFMA, 0, 1, 2048, 2560, 192),
    ("bf16", fax.PATH_MFMA, 1, 0, 2048, 2560, 128),
    ("bf16", fax.PATH_MFMA, 1, 1, 2048, 2560, 256),
]


@pytest.mark.parametrize("dtype,path,ta,tb,M,N,K", GEMM_CASES)
def test_gemm_all_orientations(dtype, path, ta, tb, M, N, K):
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    A = _store(rng.standard_normal((K, M) if ta else (M, K)), dtype)
    B = _store(rng.standard_normal((N, K) if tb else (K, N)), dtype)
    bias = _store(rng.standard_normal(N), dtype)
    R = _store(rng.standard_normal((M, N)), dtype)
    ref = (A.T if ta else A) @ (B.T if tb else B)
    Ad, Bd, bd, Rd = (to_dev(a, dtype) for a in (A, B, bias, R))
    Cd = torch.empty((M, N), dtype=TDTYPE[dtype], device=DEV)
    fax.fax_gemm(CODE[dtype], ta, tb, M, N, K, Ad, A.shape[1], Bd, B.shape[1], Cd, N, bias=bd, residual=Rd, ldr=N,
                 path=path)
    assert err(to_np(Cd), ref + bias + R, dtype) <= (1e-5 if dtype == "f32" else 4e-3)
    # fp32 output, overwrite then accumulate
    Cf = torch.full((M, N), 3.0, dtype=torch.float32, device=DEV)
    fax.fax_gemm(CODE[dtype], ta, tb, M, N, K, Ad, A.shape[1], Bd, B.shape[1], Cf, N, c_f32=1, path=path)
    assert rel_max(to_np(Cf), ref) <= 1e-5
    fax.fax_gemm(CODE[dtype], ta, tb, M, N, K, Ad, A.shape[1], Bd, B.shape[1], Cf, N, c_f32=1, accumulate=1, path=path)
    assert rel_max(to_np(Cf), 2 * ref) <= 1e-5


def test_gemm_auto_path_falls_back_on_ragged_shapes():
    rng = np.random.default_rng(0)
    M, N, K = 130, 136, 72
    A = round_to_bf16(rng.standard_normal((M, K))); B = round_to_bf16(rng.standard_normal((K, N)))
    Cd = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    fax.fax_gemm(fax.FAX_BF16, 0, 0, M, N, K, to_dev(A, "bf16"), K, to_dev(B, "bf16"), N, Cd, N)
    assert rel_fro(to_np(Cd), A @ B) <= 4e-3
    with pytest.raises(fax.FaxError):
        fax.fax_gemm(fax.FAX_BF16, 0, 0, M, N, K, to_dev(A, "bf16"), K, to_dev(B, "bf16"), N, Cd, N, path=fax.PATH_MFMA)


# ------------------------------------------------------------------------- LayerNorm
@pytest.mark.parametrize("dtype,rows,D", [("f32", 128, 128), ("f32", 37, 100), ("f32", 9, 4096), ("bf16", 300, 1024),
                                          ("bf16", 129, 4096), ("bf16", 33, 12288), ("bf16", 21, 1000),
                                          ("bf16", 17, 20000),
                                          # every lanes-per-row x vectors-per-thread form of the one-pass backward,
                                          # and a workgroup that walks over many row blocks with a ragged last one
                                          ("bf16", 70, 2048), ("f32", 50, 768), ("bf16", 20, 8192), ("bf16", 5001, 768),
                                          ("bf16", 19, 5120), ("bf16", 23, 10240), ("bf16", 2048, 1024)])
def test_layernorm_forward_backward(dtype, rows, D):
    rng = np.random.default_rng(rows + D)
    x = _store(rng.standard_normal((rows, D)) * 2 + 0.5, dtype)
    g = _store(1 + 0.1 * rng.standard_normal(D), dtype); b = _store(0.1 * rng.standard_normal(D), dtype)
    dh = _store(rng.standard_normal((rows, D)), dtype); dres = _store(rng.standard_normal((rows, D)), dtype)
    h_ref, xhat, rstd = orc.layernorm_fwd(x, g, b, 1e-5)
    dx_ref, dg_ref, db_ref = orc.layernorm_bwd(dh, xhat, rstd, g)
    td = TDTYPE[dtype]
    xd, gd, bd, dhd, drd = (to_dev(a, dtype) for a in (x, g, b, dh, dres))
    h = torch.empty_like(xd); mu = torch.empty(rows, device=DEV); rs = torch.empty(rows, device=DEV)
    fax.fax_layernorm_fwd(CODE[dtype], rows, D, xd, gd, bd, 1e-5, h, mu, rs)
    assert err(to_np(h), h_ref, dtype) <= (1e-5 if dtype == "f32" else 4e-3)
    assert rel_max(to_np(mu), x.mean(-1)) <= 1e-5 and rel_max(to_np(rs), rstd[:, 0]) <= 1e-5
    wsb = fax.fax_layernorm_bwd_workspace_bytes(D)
    ws = torch.empty(wsb, dtype=torch.uint8, device=DEV)
    dx = torch.empty_like(xd); dg = torch.full((D,), 1.0, device=DEV); db = torch.full((D,), 1.0, device=DEV)
    fax.fax_layernorm_bwd(CODE[dtype], rows, D, dhd, xd, mu, rs, gd, drd, dx, dg, db, 0, ws, wsb)
    assert err(to_np(dx), dx_ref + dres, dtype) <= (1e-5 if dtype == "f32" else 4e-3)
    assert rel_max(to_np(dg), dg_ref) <= 2e-5 and rel_max(to_np(db), db_ref) <= 2e-5
    fax.fax_layernorm_bwd(CODE[dtype], rows, D, dhd, xd, mu, rs, gd, None, dx, dg, db, 1, ws, wsb)
    assert err(to_np(dx), dx_ref, dtype) <= (1e-5 if dtype == "f32" else 4e-3)
    assert rel_max(to_np(dg), 2 * dg_ref) <= 2e-5 and rel_max(to_np(db), 2 * db_ref) <= 2e-5


# ------------------------------------------------------------------------- attention
def _attention_case(dtype, B, S, H, dh, path, scale=1.0):
    rng = np.random.default_rng(S * 3 + dh)
    Hd = H * dh
    qkv = _store(rng.standard_normal((B, S, 3 * Hd)) * scale, dtype)
    dctx = _store(rng.standard_normal((B, S, Hd)), dtype)
    ctx_ref, lse_ref = orc.attention_fwd(qkv, H, dh)
    dqkv_ref = orc.attention_bwd(dctx, qkv, H, dh)
    td = TDTYPE[dtype]
    qd, dd = to_dev(qkv, dtype), to_dev(dctx, dtype)
    ctx = torch.empty((B, S, Hd), dtype=td, device=DEV); lse = torch.empty((B, H, S), device=DEV)
    fax.fax_attention_fwd(CODE[dtype], B, S, H, dh, qd, ctx, lse, path)
    e_ctx = err(to_np(ctx), ctx_ref, dtype); e_lse = np.abs(to_np(lse) - lse_ref).max()
    dq = torch.empty_like(qd); delta = torch.empty((B, H, S), device=DEV)
    fax.fax_attention_bwd(CODE[dtype], B, S, H, dh, qd, ctx, lse, dd, dq, delta, path)
    got = to_np(dq)
    errs = [err(got[..., i * Hd:(i + 1) * Hd], dqkv_ref[..., i * Hd:(i + 1) * Hd], dtype) for i in range(3)]
    return e_ctx, e_lse, errs


@pytest.mark.parametrize("dtype,B,S,H,dh", [("f32", 2, 64, 4, 32), ("f32", 1, 131, 2, 48), ("f32", 1, 1, 1, 8),
                                            ("bf16", 2, 200, 3, 64), ("bf16", 1, 70, 2, 128)])
def test_attention_scalar_path(dtype, B, S, H, dh):
    e_ctx, e_lse, errs = _attention_case(dtype, B, S, H, dh, fax.PATH_SCALAR)
    t = 1e-5 if dtype == "f32" else 6e-3
    assert e_ctx <= t and e_lse <= (2e-5 if dtype == "f32" else 1e-4) and max(errs) <= t, (e_ctx, e_lse, errs)


@pytest.mark.parametrize("B,S,H,dh,scale", [(2, 128, 2, 64, 1.0), (1, 384, 3, 128, 1.0), (2, 512, 2, 64, 2.0),
                                            (1, 1024, 2, 128, 0.5)])
def test_attention_mfma_path(B, S, H, dh, scale):
    """scale widens the score distribution (std = scale^2 sqrt(dh)): peaky softmax rows at 2.0."""
    e_ctx, e_lse, errs = _attention_case("bf16", B, S, H, dh, fax.PATH_MFMA, scale)
    assert e_ctx <= 8e-3 and e_lse <= 2e-4 and max(errs) <= 1e-2, (e_ctx, e_lse, errs)


@pytest.mark.parametrize("dh,slope", [(128, 0.02), (128, 0.2), (64, 0.05), (64, 1.0)])
def test_attention_forward_with_steadily_rising_scores(dh, slope):
    """Scores that grow with the key index, slowly or fast: the running maximum keeps moving, so the
    forward kernel's lazily updated reference point is exercised both ways (probabilities above 1
    between updates at the small slopes; an update in every tile at the large ones)."""
    B, S, H = 1, 1024, 2
    Hd = H * dh
    rng = np.random.default_rng(int(1000 * slope) + dh)
    u = rng.standard_normal(dh); u /= np.linalg.norm(u)
    qkv = 0.3 * rng.standard_normal((B, S, 3 * Hd))
    ramp = slope * np.arange(S)[:, None] * np.sqrt(dh)            # score of (i, j) gains slope * j
    for h in range(H):
        qkv[0, :, h * dh:(h + 1) * dh] += u                       # q_i . u = 1 (+ noise)
        qkv[0, :, Hd + h * dh:Hd + (h + 1) * dh] += ramp * u      # k_j . u = slope * j * sqrt(dh)
    qkv = _store(qkv, "bf16")
    ctx_ref, lse_ref = orc.attention_fwd(qkv, H, dh)
    qd = to_dev(qkv, "bf16")
    ctx = torch.empty((B, S, Hd), dtype=torch.bfloat16, device=DEV); lse = torch.empty((B, H, S), device=DEV)
    fax.fax_attention_fwd(fax.FAX_BF16, B, S, H, dh, qd, ctx, lse, fax.PATH_MFMA)
    assert err(to_np(ctx), ctx_ref, "bf16") <= 8e-3
    assert np.abs(to_np(lse) - lse_ref).max() <= 2e-4 * max(1.0, np.abs(lse_ref).max())


def test_attention_mfma_rejects_uncovered_shapes():
    q = torch.zeros((1, 100, 3 * 64), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(fax.FaxError) as e:
        fax.fax_attention_fwd(fax.FAX_BF16, 1, 100, 1, 64, q, torch.empty((1, 100, 64), dtype=torch.bfloat16, device=DEV),
                              torch.empty((1, 1, 100), device=DEV), fax.PATH_MFMA)
    assert e.value.status == fax.FAX_ERR_UNSUPPORTED


# --------------------------------------------------------------------- cross-entropy
@pytest.mark.parametrize("dtype,N,V", [("f32", 64, 1000), ("f32", 7, 37), ("bf16", 50, 51200), ("bf16", 33, 777),
                                       ("bf16", 3, 70000)])
def test_cross_entropy(dtype, N, V):
    rng = np.random.default_rng(N + V)
    z = _store(rng.standard_normal((N, V)) * 3, dtype)
    y = rng.integers(0, V, N).astype(np.int32)
    y[0] = 0; y[-1] = V - 1
    loss_ref, dz_ref = orc.cross_entropy(z, y.astype(np.int64))
    zd = to_dev(z, dtype); yd = torch.from_numpy(y).to(DEV)
    rl = torch.empty(N, device=DEV); loss = torch.empty(1, device=DEV)
    fax.fax_cross_entropy(CODE[dtype], N, V, zd, yd, zd, rl, loss)     # gradient written in place
    assert abs(loss.item() - loss_ref) <= 2e-6 * abs(loss_ref)
    assert err(to_np(zd), dz_ref, dtype) <= (1e-5 if dtype == "f32" else 4e-3)


@pytest.mark.parametrize("dtype,N,V", [("bf16", 4, 131072),    # the longest row the register-cached kernel takes (1024 threads x 16 vectors)
                                       ("bf16", 3, 131080),    # one vector more: the three-pass kernel
                                       ("f32", 5, 65536), ("f32", 2, 65540),
                                       ("bf16", 9, 50304), ("bf16", 6, 512), ("bf16", 6, 8)])
def test_cross_entropy_row_lengths_around_the_cache_limit_and_wide_logit_ranges(dtype, N, V):
    rng = np.random.default_rng(N * 7 + V)
    z = rng.standard_normal((N, V)) * 3
    z[0, : min(V, 16)] += 60.0       # a few dominant logits: everything else underflows next to them
    z[-1] -= 80.0                    # a row far below zero
    z[N // 2, V // 2] = 88.0
    z = _store(z, dtype)
    y = rng.integers(0, V, N).astype(np.int32)
    y[0] = 3; y[-1] = V - 1
    loss_ref, dz_ref = orc.cross_entropy(z, y.astype(np.int64))
    zd = to_dev(z, dtype); yd = torch.from_numpy(y).to(DEV)
    out = torch.empty_like(zd); rl = torch.empty(N, device=DEV); loss = torch.empty(1, device=DEV)
    fax.fax_cross_entropy(CODE[dtype], N, V, zd, yd, out, rl, loss)
    assert abs(loss.item() - loss_ref) <= 4e-6 * abs(loss_ref)
    assert err(to_np(out), dz_ref, dtype) <= (1e-5 if dtype == "f32" else 4e-3)
    assert np.abs(to_np(out).sum(axis=1)).max() <= (5e-6 if dtype == "f32" else 4e-3) / N   # rows of the gradient sum to zero


def test_cross_entropy_uniform_logits_give_log_vocab():
    N, V = 5, 51200
    zd = torch.full((N, V), 0.75, dtype=torch.bfloat16, device=DEV)
    yd = torch.arange(N, dtype=torch.int32, device=DEV)
    rl = torch.empty(N, device=DEV); loss = torch.empty(1, device=DEV)
    fax.fax_cross_entropy(fax.FAX_BF16, N, V, zd, yd, zd, rl, loss)
    assert abs(loss.item() - math.log(V)) < 1e-5


# ----------------------------------------------------------------------------- AdamW
@pytest.mark.parametrize("n", [1, 4099, 1 << 20])
def test_adamw_three_steps_and_bf16_copy(n):
    rng = np.random.default_rng(n)
    p = rng.standard_normal(n).astype(np.float32).astype(np.float64)
    m = np.zeros(n); v = np.zeros(n)
    pd = to_dev(p, "f32"); md = torch.zeros(n, device=DEV); vd = torch.zeros(n, device=DEV)
    low = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    hp = fax.FaxAdamW(1e-3, 0.9, 0.999, 1e-8, 0.01)
    for t in range(1, 4):
        g = (rng.standard_normal(n) * 10 ** rng.uniform(-3, 1, n)).astype(np.float32).astype(np.float64)
        p, m, v = orc.adamw(p, m, v, g, 1e-3, 0.9, 0.999, 1e-8, 0.01, t)
        fax.fax_adamw_step(pd, md, vd, to_dev(g, "f32"), fax.FAX_F32, low, n, hp, t)
        assert rel_max(to_np(pd), p) <= 1e-6
        assert rel_max(to_np(md), m) <= 1e-6 and rel_max(to_np(vd), v) <= 1e-6
        assert torch.equal(low, pd.to(torch.bfloat16))
    # closed form of the first step from zero moments
    g = rng.standard_normal(n).astype(np.float32).astype(np.float64)
    p0 = to_np(pd)
    md.zero_(); vd.zero_()
    fax.fax_adamw_step(pd, md, vd, to_dev(g, "f32"), fax.FAX_F32, None, n, hp, 1)
    assert rel_max(to_np(pd), p0 * (1 - 1e-5) - 1e-3 * g / (np.abs(g) + 1e-8)) <= 1e-6


@pytest.mark.parametrize("n", [3, 4099, 1 << 18])
def test_adamw_takes_gradients_in_bf16(n):
    """grad_dtype = FAX_BF16: the same update from gradients stored in the compute precision (both
    sides get the gradient already rounded to bf16; the arithmetic stays fp32)."""
    rng = np.random.default_rng(n + 7)
    p = rng.standard_normal(n).astype(np.float32).astype(np.float64)
    m = np.zeros(n); v = np.zeros(n)
    pd = to_dev(p, "f32"); md = torch.zeros(n, device=DEV); vd = torch.zeros(n, device=DEV)
    low = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    hp = fax.FaxAdamW(1e-3, 0.9, 0.999, 1e-8, 0.01)
    for t in range(1, 4):
        g = _store(rng.standard_normal(n) * 10 ** rng.uniform(-3, 1, n), "bf16")
        p, m, v = orc.adamw(p, m, v, g, 1e-3, 0.9, 0.999, 1e-8, 0.01, t)
        fax.fax_adamw_step(pd, md, vd, to_dev(g, "bf16"), fax.FAX_BF16, low, n, hp, t)
        assert rel_max(to_np(pd), p) <= 1e-6
        assert rel_max(to_np(md), m) <= 1e-6 and rel_max(to_np(vd), v) <= 1e-6
        assert torch.equal(low, pd.to(torch.bfloat16))


def test_adamw_block_step_updates_all_twelve_tensors_like_the_single_tensor_call():
    """Ragged tensor sizes (not multiples of 4, some below and some above one workgroup's chunk)."""
    B, S, D, H, dh, F = 1, 8, 73, 3, 7, 1501
    dims = fax.block_dims(B, S, D, H, dh, F, fax.FAX_BF16, fax.FAX_GELU_TANH, 1e-5, 0)
    shapes = {"ln1_g": D, "ln1_b": D, "wqkv": D * 3 * H * dh, "bqkv": 3 * H * dh, "wo": H * dh * D, "bo": D,
              "ln2_g": D, "ln2_b": D, "w1": D * F, "b1": F, "w2": F * D, "b2": D}
    assert list(shapes) == list(fax.TENSOR_NAMES)
    rng = np.random.default_rng(5)
    hp = fax.FaxAdamW(1e-3, 0.9, 0.999, 1e-8, 0.01)
    p = {k: rng.standard_normal(n).astype(np.float32) for k, n in shapes.items()}
    m = {k: (0.1 * rng.standard_normal(n)).astype(np.float32) for k, n in shapes.items()}
    v = {k: (0.01 * rng.random(n)).astype(np.float32) for k, n in shapes.items()}
    g = {k: rng.standard_normal(n).astype(np.float32) for k, n in shapes.items()}
    dev = lambda d: {k: torch.from_numpy(a.copy()).to(DEV) for k, a in d.items()}
    pd, md, vd, gd = dev(p), dev(m), dev(v), dev(g)
    low = {k: torch.zeros(n, dtype=torch.bfloat16, device=DEV) for k, n in shapes.items()}
    fax.fax_adamw_block_step(dims, *(fax.block_tensors(t) for t in (pd, md, vd, gd, low)), hp, 3)
    p1, m1, v1 = dev(p), dev(m), dev(v)
    for k, n in shapes.items():
        ref_p, ref_m, ref_v = orc.adamw(p[k].astype(np.float64), m[k].astype(np.float64), v[k].astype(np.float64),
                                        g[k].astype(np.float64), 1e-3, 0.9, 0.999, 1e-8, 0.01, 3)
        assert rel_max(to_np(pd[k]), ref_p) <= 1e-6 and rel_max(to_np(md[k]), ref_m) <= 1e-6, k
        assert rel_max(to_np(vd[k]), ref_v) <= 1e-6, k
        assert torch.equal(low[k], pd[k].to(torch.bfloat16)), k
        # and bit for bit what the one-tensor entry point computes
        fax.fax_adamw_step(p1[k], m1[k], v1[k], gd[k], fax.FAX_F32, None, n, hp, 3)
        assert torch.equal(p1[k], pd[k]) and torch.equal(m1[k], md[k]) and torch.equal(v1[k], vd[k]), k
    # without the low-precision copies
    fax.fax_adamw_block_step(dims, *(fax.block_tensors(t) for t in (pd, md, vd, gd)), None, hp, 4)
    fax.fax_adamw_step(p1["w1"], m1["w1"], v1["w1"], gd["w1"], fax.FAX_F32, None, shapes["w1"], hp, 4)
    assert torch.equal(p1["w1"], pd["w1"])


# ------------------------------------------------------------------------- measured ceilings
def test_probe_kernels_run_and_are_timed():
    n = 1 << 22
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=DEV)
    dst = torch.zeros(n, dtype=torch.uint8, device=DEV)
    sink = torch.zeros(4, device=DEV)
    fax.fax_timing_enable(1)
    try:
        fax.fax_probe_copy(src, dst, n)
        fax.fax_probe_mfma(64, 100, 0, sink)
        fax.fax_probe_mfma(64, 100, 1, sink)
        torch.cuda.synchronize()
        rows = {r["name"]: r for r in fax.fax_timing_report(16)}
    finally:
        fax.fax_timing_enable(0)
    assert torch.equal(src, dst)
    assert float(sink.abs().max()) == 0.0
    assert rows["probe_copy"]["work"] == 2.0 * n
    assert rows["probe_mfma_zero"]["work"] == rows["probe_mfma_random"]["work"] == 64 * 4 * 100 * 16 * 32768.0
    assert all(rows[k]["ms"] > 0 for k in ("probe_copy", "probe_mfma_zero", "probe_mfma_random"))
    with pytest.raises(fax.FaxError):
        fax.fax_probe_copy(src, dst, 24)
    with pytest.raises(fax.FaxError):
        fax.fax_probe_mfma(0, 100, 0, sink)


# ------------------------------------------------------------------------- per-kernel timing
def test_timing_report_names_kernels_and_counts_their_work():
    """bench.py's roofline entry rests on this: HIP events around each kernel family on the launch stream."""
    M, N, K = 512, 256, 128
    A = to_dev(round_to_bf16(np.ones((M, K))), "bf16"); B = to_dev(round_to_bf16(np.ones((K, N))), "bf16")
    Cd = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    fax.fax_timing_enable(1)
    try:
        for _ in range(3):
            fax.fax_gemm(fax.FAX_BF16, 0, 0, M, N, K, A, K, B, N, Cd, N)
        torch.cuda.synchronize()
        rows = fax.fax_timing_report(64)
    finally:
        fax.fax_timing_enable(0)
    gemm = [r for r in rows if r["name"].startswith("gemm_mfma_Ak_Bm")]
    assert len(gemm) == 1, rows
    assert gemm[0]["launches"] == 3 and gemm[0]["ms"] > 0.0
    assert gemm[0]["work"] == pytest.approx(3 * 2.0 * M * N * K)
    # switched off: nothing is recorded
    fax.fax_gemm(fax.FAX_BF16, 0, 0, M, N, K, A, K, B, N, Cd, N)
    torch.cuda.synchronize()
    fax.fax_timing_enable(1)
    try:
        assert fax.fax_timing_report(64) == []
    finally:
        fax.fax_timing_enable(0)
