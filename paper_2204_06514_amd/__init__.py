"""Python binding of libfax: the per-device Transformer training step on MI355X.

Argument marshalling only.  Every function has the name and argument order of
its C entry point (include/fax.h); tensors are torch tensors on the GPU whose
data pointers are passed through, structs are ctypes mirrors of the C ones.
PyTorch supplies device memory and the current stream; all arithmetic runs in
the library's HIP kernels.  Importing this package fails if libfax.so has not
been built: there is no fallback path.
"""
import ctypes as C
import os

import torch  # loads the HIP runtime that libfax.so links against

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfax.so")

FAX_OK, FAX_ERR_INVALID_ARG, FAX_ERR_UNSUPPORTED, FAX_ERR_WORKSPACE, FAX_ERR_HIP = 0, -1, -2, -3, -4
FAX_F32, FAX_BF16 = 0, 1
FAX_GELU_TANH, FAX_GELU_ERF = 0, 1
FAX_FLAG_TP_PARTIAL = 1
FAX_FLAG_SINGLE_STREAM = 2
FAX_FLAG_SKIP_UPDATE = 1
FAX_FLAG_ACCUMULATE = 2
FAX_FLAG_DETERMINISTIC = 4
PATH_AUTO, PATH_SCALAR, PATH_MFMA = 0, 1, 2

TENSOR_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


class FaxError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("libfax status %d: %s" % (status, text))
        self.status = status


class FaxBlockDims(C.Structure):
    _fields_ = [("B", C.c_int32), ("S", C.c_int32), ("D", C.c_int32), ("H", C.c_int32), ("dh", C.c_int32),
                ("F", C.c_int32), ("dtype", C.c_int32), ("gelu", C.c_int32), ("ln_eps", C.c_float),
                ("flags", C.c_uint32)]


class FaxBlockTensors(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in TENSOR_NAMES]


class FaxSavedLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("h1", "qkv", "ctx", "lse", "x1", "h2", "dgelu", "a",
                                          "mu1", "rstd1", "mu2", "rstd2", "total")]


class FaxBwdLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("du", "dh2", "dx1", "dctx", "dqkv", "dh1", "total")]


class FaxAdamW(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("lr", "beta1", "beta2", "eps", "wd")]


class FaxModelDims(C.Structure):
    _fields_ = [("blk", FaxBlockDims), ("L", C.c_int32), ("V", C.c_int32), ("S_max", C.c_int32),
                ("flags", C.c_uint32), ("micro_batches", C.c_int32)]


class FaxModelTensors(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("pos_emb", C.c_void_p), ("lnf_g", C.c_void_p), ("lnf_b", C.c_void_p),
                ("blocks", C.POINTER(FaxBlockTensors))]


class FaxGemmPlan(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("tail", "tile_m", "tile_n", "splits")]


class FaxMesh(C.Structure):
    _fields_ = [("data", C.c_int32), ("tensor", C.c_int32)]


class FaxAnalysis(C.Structure):
    _fields_ = [("local", FaxModelDims)] + [(n, C.c_double) for n in (
        "params_global", "params_local", "bytes_master", "bytes_moments", "bytes_grads", "bytes_lowp", "bytes_saved",
        "bytes_workspace", "bytes_total", "flop_step", "flop_step_unhalved", "hbm_bytes_step")] + [
        ("launches", C.c_int32)] + [(n, C.c_double) for n in (
            "ms_gemm", "ms_attention", "ms_bandwidth", "ms_step", "bytes_tensor_axis", "bytes_data_axis")]


class FaxKernelTime(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("launches", C.c_int32), ("unit", C.c_int32), ("ms", C.c_double),
                ("work", C.c_double)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libfax.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or paper_2204_06514_amd/build.py) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, sz, i32, f32 = C.c_void_p, C.c_size_t, C.c_int, C.c_float
    P = C.POINTER
    sig = {
        "fax_version": (C.c_char_p, []),
        "fax_last_error": (C.c_char_p, []),
        "fax_block_dims_check": (i32, [P(FaxBlockDims)]),
        "fax_gemm_plan": (i32, [i32, i32, i32, i32, P(FaxGemmPlan)]),
        "fax_gemm_tile_walk": (i32, [i32, i32, i32, i32, vp, vp, i32, P(C.c_int), P(C.c_int)]),
        "fax_block_saved_layout": (i32, [P(FaxBlockDims), P(FaxSavedLayout)]),
        "fax_block_bwd_layout": (i32, [P(FaxBlockDims), P(FaxBwdLayout)]),
        "fax_block_workspace_bytes": (i32, [P(FaxBlockDims), P(sz)]),
        "fax_train_workspace_bytes": (i32, [P(FaxModelDims), P(sz)]),
        "fax_eval_workspace_bytes": (i32, [P(FaxModelDims), P(sz)]),
        "fax_eval_step": (i32, [P(FaxModelDims), P(FaxModelTensors), vp, vp, vp, vp, sz, vp]),
        "fax_block_fwd": (i32, [P(FaxBlockDims), P(FaxBlockTensors), vp, vp, vp, vp, vp, vp, sz, vp]),
        "fax_block_bwd": (i32, [P(FaxBlockDims), P(FaxBlockTensors), vp, vp, vp, vp, P(FaxBlockTensors), i32,
                                vp, vp, vp, sz, vp]),
        "fax_adamw_step": (i32, [vp, vp, vp, vp, i32, vp, sz, P(FaxAdamW), i32, vp]),
        "fax_adamw_block_step": (i32, [P(FaxBlockDims)] + [P(FaxBlockTensors)] * 5 + [P(FaxAdamW), i32, vp]),
        "fax_train_step": (i32, [P(FaxModelDims)] + [P(FaxModelTensors)] * 5 + [vp, vp, P(FaxAdamW), i32, vp, vp,
                                                                                  sz, vp]),
        "fax_gemm": (i32, [i32] * 6 + [vp, i32, vp, i32, vp, i32, i32, i32, vp, vp, i32, i32, vp]),
        "fax_layernorm_fwd": (i32, [i32, i32, i32, vp, vp, vp, f32, vp, vp, vp, vp]),
        "fax_layernorm_bwd": (i32, [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]),
        "fax_layernorm_bwd_workspace_bytes": (sz, [i32]),
        "fax_attention_fwd": (i32, [i32] * 5 + [vp, vp, vp, i32, vp]),
        "fax_attention_bwd": (i32, [i32] * 5 + [vp, vp, vp, vp, vp, vp, i32, vp]),
        "fax_cross_entropy": (i32, [i32, i32, i32, vp, vp, vp, vp, vp, vp]),
        "fax_cross_entropy_static": (i32, [i32, i32, i32, vp, vp, vp, vp, vp]),
        "fax_cross_entropy_static_max_rows": (i32, []),
        "fax_probe_mfma": (i32, [i32, i32, C.c_uint, vp, vp]),
        "fax_probe_copy": (i32, [vp, vp, sz, vp]),
        "fax_analyze": (i32, [P(FaxModelDims), P(FaxMesh), P(FaxAnalysis)]),
        "fax_timing_enable": (i32, [i32]),
        "fax_timing_report": (i32, [P(FaxKernelTime), i32, P(i32)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib, tuple(sig)


_lib, EXPORTS = _load()


def _check(status):
    if status != FAX_OK:
        raise FaxError(status, _lib.fax_last_error().decode())


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors handed to libfax must be contiguous"
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def dtype_code(t):
    return {torch.float32: FAX_F32, torch.bfloat16: FAX_BF16}[t.dtype if isinstance(t, torch.Tensor) else t]


def block_dims(B, S, D, H, dh, F, dtype, gelu=FAX_GELU_TANH, ln_eps=1e-5, flags=0):
    return FaxBlockDims(B, S, D, H, dh, F, dtype, gelu, ln_eps, flags)


def block_tensors(d):
    """dict name -> tensor (or FaxBlockTensors) -> FaxBlockTensors."""
    if isinstance(d, FaxBlockTensors):
        return d
    return FaxBlockTensors(*[_ptr(d[n]) for n in TENSOR_NAMES])


class _ModelTensors:
    """Keeps the host array of per-block pointer tables alive next to the struct."""

    def __init__(self, d):
        blocks = d["blocks"]
        self.arr = (FaxBlockTensors * len(blocks))(*[block_tensors(b) for b in blocks])
        self.struct = FaxModelTensors(_ptr(d["tok_emb"]), _ptr(d["pos_emb"]), _ptr(d["lnf_g"]), _ptr(d["lnf_b"]),
                                      C.cast(self.arr, C.POINTER(FaxBlockTensors)))


def model_tensors(d):
    return d if isinstance(d, _ModelTensors) or d is None else _ModelTensors(d)


# ---- entry points, same names and argument order as the C ABI -----------------------------------
def fax_version():
    return _lib.fax_version().decode()


def fax_last_error():
    return _lib.fax_last_error().decode()


def fax_block_dims_check(dims):
    return _lib.fax_block_dims_check(C.byref(dims))


def fax_gemm_plan(M, N, K, c_f32=0):
    """-> (tail, tile_m, tile_n, splits): the launch plan of a bf16 product (host only)."""
    out = FaxGemmPlan()
    _check(_lib.fax_gemm_plan(M, N, K, int(c_f32), C.byref(out)))
    return (out.tail, out.tile_m, out.tile_n, out.splits)


def fax_gemm_tile_walk(M, N, K, c_f32=0):
    """-> (group, [(tile_row, tile_col), ...] in work-item order) of the plan's bulk launch (host only)."""
    count, group = C.c_int(0), C.c_int(0)
    _check(_lib.fax_gemm_tile_walk(M, N, K, int(c_f32), None, None, 0, C.byref(count), C.byref(group)))
    n = count.value
    rows = (C.c_int32 * max(n, 1))(); cols = (C.c_int32 * max(n, 1))()
    _check(_lib.fax_gemm_tile_walk(M, N, K, int(c_f32), C.cast(rows, C.c_void_p), C.cast(cols, C.c_void_p), n,
                                   C.byref(count), C.byref(group)))
    return group.value, [(rows[i], cols[i]) for i in range(n)]


def fax_block_saved_layout(dims):
    out = FaxSavedLayout()
    _check(_lib.fax_block_saved_layout(C.byref(dims), C.byref(out)))
    return out


def fax_block_bwd_layout(dims):
    out = FaxBwdLayout()
    _check(_lib.fax_block_bwd_layout(C.byref(dims), C.byref(out)))
    return out


def fax_block_workspace_bytes(dims):
    out = C.c_size_t()
    _check(_lib.fax_block_workspace_bytes(C.byref(dims), C.byref(out)))
    return out.value


def fax_train_workspace_bytes(mdims):
    out = C.c_size_t()
    _check(_lib.fax_train_workspace_bytes(C.byref(mdims), C.byref(out)))
    return out.value


def fax_eval_workspace_bytes(mdims):
    out = C.c_size_t()
    _check(_lib.fax_eval_workspace_bytes(C.byref(mdims), C.byref(out)))
    return out.value


def fax_analyze(mdims, data=1, tensor=1):
    """mdims: the GLOBAL model; returns the FaxAnalysis of one device of a data x tensor mesh."""
    out = FaxAnalysis()
    _check(_lib.fax_analyze(C.byref(mdims), C.byref(FaxMesh(data, tensor)), C.byref(out)))
    return out


def fax_eval_step(mdims, params, tokens, labels, loss_out, ws, ws_bytes, stream=None):
    tab = model_tensors(params)
    _check(_lib.fax_eval_step(C.byref(mdims), C.byref(tab.struct) if tab is not None else None, _ptr(tokens), _ptr(labels), _ptr(loss_out), _ptr(ws),
                              ws_bytes, _stream(stream)))


def fax_block_fwd(dims, params, x, y, saved, p_attn=None, p_mlp=None, ws=None, ws_bytes=0, stream=None):
    _check(_lib.fax_block_fwd(C.byref(dims), C.byref(block_tensors(params)), _ptr(x), _ptr(y), _ptr(saved),
                              _ptr(p_attn), _ptr(p_mlp), _ptr(ws), ws_bytes, _stream(stream)))


def fax_block_bwd(dims, params, x, dy, saved, dx, grads, accumulate, dh1_partial, dh2_partial, ws, ws_bytes, stream=None):
    _check(_lib.fax_block_bwd(C.byref(dims), C.byref(block_tensors(params)), _ptr(x), _ptr(dy), _ptr(saved), _ptr(dx),
                              C.byref(block_tensors(grads)), int(accumulate), _ptr(dh1_partial), _ptr(dh2_partial),
                              _ptr(ws), ws_bytes, _stream(stream)))


def fax_adamw_step(master, m, v, grad, grad_dtype, lowp, n, hp, step, stream=None):
    _check(_lib.fax_adamw_step(_ptr(master), _ptr(m), _ptr(v), _ptr(grad), int(grad_dtype), _ptr(lowp), n, C.byref(hp),
                               step, _stream(stream)))


def fax_adamw_block_step(dims, master, m, v, grads, lowp, hp, step, stream=None):
    """master, m, v, grads, lowp: FaxBlockTensors (see block_tensors); lowp may be None."""
    _check(_lib.fax_adamw_block_step(C.byref(dims), C.byref(master), C.byref(m), C.byref(v), C.byref(grads),
                                     C.byref(lowp) if lowp is not None else None, C.byref(hp), step, _stream(stream)))


def fax_train_step(mdims, params, master, m, v, grads, tokens, labels, hp, step, loss_out, ws, ws_bytes, stream=None):
    tabs = [model_tensors(t) for t in (params, master, m, v, grads)]
    refs = [C.byref(t.struct) if t is not None else None for t in tabs]
    _check(_lib.fax_train_step(C.byref(mdims), *refs, _ptr(tokens), _ptr(labels),
                               C.byref(hp) if hp is not None else None, step, _ptr(loss_out), _ptr(ws), ws_bytes,
                               _stream(stream)))


def fax_gemm(dtype, ta, tb, M, N, K, A, lda, B, ldb, Cmat, ldc, c_f32=0, accumulate=0, bias=None, residual=None,
             ldr=0, path=PATH_AUTO, stream=None):
    _check(_lib.fax_gemm(dtype, int(ta), int(tb), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(Cmat), ldc, int(c_f32),
                         int(accumulate), _ptr(bias), _ptr(residual), ldr, path, _stream(stream)))


def fax_layernorm_fwd(dtype, rows, D, x, gamma, beta, eps, h, mu, rstd, stream=None):
    _check(_lib.fax_layernorm_fwd(dtype, rows, D, _ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(h), _ptr(mu),
                                  _ptr(rstd), _stream(stream)))


def fax_layernorm_bwd_workspace_bytes(D):
    return _lib.fax_layernorm_bwd_workspace_bytes(D)


def fax_layernorm_bwd(dtype, rows, D, dh, x, mu, rstd, gamma, dres, dx, dgamma, dbeta, accumulate, ws, ws_bytes,
                      stream=None):
    _check(_lib.fax_layernorm_bwd(dtype, rows, D, _ptr(dh), _ptr(x), _ptr(mu), _ptr(rstd), _ptr(gamma), _ptr(dres),
                                  _ptr(dx), _ptr(dgamma), _ptr(dbeta), int(accumulate), _ptr(ws), ws_bytes,
                                  _stream(stream)))


def fax_attention_fwd(dtype, B, S, H, dh, qkv, ctx, lse, path=PATH_AUTO, stream=None):
    _check(_lib.fax_attention_fwd(dtype, B, S, H, dh, _ptr(qkv), _ptr(ctx), _ptr(lse), path, _stream(stream)))


def fax_attention_bwd(dtype, B, S, H, dh, qkv, ctx, lse, dctx, dqkv, delta, path=PATH_AUTO, stream=None):
    _check(_lib.fax_attention_bwd(dtype, B, S, H, dh, _ptr(qkv), _ptr(ctx), _ptr(lse), _ptr(dctx), _ptr(dqkv),
                                  _ptr(delta), path, _stream(stream)))


def fax_timing_enable(on):
    _check(_lib.fax_timing_enable(int(on)))


def fax_timing_report(capacity=64):
    """-> list of dicts {name, launches, ms, work, unit} (unit 0 = flop, 1 = byte)."""
    rows = (FaxKernelTime * capacity)()
    n = C.c_int(0)
    _check(_lib.fax_timing_report(rows, capacity, C.byref(n)))
    return [dict(name=r.name.decode(), launches=r.launches, ms=r.ms, work=r.work, unit=r.unit) for r in rows[:n.value]]


def fax_cross_entropy(dtype, N, V, logits, labels, dlogits, row_loss, loss_out, stream=None):
    _check(_lib.fax_cross_entropy(dtype, N, V, _ptr(logits), _ptr(labels), _ptr(dlogits), _ptr(row_loss),
                                  _ptr(loss_out), _stream(stream)))


def fax_cross_entropy_static(dtype, N, V, logits, labels, dlogits, loss_out, stream=None):
    _check(_lib.fax_cross_entropy_static(dtype, N, V, _ptr(logits), _ptr(labels), _ptr(dlogits), _ptr(loss_out),
                                         _stream(stream)))


def fax_cross_entropy_static_max_rows():
    return _lib.fax_cross_entropy_static_max_rows()


def fax_probe_mfma(workgroups, iters, seed, sink, stream=None):
    _check(_lib.fax_probe_mfma(workgroups, iters, seed, _ptr(sink), _stream(stream)))


def fax_probe_copy(src, dst, nbytes, stream=None):
    _check(_lib.fax_probe_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)))
