"""Philox-seeded tensors for a block, a stack of blocks, and the full model.

Every tensor is drawn in a fixed order from one counter-based stream, in
float64, then (for the bf16 workloads) rounded once to the nearest bfloat16,
ties to even.  The rounded values are what both the oracle and the device
path receive, so input quantisation is charged to neither.
"""
import numpy as np

PARAM_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
               "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")
MATRIX_NAMES = ("wqkv", "wo", "w1", "w2")


def bf16_bits(a):
    """float array -> uint16 bfloat16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)
    r[nan] = 0x7FC0
    return r


def from_bf16_bits(b):
    """uint16 bfloat16 bit patterns -> float32 array (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(a):
    """Values of `a` rounded to the nearest bfloat16, returned as float64."""
    return from_bf16_bits(bf16_bits(a)).astype(np.float64)


def _store(a, dtype):
    if dtype == "bf16":
        return round_to_bf16(a)
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    raise ValueError(dtype)


def _param_shapes(sh):
    D, Hd, F = sh.D, sh.Hd, sh.F
    return {"ln1_g": (D,), "ln1_b": (D,), "wqkv": (D, 3 * Hd), "bqkv": (3 * Hd,),
            "wo": (Hd, D), "bo": (D,), "ln2_g": (D,), "ln2_b": (D,),
            "w1": (D, F), "b1": (F,), "w2": (F, D), "b2": (D,)}


def make_block_params(sh, rng, generic=False):
    """Block parameters.  Default: the benchmark recipe (matrices N(0,sigma),
    biases 0, gain 1, shift 0).  generic=True perturbs biases, gains and
    shifts too, so that tests exercise every term."""
    p = {}
    for name, shape in _param_shapes(sh).items():
        if name in MATRIX_NAMES:
            a = rng.standard_normal(shape) * sh.sigma_w
        elif name.endswith("_g"):
            a = 1.0 + (0.1 * rng.standard_normal(shape) if generic else 0.0) * np.ones(shape)
        else:
            a = (0.1 * rng.standard_normal(shape) if generic else np.zeros(shape))
        p[name] = _store(a, sh.dtype)
    return p


def make_block_inputs(sh, seed=0, generic=False):
    """(params, x, dy) for one block: x and the upstream gradient ~ N(0,1)."""
    rng = np.random.Generator(np.random.Philox(seed))
    p = make_block_params(sh, rng, generic)
    x = _store(rng.standard_normal((sh.B, sh.S, sh.D)), sh.dtype)
    dy = _store(rng.standard_normal((sh.B, sh.S, sh.D)), sh.dtype)
    return p, x, dy


def make_stack_inputs(sh, seed=0, generic=False):
    """([params]*L, x, dy) for L stacked blocks."""
    rng = np.random.Generator(np.random.Philox(seed))
    ps = [make_block_params(sh, rng, generic) for _ in range(sh.L)]
    x = _store(rng.standard_normal((sh.B, sh.S, sh.D)), sh.dtype)
    dy = _store(rng.standard_normal((sh.B, sh.S, sh.D)), sh.dtype)
    return ps, x, dy


def make_model_inputs(ms, seed=0, generic=False):
    """(params, tokens, labels) for the full model.

    params = {"tok_emb": [V,D], "pos_emb": [S_max,D], "lnf_g", "lnf_b", "blocks": [..]}.
    S+1 ids are drawn per row; tokens are the first S, labels the last S, so
    each label is the next token and every position counts in the loss.
    """
    sh = ms.blk
    rng = np.random.Generator(np.random.Philox(seed))
    p = {"tok_emb": _store(rng.standard_normal((ms.V, sh.D)) * 0.02, sh.dtype),
         "pos_emb": _store(rng.standard_normal((ms.S_max, sh.D)) * 0.02, sh.dtype)}
    if generic:
        p["lnf_g"] = _store(1.0 + 0.1 * rng.standard_normal(sh.D), sh.dtype)
        p["lnf_b"] = _store(0.1 * rng.standard_normal(sh.D), sh.dtype)
    else:
        p["lnf_g"] = np.ones(sh.D)
        p["lnf_b"] = np.zeros(sh.D)
    p["blocks"] = [make_block_params(sh, rng, generic) for _ in range(sh.L)]
    ids = rng.integers(0, ms.V, size=(sh.B, sh.S + 1), dtype=np.int64).astype(np.int32)
    tokens = np.ascontiguousarray(ids[:, :-1])
    labels = np.ascontiguousarray(ids[:, 1:])
    return p, tokens, labels
