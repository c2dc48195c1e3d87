"""CPU-only checks of the C-ABI library: it loads, exports what the header declares, validates
arguments before touching the GPU, and reports consistent buffer layouts."""
import ctypes as C
import os
import re

import pytest

import paper_2204_06514_amd as fax

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "fax.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fax_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert {"fax_block_fwd", "fax_block_bwd", "fax_adamw_step", "fax_train_step"} <= set(names)
    lib = C.CDLL(fax.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(fax.EXPORTS), set(names) ^ set(fax.EXPORTS)


def test_version_names_the_target():
    assert "gfx950" in fax.fax_version()


def _dims(**kw):
    base = dict(B=2, S=64, D=128, H=4, dh=32, F=512, dtype=fax.FAX_F32)
    base.update(kw)
    return fax.block_dims(**base)


def test_dims_validation():
    assert fax.fax_block_dims_check(_dims()) == fax.FAX_OK
    assert fax.fax_block_dims_check(_dims(B=0)) == fax.FAX_ERR_INVALID_ARG
    assert "non-positive" in fax.fax_last_error()
    assert fax.fax_block_dims_check(_dims(dtype=7)) == fax.FAX_ERR_INVALID_ARG
    assert fax.fax_block_dims_check(_dims(gelu=3)) == fax.FAX_ERR_INVALID_ARG
    assert fax.fax_block_dims_check(_dims(dh=512)) == fax.FAX_ERR_UNSUPPORTED
    assert fax.fax_block_dims_check(_dims(H=3, dh=32)) == fax.FAX_OK      # H*dh need not equal D


def test_saved_layout_is_disjoint_and_sized():
    d = _dims(dtype=fax.FAX_BF16)
    lay = fax.fax_block_saved_layout(d)
    T, D, Hd, F = 128, 128, 128, 512
    sizes = {"h1": T * D * 2, "qkv": T * 3 * Hd * 2, "ctx": T * Hd * 2, "lse": 2 * 4 * 64 * 4, "x1": T * D * 2,
             "h2": T * D * 2, "dgelu": T * F * 2, "a": T * F * 2, "mu1": T * 4, "rstd1": T * 4, "mu2": T * 4, "rstd2": T * 4}
    spans = sorted((getattr(lay, k), getattr(lay, k) + n) for k, n in sizes.items())
    for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
        assert a1 <= b0
    assert spans[-1][1] <= lay.total
    assert all(s % 256 == 0 for s, _ in spans)
    bl = fax.fax_block_bwd_layout(d)
    assert bl.total == fax.fax_block_workspace_bytes(d)


def test_null_and_misaligned_pointers_are_rejected_before_any_launch():
    d = _dims()
    good = {n: 4096 for n in fax.TENSOR_NAMES}
    with pytest.raises(fax.FaxError) as e:
        fax.fax_block_fwd(d, dict(good, wo=None), 4096, 8192, 4096, stream=0)
    assert e.value.status == fax.FAX_ERR_INVALID_ARG and "params.wo" in str(e.value)
    with pytest.raises(fax.FaxError) as e:
        fax.fax_block_fwd(d, good, 4096 + 4, 8192, 4096, stream=0)
    assert "aligned" in str(e.value)
    with pytest.raises(fax.FaxError) as e:
        fax.fax_block_fwd(d, good, 4096, 4096, 4096, stream=0)
    assert "alias" in str(e.value)
    with pytest.raises(fax.FaxError) as e:
        fax.fax_block_bwd(d, good, 4096, 4096, 4096, 4096, good, 0, None, None, 4096, 16, stream=0)
    assert e.value.status == fax.FAX_ERR_WORKSPACE
    with pytest.raises(fax.FaxError) as e:                       # the optional partial-sum outputs are checked like the rest
        fax.fax_block_bwd(d, good, 4096, 4096, 4096, 4096, good, 0, 4096 + 8, None, 4096, 1 << 40, stream=0)
    assert "dh1_partial" in str(e.value) and "aligned" in str(e.value)


def test_adamw_and_train_argument_checks():
    hp = fax.FaxAdamW(1e-3, 0.9, 0.999, 1e-8, 0.01)
    with pytest.raises(fax.FaxError):
        fax.fax_adamw_step(4096, 4096, 4096, 4096, fax.FAX_F32, None, 16, hp, 0, stream=0)       # step < 1
    with pytest.raises(fax.FaxError):
        fax.fax_adamw_step(4096, 4096, 4096, 4096, fax.FAX_F32, None, 16, fax.FaxAdamW(1e-3, 1.0, 0.999, 1e-8, 0.0), 1, stream=0)
    fax.fax_adamw_step(None, None, None, None, fax.FAX_F32, None, 0, hp, 1, stream=0)            # n = 0 is a no-op
    with pytest.raises(fax.FaxError) as e:
        fax.fax_adamw_step(4096, 4096, 4096, 4096, 7, None, 16, hp, 1, stream=0)                 # not a dtype
    assert "grad_dtype" in str(e.value)
    md = fax.FaxModelDims(_dims(), 2, 100, 32, 0)                                   # S_max < S
    with pytest.raises(fax.FaxError):
        fax.fax_train_workspace_bytes(md)
    md = fax.FaxModelDims(_dims(), 2, 100, 64, 0)
    assert fax.fax_train_workspace_bytes(md) > 0
    # the validation step keeps one layer's activations, not L: smaller workspace, same dims checks
    assert 0 < fax.fax_eval_workspace_bytes(md) < fax.fax_train_workspace_bytes(md)
    with pytest.raises(fax.FaxError):
        fax.fax_eval_workspace_bytes(fax.FaxModelDims(_dims(), 2, 100, 32, 0))
    with pytest.raises(fax.FaxError):   # NULL parameter table is caught before anything is launched
        fax.fax_eval_step(md, None, 4096, 4096, 4096, 4096, fax.fax_eval_workspace_bytes(md), stream=0)


def test_gemm_argument_checks():
    with pytest.raises(fax.FaxError):
        fax.fax_gemm(fax.FAX_F32, 0, 0, 8, 8, 8, 4096, 4, 4096, 8, 4096, 8, stream=0)   # lda < K
    with pytest.raises(fax.FaxError):
        fax.fax_gemm(fax.FAX_BF16, 0, 0, 8, 8, 8, 4096, 8, 4096, 8, 4096, 8, accumulate=1, stream=0)
    with pytest.raises(fax.FaxError) as e:
        fax.fax_gemm(fax.FAX_F32, 0, 0, 128, 128, 64, 4096, 64, 4096, 128, 4096, 128, path=fax.PATH_MFMA, stream=0)
    assert e.value.status == fax.FAX_ERR_UNSUPPORTED
    fax.fax_gemm(fax.FAX_F32, 0, 0, 0, 8, 8, None, 8, None, 8, None, 8, stream=0)       # empty is a no-op


def test_adamw_hyper_parameters_are_checked_by_every_entry_point_that_takes_them():
    import ctypes as C
    d = _dims()
    good = fax.block_tensors({n: 4096 for n in fax.TENSOR_NAMES})
    bad_hps = [fax.FaxAdamW(1e-3, 0.9, 1.0, 1e-8, 0.0),      # beta2 = 1: infinite bias correction
               fax.FaxAdamW(1e-3, -0.1, 0.999, 1e-8, 0.0),
               fax.FaxAdamW(1e-3, 0.9, 0.999, -1e-8, 0.0),    # negative epsilon
               fax.FaxAdamW(float("nan"), 0.9, 0.999, 1e-8, 0.0)]
    for hp in bad_hps:
        with pytest.raises(fax.FaxError) as e:
            fax.fax_adamw_step(4096, 4096, 4096, 4096, fax.FAX_F32, None, 16, hp, 1, stream=0)
        assert e.value.status == fax.FAX_ERR_INVALID_ARG
        with pytest.raises(fax.FaxError) as e:
            fax.fax_adamw_block_step(d, good, good, good, good, None, hp, 1, stream=0)
        assert e.value.status == fax.FAX_ERR_INVALID_ARG
    # the train step: same check, before anything is launched (all pointers here are fake)
    md = fax.FaxModelDims(_dims(), 1, 100, 64, 0)
    tabs = {"tok_emb": 4096, "pos_emb": 4096, "lnf_g": 4096, "lnf_b": 4096, "blocks": [{n: 4096 for n in fax.TENSOR_NAMES}]}
    for hp in bad_hps:
        with pytest.raises(fax.FaxError) as e:
            fax.fax_train_step(md, tabs, tabs, tabs, tabs, tabs, 4096, 4096, hp, 1, 4096, 4096, 1 << 40, stream=0)
        assert e.value.status == fax.FAX_ERR_INVALID_ARG
    with pytest.raises(fax.FaxError) as e:
        fax.fax_train_step(md, tabs, tabs, tabs, tabs, tabs, 4096, 4096, fax.FaxAdamW(1e-3, 0.9, 0.999, 1e-8, 0.0), 0, 4096, 4096,
                           1 << 40, stream=0)
    assert "step" in str(e.value)
    # NULL output pointers of the size queries
    lib = C.CDLL(fax.LIB_PATH)
    lib.fax_eval_workspace_bytes.argtypes = [C.POINTER(fax.FaxModelDims), C.c_void_p]
    assert lib.fax_eval_workspace_bytes(C.byref(md), None) == fax.FAX_ERR_INVALID_ARG
    lib.fax_gemm_plan.argtypes = [C.c_int] * 4 + [C.c_void_p]
    assert lib.fax_gemm_plan(256, 256, 64, 0, None) == fax.FAX_ERR_INVALID_ARG


def test_gemm_plan_query():
    # the d_model = 4096 block: every product on 256 x 256 tiles, no split, no strip
    for shape in [(8192, 12288, 4096, 0), (8192, 4096, 16384, 0), (4096, 16384, 8192, 1), (16384, 4096, 8192, 1)]:
        assert fax.fax_gemm_plan(*shape) == (0, 256, 256, 1), shape
    # a narrow model's weight gradient over 65536 tokens: the contraction is cut into ranges
    tail, tm, tn, splits = fax.fax_gemm_plan(768, 3072, 65536, 1)
    assert tail == 0 and splits > 1 and 65536 // 64 // splits >= 8
    # the bf16-output forms never split
    assert fax.fax_gemm_plan(768, 3072, 65536, 0)[3] == 1
    # a vocabulary that is an odd multiple of 128: bulk on 256-wide tiles, last 128 apart
    assert fax.fax_gemm_plan(65536, 50304, 768, 0)[0] == 2
    assert fax.fax_gemm_plan(50304, 768, 65536, 1)[0] == 1
    # no tile class divides the shape: the scalar kernel's job
    assert fax.fax_gemm_plan(100, 72, 64, 0)[1] == 0
    with pytest.raises(fax.FaxError):
        fax.fax_gemm_plan(0, 128, 64)


def test_gemm_tile_walks_visit_every_tile_once():
    """The persistent GEMM hands its output tiles to the workgroups in one of three orders, chosen per
    shape.  Each must be a bijection onto the tile grid; the side-by-side walk must give every round of
    256 work items a 16 x 16 block of tiles and every XCD (work items with equal number mod 8) a 4 x 8
    block of it; the grouped walks must give an XCD's 32 tiles of a round at most 12 operand panels
    when the shape holds whole blocks."""
    shapes = [  # the benchmark shapes: forward, input-gradient and weight-gradient products
        (8192, 12288, 4096, 0), (8192, 4096, 4096, 0), (8192, 16384, 4096, 0), (8192, 4096, 16384, 0),
        (4096, 12288, 8192, 1), (4096, 4096, 8192, 1), (4096, 16384, 8192, 1), (16384, 4096, 8192, 1),
        (16384, 4608, 12288, 0), (16384, 12288, 1536, 0), (16384, 6144, 12288, 0), (12288, 4608, 16384, 1),
        (16384, 6144, 2048, 0), (16384, 2048, 8192, 0), (2048, 8192, 16384, 1),
        (65536, 2304, 768, 0), (65536, 768, 3072, 0), (768, 3072, 65536, 1), (65536, 50304, 768, 0), (50304, 768, 65536, 1),
        (8192, 3072, 1024, 0), (1024, 4096, 8192, 1), (2048, 1920, 5120, 0), (2048, 5120, 640, 0), (5120, 2560, 2048, 1),
        # odd tile counts and single rows / columns of tiles
        (256, 256, 64, 0), (1280, 256, 1024, 0), (256, 3328, 2048, 0), (2304, 1792, 4096, 0), (128, 128, 64, 0)]
    seen_groups = set()
    for M, N, K, f32 in shapes:
        tail, tile_m, tile_n, splits = fax.fax_gemm_plan(M, N, K, f32)
        group, walk = fax.fax_gemm_tile_walk(M, N, K, f32)
        tiles_m = (M - 128 if tail == 1 else M) // tile_m
        tiles_n = (N - 128 if tail == 2 else N) // tile_n
        assert len(walk) == tiles_m * tiles_n, (M, N, K)
        assert sorted(walk) == [(r, c) for r in range(tiles_m) for c in range(tiles_n)], (M, N, K, group)
        seen_groups.add(group)
        if group == 0:
            assert tiles_m % 16 == 0 and tiles_n % 16 == 0 and splits == 1
            for rnd in range(len(walk) // 256):
                blk = walk[256 * rnd:256 * rnd + 256]
                r0, c0 = min(r for r, _ in blk), min(c for _, c in blk)
                assert r0 % 16 == 0 and c0 % 16 == 0
                assert all(r0 <= r < r0 + 16 and c0 <= c < c0 + 16 for r, c in blk)
                for x in range(8):
                    mine = blk[x::8]
                    assert len({r for r, _ in mine}) == 4 and len({c for _, c in mine}) == 8, (M, N, K, rnd, x)
        elif len(walk) % 256 == 0 and tiles_n % (32 // group) == 0 and tiles_m % group == 0 and (len(walk) // 8) % 32 == 0:
            for rnd in range(len(walk) // 256):
                blk = walk[256 * rnd:256 * rnd + 256]
                for x in range(8):
                    mine = blk[x::8]
                    assert len({r for r, _ in mine}) + len({c for _, c in mine}) <= 12, (M, N, K, group, rnd, x)
    assert seen_groups >= {0, 4, 8}
    # no tile class: nothing to walk
    assert fax.fax_gemm_tile_walk(100, 72, 64, 0) == (-1, [])


def test_static_cross_entropy_checks_its_arguments_before_any_launch():
    assert fax.fax_cross_entropy_static_max_rows() == 1 << 18
    with pytest.raises(fax.FaxError) as e:
        fax.fax_cross_entropy_static(fax.FAX_BF16, (1 << 18) + 1, 512, 4096, 4096, 4096, 4096, stream=0)
    assert e.value.status == fax.FAX_ERR_WORKSPACE and "262144" in str(e.value)
    with pytest.raises(fax.FaxError) as e:
        fax.fax_cross_entropy_static(fax.FAX_BF16, 16, 512, None, 4096, 4096, 4096, stream=0)
    assert e.value.status == fax.FAX_ERR_INVALID_ARG
    with pytest.raises(fax.FaxError) as e:
        fax.fax_cross_entropy_static(7, 16, 512, 4096, 4096, 4096, 4096, stream=0)
    assert e.value.status == fax.FAX_ERR_INVALID_ARG
