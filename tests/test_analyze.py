"""The host-side static analyser (fax_analyze): runs without a GPU.

Pins: the one memory figure the paper states (Sec. 3: a 6.7B-parameter model takes 25 GiB as
float32), the divisibility rule of Sec. 3.2, parameter counts against the element counts of the
tensors the workload generator actually produces, work against the independent formulas in
workloads/configs.py, and memory against the library's own layout calls."""
import numpy as np
import pytest

import paper_2204_06514_amd as fax
from workloads import get_config, make_model_inputs
from workloads.configs import BlockShape, ModelShape

CODE = {"f32": fax.FAX_F32, "bf16": fax.FAX_BF16}


def mdims(ms):
    b = ms.blk
    blk = fax.block_dims(b.B, b.S, b.D, b.H, b.dh, b.F, CODE[b.dtype], fax.FAX_GELU_TANH, b.ln_eps, 0)
    return fax.FaxModelDims(blk, b.L, ms.V, ms.S_max, 0)


def test_memory_of_the_6p7b_model_matches_the_papers_figure():
    # Sec. 3: "6.7B parameters ... 25 GiB ... float32".  The usual shape of that size: 32 layers, width 4096.
    ms = ModelShape(BlockShape(B=1, S=2048, D=4096, H=32, dh=128, F=16384, dtype="bf16", sigma_w=0.02, L=32),
                    V=50304, S_max=2048)
    a = fax.fax_analyze(mdims(ms))
    assert abs(a.params_global - 6.7e9) < 0.1e9
    assert abs(a.bytes_master / 2**30 - 25.0) < 0.5
    # ... and with the optimizer state it no longer fits a 40 GB accelerator, which is the section's point
    assert (a.bytes_master + a.bytes_moments) / 1e9 > 40


def test_parameter_count_equals_the_generated_tensors():
    ms = get_config("cfg5").scaled(V=640, S_max=96, B=2, S=64, D=128, H=4, dh=32, F=256, L=3)
    p, _, _ = make_model_inputs(ms, seed=0)
    n = sum(np.asarray(p[k]).size for k in ("tok_emb", "pos_emb", "lnf_g", "lnf_b"))
    n += sum(np.asarray(t).size for blk in p["blocks"] for t in blk.values())
    a = fax.fax_analyze(mdims(ms))
    assert a.params_global == n == a.params_local == ms.param_count()


@pytest.mark.parametrize("name", ["cfg5", "fig4_124m"])
def test_work_and_memory_agree_with_formulas_and_layouts(name):
    ms = get_config(name)
    md = mdims(ms)
    a = fax.fax_analyze(md)
    assert a.flop_step == ms.flops_fwd_bwd(True)
    assert a.flop_step_unhalved == ms.flops_fwd_bwd(False)
    assert a.bytes_saved == ms.L * fax.fax_block_saved_layout(md.blk).total
    assert a.bytes_saved + a.bytes_workspace == fax.fax_train_workspace_bytes(md)
    assert a.bytes_master == 4 * ms.param_count() and a.bytes_moments == 2 * a.bytes_master
    assert a.bytes_lowp == 2 * ms.param_count()
    assert a.bytes_total == a.bytes_master + a.bytes_moments + a.bytes_grads + a.bytes_lowp + a.bytes_saved + a.bytes_workspace
    assert a.bytes_tensor_axis == 0 and a.bytes_data_axis == 0
    assert a.ms_step == pytest.approx(a.ms_gemm + a.ms_attention + a.ms_bandwidth)
    # the prediction is of the right order: between the time at full MFMA peak and 10x that
    floor_ms = a.flop_step / 2516.6e12 * 1e3
    assert floor_ms < a.ms_step < 10 * floor_ms


def test_local_share_on_a_mesh_is_the_tensor_parallel_config():
    """cfg4 is one of 8 tensor-parallel ranks of a 12288-wide block: the analyser derives its dims."""
    c4 = get_config("cfg4")
    g = ModelShape(BlockShape(B=c4.B * 2, S=c4.S, D=c4.D, H=c4.H * 8, dh=c4.dh, F=c4.F * 8, dtype="bf16", sigma_w=0.006, L=4),
                   V=51200, S_max=2048)
    a = fax.fax_analyze(mdims(g), data=2, tensor=8)
    l = a.local.blk
    assert (l.B, l.S, l.D, l.H, l.dh, l.F) == (c4.B, c4.S, c4.D, c4.H, c4.dh, c4.F)
    assert l.flags & fax.FAX_FLAG_TP_PARTIAL
    assert a.local.V == 51200 // 8
    # sharded: the four matrices and the biases in front of a reduction; replicated: LayerNorm, bo, b2, positions
    D, Hd, F = c4.D, c4.H * c4.dh, c4.F
    per_block = D * 3 * Hd + 3 * Hd + Hd * D + D * F + F + F * D + 6 * D
    assert a.params_local == 4 * per_block + (51200 // 8) * D + 2048 * D + 2 * D
    assert a.params_local < a.params_global / 7
    # exchange volumes: four [T, D] sums per block over the tensor axis, the gradients once over the data axis
    assert a.bytes_tensor_axis == 4 * 4 * (c4.B * c4.S) * D * 2
    assert a.bytes_data_axis == 4 * a.params_local
    # more ranks on the tensor axis: less memory and less predicted time per device
    a4 = fax.fax_analyze(mdims(g), data=2, tensor=4)
    assert a4.bytes_total > a.bytes_total and a4.ms_step > a.ms_step


def test_a_vocabulary_slice_that_would_leave_the_mfma_path_is_not_split():
    g = get_config("fig4_124m")      # 50304 = 393 * 128 rows: no multiple of 128 per rank on 4 ranks
    a = fax.fax_analyze(mdims(g), tensor=4)
    assert a.local.V == 50304 and a.local.blk.H == 3


def test_mesh_must_divide_batch_heads_and_width():
    md = mdims(get_config("cfg5"))     # B=8, H=16, F=8192
    for kw, word in ((dict(data=3), "batch"), (dict(tensor=3), "heads"), (dict(tensor=0), "mesh")):
        with pytest.raises(fax.FaxError) as e:
            fax.fax_analyze(md, **kw)
        assert e.value.status == fax.FAX_ERR_INVALID_ARG and word in str(e.value)
    odd = mdims(get_config("cfg5").scaled(F=8200))
    odd.blk.H = 16
    with pytest.raises(fax.FaxError) as e:
        fax.fax_analyze(odd, tensor=16)
    assert "feed-forward" in str(e.value)
