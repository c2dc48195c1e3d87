"""The end-to-end AdamW comparison used by the GPU tests must reject an update that was skipped,
applied with the wrong sign, or applied without its moments being written.  Checked here on the
CPU by handing it such results in place of the device's (the mistake is planted on this side)."""
import numpy as np
import pytest

from oracle import transformer as orc
from workloads.configs import ADAMW_DEFAULT as HP
from helpers import adamw_step_report


def _case(dtype):
    rng = np.random.default_rng(0)
    p0 = rng.standard_normal((64, 48)) * 0.02
    g = rng.standard_normal((64, 48)) * 3.0
    # what a correct low-precision path returns: gradients off by about half a percent of their scale
    g_dev = g + (5e-3 * 3.0 * rng.standard_normal(g.shape) if dtype == "bf16" else 0.0)
    p, m, v = orc.adamw(p0, 0.0, 0.0, g_dev, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["wd"], 1)
    return p0, g, p, m, v


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_a_correct_update_passes(dtype):
    p0, g, p, m, v = _case(dtype)
    assert adamw_step_report(p, m, v, p0, g, HP, dtype=dtype) == {}


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_a_skipped_update_fails(dtype):
    p0, g, p, m, v = _case(dtype)
    bad = adamw_step_report(p0.copy(), m, v, p0, g, HP, dtype=dtype)
    assert "not_moved" in bad
    bad = adamw_step_report(p, np.zeros_like(m), np.zeros_like(v), p0, g, HP, dtype=dtype)
    assert "m" in bad and "v" in bad


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_a_wrong_sign_fails(dtype):
    p0, g, p, m, v = _case(dtype)
    wrong = p0 + (p0 - p)
    bad = adamw_step_report(wrong, m, v, p0, g, HP, dtype=dtype)
    assert ("displaced_elsewhere" in bad) or ("p" in bad)


def test_weight_decay_left_out_fails_in_fp32():
    p0, g, p, m, v = _case("f32")
    no_decay, _, _ = orc.adamw(p0 * 50, 0.0, 0.0, g, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], 0.0, 1)
    bad = adamw_step_report(no_decay, m, v, p0 * 50, g, HP, dtype="f32")
    assert "p" in bad
