"""The few numbers the paper prints, and the parameter / flop bookkeeping the benchmark relies on."""
import os

from workloads import get_config

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_printed_values.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def test_fp32_parameter_memory_statement():
    g = _golden()
    assert round(6.7e9 * 4 / 2 ** 30) == g["params_6p7B_fp32_GiB"]


def test_workload_sequence_length_matches_the_paper():
    g = _golden()
    for name in ("cfg3", "cfg4"):
        assert get_config(name).S == g["sequence_length"]
    assert get_config("cfg5").blk.S == g["sequence_length"]


def test_parameter_and_flop_counts():
    c1 = get_config("cfg1")
    D, F = c1.D, c1.F
    assert c1.block_param_count() == 4 * D * D + 2 * D * F + 9 * D + F == 198272
    c3 = get_config("cfg3")
    assert abs(c3.block_flops_fwd_bwd(True) - 10.31e12) < 0.01e12      # 3 x (GEMM + causal attention)
    assert abs(c3.block_flops_fwd_bwd(False) - 10.72e12) < 0.01e12
    c5 = get_config("cfg5")
    assert abs(c5.param_count() - 713.4e6) < 0.1e6
    assert abs(c5.flops_fwd_bwd(True) - 74.63e12) < 0.05e12
