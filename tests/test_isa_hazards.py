"""CPU-only check of the generated GEMM code.  An earlier version of the main loop issued its
global loads through inline assembly, where the compiler does not know that the destination
registers are busy until the matching wait; a register it considered dead was reused while the
load was in flight.  The loads now go straight to LDS through a compiler builtin, and this test
stays as a guard: it compiles the kernels to gfx950 assembly and walks every kernel with an exact
model of the load counter (loads return in order; s_waitcnt vmcnt(N) leaves at most N in flight).
No instruction may write a vector register that an in-flight load will still write."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2204_06514_amd", "csrc", "kernels_gemm_mfma.hip")


def _regs(tok):
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def scan(asm_text):
    """-> (kernels scanned, {kernel: [offending instructions]})"""
    kernels = re.split(r"\n(?=_ZN3fax16gemm_mfma_kernel[^\n]*:\s)", asm_text)
    bad = {}
    for k in kernels[1:]:
        name = k.split(":")[0]
        queue, viol = [], []
        for ln in k.split("s_endpgm")[0].split("\n"):
            ln = ln.split(";")[0].strip()
            if not ln or ln.endswith(":") or ln.startswith("."):
                continue
            parts = ln.replace(",", " ").split()
            op = parts[0]
            m = re.match(r"s_waitcnt.*vmcnt\((\d+)\)", ln)
            if m:
                del queue[:max(0, len(queue) - int(m.group(1)))]
                continue
            if op.startswith(("global_load_lds", "buffer_load_lds")):
                queue.append(set())   # lands in LDS: counts towards vmcnt, writes no vector register
                continue
            if op.startswith(("global_load", "buffer_load", "scratch_load")):
                queue.append(_regs(parts[1]))
                continue
            if op.startswith(("v_cmp", "s_", "ds_write", "global_store")):
                continue
            if op.startswith(("v_", "ds_read")) and queue:
                if _regs(parts[1]) & set().union(*queue):
                    viol.append(ln)
        if viol:
            bad[name] = viol
    return len(kernels) - 1, bad


def test_scanner_catches_a_planted_clobber():
    asm = ("\n_ZN3fax16gemm_mfma_kernelIfake:  \n global_load_dwordx4 v[4:7], v[0:1], off\n v_add_u32_e32 v5, v1, v2\n"
           " s_waitcnt vmcnt(0)\n v_add_u32_e32 v6, v1, v2\n s_endpgm\n")
    n, bad = scan(asm)
    assert n == 1 and list(bad.values()) == [["v_add_u32_e32 v5 v1 v2".replace(" v1", ", v1").replace(" v2", ", v2")]]


def test_no_write_to_registers_with_loads_in_flight(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    out = tmp_path / "gemm.s"
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics", "-Xclang",
           "-target-feature", "-Xclang", "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(out), SRC]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    n, bad = scan(out.read_text())
    assert n >= 20, n
    assert not bad, {k: v[:3] for k, v in bad.items()}
