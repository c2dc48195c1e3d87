"""CPU-only checks of the generated GEMM and attention code.

The GEMM main loop issues its slab loads through inline assembly (direct global -> LDS loads), which
the compiler knows nothing about: it neither counts them in its own waits nor knows which
registers they occupy.  Two things therefore have to hold in the emitted gfx950 assembly:

 1. inline assembly never loads into vector registers (an earlier version did, and a register the
    compiler considered dead was reused while the load was in flight); the only memory
    instruction allowed inside an assembly block is the LDS-destination load;
 2. loads of this kind return in order and are counted by vmcnt; walking each kernel in
    straight-line order (which is how the main loop is laid out) with that counter, a workgroup
    barrier is never reached with more of them in flight than one operand slab's worth per wave
    (the A slab just requested, which no wave reads before a later barrier: 8 instructions at
    256-row tiles, 4 at 128-row tiles), and the program never ends with any in flight.

The attention kernels load their tiles the same way and wait for all of them before every barrier
(allowed in flight: none).  Compiler-issued loads are the compiler's own business and are not
modelled here."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2204_06514_amd", "csrc", "kernels_gemm_mfma.hip")
SRC_ATTN = os.path.join(ROOT, "paper_2204_06514_amd", "csrc", "kernels_attn_mfma.hip")
SRC_DKV16 = os.path.join(ROOT, "paper_2204_06514_amd", "csrc", "kernels_attn_dkv16.hip")

ASM_ALLOWED = ("s_mov_b32 m0", "s_nop", "global_load_lds_dword", "s_waitcnt", "s_barrier")


def scan(asm_text, kernel_re=r"_ZN3fax16gemm_mfma_kernel"):
    """-> (kernels scanned, {kernel: [problems]})"""
    kernels = re.split(r"\n(?=" + kernel_re + r"[^\n]*:\s)", asm_text)
    bad = {}
    for k in kernels[1:]:
        name = k.split(":")[0]
        problems, in_asm, in_flight = [], False, 0
        # GEMM, the A slab: 8 load instructions per wave at 256 rows, 4 at 128; attention: nothing
        allowed = 0 if "attn" in name else 8 if "ILi256ELi" in name else 4
        jumps, fell_through = {}, True   # label -> most loads in flight at a jump to it seen so far
        for ln in k.split("s_endpgm")[0].split("\n") + ["s_endpgm"]:
            if "#ASMSTART" in ln:
                in_asm = True
                continue
            if "#ASMEND" in ln:
                in_asm = False
                continue
            ln = ln.split(";")[0].strip()
            if ln.startswith(".LBB") and ln.endswith(":"):
                # a block entered only by jumps from above inherits their count, not that of the
                # block laid out before it (which left with an unconditional branch)
                seen = jumps.get(ln[:-1])
                if fell_through:
                    in_flight = max(in_flight, seen or 0)
                elif seen is not None:
                    in_flight = seen
                fell_through = True
                continue
            if not ln or ln.endswith(":") or ln.startswith("."):
                continue
            m = re.match(r"s_c?branch\w*\s+(\.LBB\w+)", ln)
            if m:
                jumps[m.group(1)] = max(jumps.get(m.group(1), 0), in_flight)
                fell_through = not ln.startswith("s_branch")
                continue
            if in_asm and not ln.startswith(ASM_ALLOWED):
                problems.append("in asm block: " + ln)
            if not in_asm and re.search(r"\bm0\b", ln):
                problems.append("m0 used outside the asm blocks: " + ln)
            m = re.match(r"s_waitcnt.*vmcnt\((\d+)\)", ln)
            if ln.startswith("global_load_lds"):
                in_flight += 1
            elif m:
                in_flight = min(in_flight, int(m.group(1)))
            elif ln.startswith("s_barrier") and in_flight > allowed:
                problems.append("%d LDS loads possibly in flight at s_barrier" % in_flight)
            elif ln.startswith("s_endpgm") and in_flight:
                problems.append("%d LDS loads possibly in flight at s_endpgm" % in_flight)
        if problems:
            bad[name] = problems
    return len(kernels) - 1, bad


def test_scanner_catches_planted_mistakes():
    head = "\n_ZN3fax16gemm_mfma_kernelILi128ELi128Efake:  \n"
    name = head.strip().rstrip(":")
    dma = " ;;#ASMSTART\n s_mov_b32 m0, s5\n s_nop 0\n global_load_lds_dwordx4 v1, s[2:3]\n ;;#ASMEND\n"
    ok = head + dma * 6 + " ;;#ASMSTART\n s_waitcnt vmcnt(4) lgkmcnt(0)\n s_barrier\n ;;#ASMEND\n" \
        + " ;;#ASMSTART\n s_waitcnt vmcnt(0)\n ;;#ASMEND\n s_endpgm\n"
    assert scan(ok) == (1, {})
    no_wait = head + dma * 6 + " s_barrier\n ;;#ASMSTART\n s_waitcnt vmcnt(0)\n ;;#ASMEND\n s_endpgm\n"
    assert "6 LDS loads possibly in flight at s_barrier" in scan(no_wait)[1][name][0]
    no_drain = head + dma + " s_endpgm\n"
    assert "in flight at s_endpgm" in scan(no_drain)[1][name][0]
    reg_load = head + " ;;#ASMSTART\n global_load_dwordx4 v[4:7], v[0:1], off\n ;;#ASMEND\n s_endpgm\n"
    assert "in asm block" in scan(reg_load)[1][name][0]
    # a block after an unconditional branch counts what the jumps to it carry, not what precedes it in the layout
    tail_ok = head + " s_cbranch_scc1 .LBB0_9\n" + dma * 3 + " s_branch .LBB0_1\n.LBB0_9:\n s_endpgm\n"
    assert scan(tail_ok) == (1, {})
    tail_bad = head + dma * 2 + " s_cbranch_scc1 .LBB0_9\n s_branch .LBB0_1\n.LBB0_9:\n s_endpgm\n"
    assert "2 LDS loads possibly in flight at s_endpgm" in scan(tail_bad)[1][name][0]
    m0_clobber = head + " s_mov_b32 m0, -1\n s_endpgm\n"
    assert "m0 used outside" in scan(m0_clobber)[1][name][0]


def _assembly(tmp_path, src, extra=()):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    out = tmp_path / "kernels.s"
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics", "-Xclang",
           "-target-feature", "-Xclang", "-packed-fp32-ops", *extra, "-I", os.path.join(ROOT, "include"), "-S",
           "--cuda-device-only", "-o", str(out), src]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return out.read_text()


def test_direct_to_lds_loads_are_waited_for(tmp_path):
    n, bad = scan(_assembly(tmp_path, SRC))
    assert n >= 60, n
    assert not bad, {k: v[:3] for k, v in bad.items()}


def test_attention_tile_loads_are_waited_for(tmp_path):
    text = _assembly(tmp_path, SRC_ATTN, ("-mllvm", "-amdgpu-mfma-vgpr-form=1"))   # options as in build.py
    n, bad = scan(text, r"_ZN3fax\d+attn_\w+")
    assert n >= 5, n   # forward and dQ at two head widths, dK/dV at 64
    assert not bad, {k: v[:3] for k, v in bad.items()}
    n, bad = scan(_assembly(tmp_path, SRC_DKV16, ("-mllvm", "-amdgpu-mfma-vgpr-form=1")), r"_ZN3fax\d+attn_\w+")
    assert n >= 1, n   # dK/dV at 128
    assert not bad, {k: v[:3] for k, v in bad.items()}
