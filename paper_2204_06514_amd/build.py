"""Compile the HIP sources under csrc/ into libfax.so (gfx950), in-tree.

Each .hip file is compiled to an object in parallel, then linked.  The flag
that disables packed-fp32 instruction selection is applied to every device
compile.
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfax.so")

SOURCES = ["fax_api.hip", "kernels_norm.hip", "kernels_gemm_simt.hip", "kernels_gemm_mfma.hip",
           "kernels_attn_simt.hip", "kernels_attn_mfma.hip", "kernels_attn_dkv16.hip", "kernels_loss_opt.hip",
           "analyze.hip", "probes.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _hipcc():
    for c in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if c and os.path.exists(c):
            return c
    raise RuntimeError("hipcc not found")


# Per-file additions.  The attention kernels run their softmax arithmetic on MFMA results: with the
# accumulators in AGPRs (the compiler's default under register pressure) every score costs an extra
# copy instruction on the vector unit, which bounds those kernels; the VGPR form avoids most copies.
EXTRA = {"kernels_attn_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "kernels_attn_dkv16.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [_hipcc()] + FLAGS + EXTRA.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    log = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, log))
    return obj, log


def build(verbose=False, jobs=8):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(_compile, SOURCES))
    if verbose:
        for _, log in results:
            if log.strip():
                print(log)
    objs = [o for o, _ in results]
    r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
