"""Builds libquest.so (the C-ABI HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libquest.so")
PROBE_LIB = os.path.join(_HERE, "libquest_probe.so")   # measurement aid of bench.py (include/quest_probe.h)
SOURCES = ["quest_api.hip", "hadamard_quantize.hip", "hadamard_quantize_mfma.hip",
           "lowbit_gemm.hip", "fp4_gemm.hip", "trust_backward.hip", "trust_backward_mfma.hip", "grad_gemm.hip"]
# per-source extra flags: kernels whose MFMA results are consumed by vector code keep them in VGPRs
EXTRA_FLAGS = {"hadamard_quantize_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
               "trust_backward_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed fp32 VALU forms stay off: plain fp32 ops only
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = False) -> str:
    """Compile every source and link libquest.so; always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objects = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objects.append(obj)
        cmd = [hipcc, *HIPCC_FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    for cmd, proc in procs:
        out = proc.communicate()[0].decode()
        lines = [l for l in out.splitlines() if "not a recognized feature" not in l]
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + "\n".join(lines))
        if verbose and lines:
            print("\n".join(lines))
    tmp = LIB + f".tmp{os.getpid()}"
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objects])
    os.replace(tmp, LIB)
    tmp = PROBE_LIB + f".tmp{os.getpid()}"
    out = subprocess.run([hipcc, *HIPCC_FLAGS, "-shared", os.path.join(CSRC, "peak_probe.hip"), "-o", tmp],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    if out.returncode != 0:
        raise RuntimeError("hipcc failed on peak_probe.hip\n" + out.stdout.decode())
    os.replace(tmp, PROBE_LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
