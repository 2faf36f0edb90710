"""Build libvabft.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libvabft.so")

SOURCES = ["gemm16_bf16_nn.hip", "gemm16_bf16_nt.hip", "gemm16_f16_nn.hip", "gemm16_f16_nt.hip", "gemm8_f8_nt.hip",
           "gemm8_bf8_nt.hip", "gemm16_f8_edge.hip", "api.hip",
           "encode.hip", "blocks.hip", "gemm_f32.hip", "gemm_f64.hip", "probe.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# The FP32 / FP64 kernels need at most 128 accumulator registers: keep them in the ordinary
# vector register file (VGPR-form MFMA).  Left to its heuristic the compiler puts them in the
# accumulation file and copies all of them in and out around the MFMAs of every loop iteration.
EXTRA_FLAGS = {
    "gemm_f32.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "gemm_f64.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "probe.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
}


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and "--hip-link" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


# Translation units whose kernels issue MFMAs and global -> LDS loads from inline assembly: their device
# assembly is checked for pipeline hazards the compiler cannot pad (asm_lint.py).
LINTED = ["gemm16_bf16_nn.hip", "gemm16_bf16_nt.hip", "gemm16_f16_nn.hip", "gemm16_f16_nt.hip"]


def build_library(verbose: bool = True, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(pair):
        src, out_path = pair
        mode = ["-S", "--cuda-device-only"] if out_path.endswith(".s") else ["-c"]
        out = _run([hipcc, *FLAGS, *EXTRA_FLAGS.get(src, []), *mode, os.path.join(CSRC, src), "-o", out_path])
        if verbose and out.strip():
            print(out, file=sys.stderr)
        return out_path

    asms = [os.path.join(OBJ, s.replace(".hip", ".s")) for s in LINTED]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(compile_one, list(zip(SOURCES, objs)) + list(zip(LINTED, asms))))
    sys.path.insert(0, PKG)
    try:
        import asm_lint
    finally:
        sys.path.pop(0)
    problems = []
    for a in asms:
        with open(a) as f:
            problems += asm_lint.lint(f.read())
    if problems:
        raise RuntimeError("pipeline hazards in the generated assembly:\n" + "\n".join(problems))
    out = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if verbose and out.strip():
        print(out, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library())
