"""Builds libckv.so (the HIP kernels and their C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
INCLUDE = PKG.parent / "include"
LIB = PKG / "libckv.so"
SCAN_SOURCES = ["ckv_scan_bf16_d128_nq78.hip", "ckv_scan_bf16_d128_nq56.hip", "ckv_scan_bf16_d64_nq78.hip",
                "ckv_scan_bf16_d64_nq56.hip", "ckv_scan_bf16_d128.hip", "ckv_scan_bf16_d64.hip", "ckv_scan_f32_d64.hip",
                "ckv_scan_f32_d128.hip"]
SOURCES = SCAN_SOURCES + ["ckv_api.hip", "ckv_scores.hip", "ckv_tables.hip", "ckv_select.hip", "ckv_gather.hip", "ckv_shared.hip", "ckv_decode.hip"]
# Packed-FP32 instructions are switched off for the device pass (some forms have given wrong
# results on the target machines); the host pass does not know the feature and says so, harmlessly.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


# The scan kernels never produce or consume NaN (masked logits are -inf, never inf - inf), so the
# compiler may skip the NaN-quieting moves it otherwise puts in front of every max.
# MFMA results stay in ordinary vector registers (the vector ALU consumes every one of them); the
# register allocator then parks the MFMA-only operands (Q, K) in accumulation registers instead.
EXTRA_FLAGS = {src: ["-fno-honor-nans", "-mllvm", "-amdgpu-mfma-vgpr-form"] for src in SCAN_SOURCES}


def build_library(verbose: bool = False) -> Path:
    """Compile every source and link libckv.so. Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = PKG / "_build"
    objdir.mkdir(exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = objdir / (src + ".o")
        extra = EXTRA_FLAGS.get(src, [])
        cmd = [hipcc, *FLAGS, *extra, f"-I{INCLUDE}", f"-I{CSRC}", "-c", str(CSRC / src), "-o", str(obj)]
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for src, obj, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out, file=sys.stderr)
        objs.append(str(obj))
    tmp = LIB.with_suffix(f".tmp{os.getpid()}.so")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", str(tmp)], check=True)
    os.replace(tmp, LIB)
    return LIB


def build_probes() -> list:
    """Compile the measurement probes under probes/ (stand-alone HIP programs; not part of the library)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    probes = PKG / "probes"
    subprocess.run([sys.executable, str(probes / "issue_patterns.py")], check=True)
    out = []
    for name in ("read_bandwidth", "issue_patterns"):
        exe = probes / name
        subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-w", "-Xclang", "-target-feature", "-Xclang",
                        "-packed-fp32-ops", str(probes / (name + ".hip")), "-o", str(exe)], check=True)
        out.append(exe)
    return out


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "probes":
        print(*build_probes(), sep="\n")
    else:
        print(build_library(verbose=True))
