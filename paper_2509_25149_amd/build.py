"""Builds libnvfp4_hip.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import json
import os
import re
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libnvfp4_hip.so")
RESOURCES = os.path.join(PKG, "libnvfp4_hip.resources.json")   # per-kernel register / scratch use, written by the build
SOURCES = ["api.hip", "quantize.hip", "quantize_wide.hip", "quantize_rowrot.hip", "quantize_mx.hip", "gemm.hip", "gemm_f16.hip", "gemm_mx.hip", "dequantize.hip", "selftest.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fPIC", "-shared",
         "-Rpass-analysis=kernel-resource-usage"]   # the compiler reports every kernel's registers, spills and scratch


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-I", os.path.join(ROOT, "include"), "-o", LIB] + \
          [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    remark = "[-Rpass-analysis=kernel-resource-usage]"
    log = "\n".join(line for line in res.stdout.splitlines() if remark not in line)
    if verbose or res.returncode != 0:
        print(log)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libnvfp4_hip.so")
    with open(RESOURCES, "w") as fh:
        json.dump(kernel_resources(res.stdout), fh, indent=1, sort_keys=True)
    return LIB


def kernel_resources(compiler_output: str) -> dict:
    """{mangled kernel name: {"VGPRs": .., "AGPRs": .., "ScratchSize": bytes per lane, "VGPRs Spill": .., ...}}
    from the compiler's kernel-resource-usage remarks."""
    out, cur = {}, None
    for line in compiler_output.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\S+) \[-Rpass", line)
        if m and cur is not None:
            v = m.group(2)
            cur[m.group(1).strip()] = int(v) if v.lstrip("-").isdigit() else v
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
