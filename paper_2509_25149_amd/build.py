"""Builds libnvfp4_hip.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import json
import os
import re
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libnvfp4_hip.so")
RESOURCES = os.path.join(PKG, "libnvfp4_hip.resources.json")   # per-kernel register / scratch use, written by the build
SOURCES = ["api.hip", "quantize.hip", "quantize_wide.hip", "quantize_rowrot.hip", "quantize_rowscale.hip", "quantize_mx.hip", "gemm.hip", "gemm_f16.hip", "gemm_mx.hip", "dequantize.hip", "selftest.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fPIC",
         "-Rpass-analysis=kernel-resource-usage"]   # the compiler reports every kernel's registers, spills and scratch


def build_library(verbose: bool = False) -> str:
    """One hipcc per source file, a few at a time (no device code crosses a file boundary), then one link."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = max(1, min(len(SOURCES), int(os.environ.get("MAX_JOBS", os.cpu_count() or 1)), 16))
    objdir = tempfile.mkdtemp(prefix="nvfp4_build_")
    remark = "[-Rpass-analysis=kernel-resource-usage]"

    def compile_one(src: str):
        obj = os.path.join(objdir, src + ".o")
        cmd = [hipcc] + FLAGS + ["-I", os.path.join(ROOT, "include"), "-c", os.path.join(CSRC, src), "-o", obj]
        return obj, subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)

    try:
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            done = list(pool.map(compile_one, SOURCES))
        output = "\n".join(res.stdout for _, res in done)
        failed = [src for src, (_, res) in zip(SOURCES, done) if res.returncode != 0]
        link = None
        if not failed:
            link = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [obj for obj, _ in done],
                                  stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            output += "\n" + link.stdout
        log = "\n".join(line for line in output.splitlines() if remark not in line)
        if verbose or failed or link.returncode != 0:
            print(log)
        if failed or link.returncode != 0:
            raise RuntimeError("hipcc failed building libnvfp4_hip.so" + (": " + ", ".join(failed) if failed else " (link)"))
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    with open(RESOURCES, "w") as fh:
        json.dump(kernel_resources(output), fh, indent=1, sort_keys=True)
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


PROBE_SRC = os.path.join(ROOT, "bench_probe.hip")
PROBE_LIB = os.path.join(ROOT, "libbench_probe.so")


def build_bench_probe() -> str:
    """bench.py's measurement aids (a register-only MFMA loop, a plain copy kernel): a library of their own beside
    bench.py, not part of libnvfp4_hip.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-fPIC", "-shared", "-o", PROBE_LIB, PROBE_SRC]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        print(res.stdout)
        raise RuntimeError("hipcc failed building libbench_probe.so")
    return PROBE_LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_bench_probe())
