"""bench.py's contract: one JSON line with the agreed fields; more than one GPU is refused with a message."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_probe_library_rejects_bad_arguments():
    """bench.py's measurement aids (bench_probe.hip) are a library of their own; its argument checks need no GPU."""
    import ctypes
    path = os.path.join(ROOT, "libbench_probe.so")
    if not os.path.exists(path):
        pytest.skip("libbench_probe.so is built by __graft_entry__.build()")
    L = ctypes.CDLL(path)
    L.bench_mfma_rate.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    L.bench_stream_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    flops, OUT = ctypes.c_double(0.0), 0x50000
    assert L.bench_mfma_probe_threads() == 512 * 256
    assert L.bench_mfma_rate(0, 10, None, ctypes.byref(flops), None) == -1
    assert L.bench_mfma_rate(0, 10, OUT, None, None) == -1
    assert L.bench_mfma_rate(3, 10, OUT, ctypes.byref(flops), None) == -1
    assert L.bench_mfma_rate(0, 0, OUT, ctypes.byref(flops), None) == -1
    assert L.bench_mfma_rate(0, (1 << 24) + 1, OUT, ctypes.byref(flops), None) == -1
    assert L.bench_stream_copy(None, OUT, 16, None) == -1
    assert L.bench_stream_copy(OUT, OUT + 4096, 24, None) == -1
    assert L.bench_stream_copy(OUT + 8, OUT + 4096, 32, None) == -1


@pytest.mark.gpu
def test_probe_kernels_compute_what_they_say():
    import torch
    sys.path.insert(0, ROOT)
    import bench
    # all-ones operands: every accumulator entry is 32 * iters, a thread's checksum 16 accumulators x 4 entries of it
    n = bench.probe_lib().bench_mfma_probe_threads()
    buf = torch.zeros(n, dtype=torch.float32, device="cuda")
    flops = bench.mfma_rate(torch, 0, 100, buf)
    torch.cuda.synchronize()
    assert flops == (n // 64) * 100 * 16 * 2 * 16 * 16 * 32
    assert torch.all(buf == 2048.0 * 100).item()
    for kind in (1, 2):
        bench.mfma_rate(torch, kind, 50, buf)
        torch.cuda.synchronize()
        assert torch.isfinite(buf).all().item() and buf.abs().max().item() > 0
    src = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    bench.stream_copy(torch, src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


@pytest.mark.gpu
def test_one_json_line_with_the_agreed_fields():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "2", "--warmup", "1", "--no-cpu-baseline",
                          "--no-mxfp4", "--no-rht-sweep", "--no-layer-calls", "--no-row-scales"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and "workload" in d["config"]
    r = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "mfma_util"):
        assert key in r, key
    for key in ("ms_per_step_median", "ms_per_step_min"):
        assert d[key] <= d["ms_per_step"] * 1.5
    q = d["roofline_quantize"]
    assert q["bound"] == "hbm" and q["peak"] == 8000.0 and abs(q["frac"] - q["achieved"] / q["peak"]) < 1e-9
    assert r["bound"] == "mfma" and r["peak"] == 2500.0 and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    assert 0.2 < r["frac"] < 1.0 and d["value"] > 300.0
    assert abs(d["value"] - 3 * 2 * 8192 * 5120 * 20480 / (d["ms_per_step"] * 1e-3) / 1e12) < 1e-6 * d["value"]
