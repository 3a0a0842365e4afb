#!/usr/bin/env python3
"""Benchmark of the NVFP4 hot path on one MI355X.

One "step" is one NVFP4 linear layer of the 12B model's MLP up-projection,
forward and backward, on 8192 tokens (model dimension 5120, FFN dimension 20480):

    qX  = quantize(X,  row + rotated col, 1x16, RNE)
    qW  = quantize(W,  row + col, 16x16, RNE)
    Y   = gemm(qX, qW, FPROP)  -> bf16  [8192, 20480]   (K = 5120)
    qdY = quantize(dY, row + rotated col, 1x16, SR)
    dX  = gemm(qdY, qW, DGRAD) -> bf16  [8192, 5120]    (K = 20480)
    dW  = gemm(qX, qdY, WGRAD) -> fp32  [5120, 20480]   (K = 8192)
    Xd  = dequantize(qX row copy) -> bf16

Inputs are seeded synthetic tensors already resident in HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

TOKENS, D_MODEL, D_FFN = 8192, 5120, 20480
PEAK_HBM_GBPS = 8000.0
PEAK_MFMA_F16_TFLOPS = 2500.0
PEAK_MFMA_F8_TFLOPS = 5000.0
PEAK_MFMA_F4_TFLOPS = 10100.0

# HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by the 1 GiB calibration
# copy below (profiles/bench_linear_layer_12B_hbm_traffic_pmc.txt).  They cannot be measured from inside
# this script; they are constants of the committed kernels at this workload and are refreshed with the
# profile.  GEMM: average over the step's three nvfp4_gemm calls (decode pass + FP16 GEMM, workspace
# traffic included).  Quantize: the step's three nvfp4_quantize calls together.
MEASURED_TRAFFIC_BYTES = {"gemm_call": 3.53e9, "quantize_calls": 1.65e9}


def make_inputs(torch):
    g = torch.Generator(device="cuda")
    g.manual_seed(20250925)
    x = torch.randn((TOKENS, D_MODEL), generator=g, device="cuda", dtype=torch.float32)
    hit = torch.rand((TOKENS, D_MODEL), generator=g, device="cuda") < 1e-3
    x = torch.where(hit, x * 50.0, x).to(torch.bfloat16)                       # N(0,1) + 0.1% x50 outliers
    w = (torch.randn((D_MODEL, D_FFN), generator=g, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
    z = torch.randn((4, TOKENS, D_FFN), generator=g, device="cuda", dtype=torch.float32)
    dy = (z[0] / torch.sqrt((z[1] ** 2 + z[2] ** 2 + z[3] ** 2) / 3.0) * 1e-3).to(torch.bfloat16)  # 1e-3 * t(3)
    del z, hit
    return x, w, dy


def quant_bytes(n_elems: int, copies: int) -> float:
    """Algorithmic HBM bytes of one quantize call, one-pass accounting: the bf16
    tensor read once, plus per copy n/2 code bytes and n/16 scale bytes."""
    return 2.0 * n_elems + copies * (n_elems / 2.0 + n_elems / 16.0)


def cpu_baseline(torch, nv, x, w):
    """Time the CPU oracle on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    m, n = 8192, 8192
    xb = x[:m].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    wb = w[:, :n].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    oracle.lib()
    t0 = time.perf_counter()
    ox = oracle.quantize(xb, oracle.ROW)
    ow = oracle.quantize(wb, oracle.COL, oracle.BLOCK_16x16)
    t1 = time.perf_counter()
    ref = oracle.gemm_f64(ox, ow)
    t2 = time.perf_counter()
    # spot-check the GPU path on the same sample while we are here
    qx = nv.nvfp4_quantize(x[:m].contiguous(), nv.LAYOUT_ROW)
    qw = nv.nvfp4_quantize(w[:, :n].contiguous(), nv.LAYOUT_COL, nv.BLOCK_16x16)
    y = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP).cpu().numpy().astype(np.float64)
    err = float(np.linalg.norm(y - ref) / np.linalg.norm(ref))
    exact = bool(np.array_equal(qx.row_codes.cpu().numpy(), ox.codes) and
                 np.array_equal(qw.col_codes.cpu().numpy(), ow.codes) and
                 np.array_equal(qx.row_scales.cpu().numpy(), ox.scales))
    flops = 2.0 * m * n * D_MODEL
    q_bytes = quant_bytes(m * D_MODEL, 1) + quant_bytes(D_MODEL * n, 1)
    return {
        "value": flops / (t2 - t0) / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": f"Fprop on {m} tokens x {n} FFN columns: quantize X[{m}x{D_MODEL}] (1x16) and "
                  f"W[{D_MODEL}x{n}] (16x16), fp64 GEMM {m}x{n}x{D_MODEL}",
        "gemm_TFLOPs": flops / (t2 - t1) / 1e12, "quantize_GBps": q_bytes / (t1 - t0) / 1e9,
        "seconds": t2 - t0, "gpu_vs_oracle_rel_fro": err, "gpu_codes_bit_exact": exact,
    }


def mxfp4_comparison(torch, nv, x, w, dy, iters: int = 5):
    """The same layer step in the paper's comparison format MXFP4 (Sec. 2, Sec. 5), which this chip's block-scaled
    FP4 matrix instruction consumes natively: no decode pass, no workspace.  Outside the timed region of `value`."""
    RC = nv.LAYOUT_ROW | nv.LAYOUT_COL
    qx = nv.alloc_qtensor(TOKENS, D_MODEL, RC, block_dim=nv.BLOCK_MX32)
    qw = nv.alloc_qtensor(D_MODEL, D_FFN, RC, block_dim=nv.BLOCK_MX32)
    qdy = nv.alloc_qtensor(TOKENS, D_FFN, RC, block_dim=nv.BLOCK_MX32)
    y = torch.empty((TOKENS, D_FFN), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty((TOKENS, D_MODEL), dtype=torch.bfloat16, device="cuda")
    dw = torch.empty((D_MODEL, D_FFN), dtype=torch.float32, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)
    q_ms, g_ms, total = 0.0, 0.0, 0.0
    for it in range(iters + 1):
        m = [ev() for _ in range(7)]
        m[0].record()
        nv.nvfp4_quantize(x, RC, nv.BLOCK_MX32, nv.ROUND_RNE, True, 2025, 0, out=qx)
        m[1].record()
        nv.nvfp4_quantize(w, RC, nv.BLOCK_MX32, nv.ROUND_RNE, False, 0, 0, out=qw)
        m[2].record()
        nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_BF16, out=y)
        m[3].record()
        nv.nvfp4_quantize(dy, RC, nv.BLOCK_MX32, nv.ROUND_SR, True, 2025, 77 + it, out=qdy)
        m[4].record()
        nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_BF16, out=dx)
        m[5].record()
        nv.nvfp4_gemm(qx, qdy, nv.OP_WGRAD, nv.OUT_F32, out=dw)
        m[6].record()
        torch.cuda.synchronize()
        if it == 0:
            continue                                  # warm-up
        q_ms += m[0].elapsed_time(m[2]) + m[3].elapsed_time(m[4])
        g_ms += m[2].elapsed_time(m[3]) + m[4].elapsed_time(m[6])
        total += m[0].elapsed_time(m[6])
    flops = 2.0 * TOKENS * D_MODEL * D_FFN
    gemm_tflops = 3 * flops / (g_ms / iters * 1e-3) / 1e12
    return {"note": "comparison format, not part of `value`: quantize X, W, dY to MXFP4 (1x32 blocks, UE8M0 scales, one pass, "
                    "32-point RHT, SR on dY) and the three GEMMs on the block-scaled FP4 MFMA",
            "ms_per_step": total / iters, "TFLOPs_step": 3 * flops / (total / iters * 1e-3) / 1e12,
            "gemm_TFLOPs_per_launch_avg": gemm_tflops, "gemm_frac_of_fp4_mfma_peak": gemm_tflops / PEAK_MFMA_F4_TFLOPS,
            "quantize_ms_per_step": q_ms / iters}


def rht_size_sweep(torch, nv, x, dy, iters: int = 5):
    """The Wgrad operands' quantize calls with the rotation sizes the paper ablates (Sec. 4.2 "Hadamard matrix size",
    App. E.4) beside its choice d = 16.  Outside the timed region of `value`."""
    RC = nv.LAYOUT_ROW | nv.LAYOUT_COL
    qx = nv.alloc_qtensor(TOKENS, D_MODEL, RC)
    qdy = nv.alloc_qtensor(TOKENS, D_FFN, RC)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    res = {}
    for d, layout in ((2, RC), (4, RC), (16, RC), (32, RC), (128, RC), (16, RC | nv.LAYOUT_ROW_RHT)):
        tx = tg = 0.0
        for it in range(iters + 1):
            m = [ev() for _ in range(3)]
            m[0].record()
            nv.nvfp4_quantize(x, layout, nv.BLOCK_1x16, nv.ROUND_RNE, d, 2025, 0, out=qx)
            m[1].record()
            nv.nvfp4_quantize(dy, layout, nv.BLOCK_1x16, nv.ROUND_SR, d, 2025, 77 + it, out=qdy)
            m[2].record()
            torch.cuda.synchronize()
            if it:
                tx += m[0].elapsed_time(m[1])
                tg += m[1].elapsed_time(m[2])
        res[f"d{d}" + ("_row_copy_rotated_too" if layout != RC else "")] = {"X_ms": tx / iters, "dY_ms": tg / iters,
                        "GBps_one_pass_accounting": (quant_bytes(TOKENS * D_MODEL, 2) + quant_bytes(TOKENS * D_FFN, 2))
                                                    / ((tx + tg) / iters * 1e-3) / 1e9}
    res["note"] = ("not part of `value`: nvfp4_quantize of X (RNE) and dY (SR), row + rotated col copy, per rotation size; "
                   "d <= 16 rotate inside a lane's 16 rows, d = 32 / 128 exchange through LDS; the last entry also rotates the "
                   "row copy along its columns (the Fprop / Dgrad operands of App. E.4.1)")
    return res


def known_amax_block(torch, nv, x, w, dy, iters: int = 5):
    """The three quantize calls when the amax is already known (nvfp4_amax once, then nvfp4_quantize_with_amax):
    App. B.1's extra pass through device memory is gone.  Outside the timed region of `value`."""
    RC = nv.LAYOUT_ROW | nv.LAYOUT_COL
    cases = {"X_8192x5120_rne_rht": (x, nv.BLOCK_1x16, nv.ROUND_RNE, 16),
             "W_5120x20480_2d": (w, nv.BLOCK_16x16, nv.ROUND_RNE, 0),
             "dY_8192x20480_sr_rht": (dy, nv.BLOCK_1x16, nv.ROUND_SR, 16)}
    ev = lambda: torch.cuda.Event(enable_timing=True)
    res = {}
    for name, (t, bd, rnd, rht) in cases.items():
        q = nv.alloc_qtensor(t.shape[0], t.shape[1], RC, block_dim=bd)
        amax = nv.nvfp4_amax(t, rht, 2025)
        tot = 0.0
        for it in range(iters + 1):
            a, b = ev(), ev()
            a.record()
            nv.nvfp4_quantize_with_amax(t, amax, RC, bd, rnd, rht, 2025, 77 + it, out=q)
            b.record()
            torch.cuda.synchronize()
            if it:
                tot += a.elapsed_time(b)
        ms = tot / iters
        res[name] = {"ms": ms, "GBps": quant_bytes(t.numel(), 2) / (ms * 1e-3) / 1e9}
    res["note"] = "not part of `value`: pass 2 alone with a supplied amax; GB/s = bf16 read once + both copies written"
    return res


def matrix_pipe_context(torch, nv, reps: int = 3, iters: int = 100000):
    """What the FP16 matrix pipe sustains on this machine, measured beside the step: the library's register-only MFMA loop
    (no memory traffic) per operand kind, and the vendor library's FP16 GEMM (torch.matmul) at the Fprop shape on
    random data.  Context for `roofline.frac`; outside the timed region of `value`."""
    ev = lambda: torch.cuda.Event(enable_timing=True)
    buf = torch.empty(nv.MFMA_PROBE_WORKGROUPS * 256, dtype=torch.float32, device="cuda")
    res = {}
    for kind, name in ((0, "ones"), (1, "random_fp16"), (2, "nvfp4_like_values")):
        nv.nvfp4_selftest_mfma_rate(kind, iters // 10, buf)
        a, b = ev(), ev()
        a.record()
        flops = sum(nv.nvfp4_selftest_mfma_rate(kind, iters, buf) for _ in range(reps))
        b.record()
        torch.cuda.synchronize()
        res[f"register_only_mfma_{name}_TFLOPs"] = flops / (a.elapsed_time(b) * 1e-3) / 1e12
    g = torch.Generator(device="cuda").manual_seed(5)
    xa = torch.randn((TOKENS, D_MODEL), generator=g, device="cuda", dtype=torch.float16)
    wb = torch.randn((D_MODEL, D_FFN), generator=g, device="cuda", dtype=torch.float16)
    yc = torch.empty((TOKENS, D_FFN), device="cuda", dtype=torch.float16)
    for _ in range(3):
        torch.matmul(xa, wb, out=yc)
    a, b = ev(), ev()
    a.record()
    for _ in range(10):
        torch.matmul(xa, wb, out=yc)
    b.record()
    torch.cuda.synchronize()
    res["vendor_fp16_gemm_fprop_shape_TFLOPs"] = 10 * 2.0 * TOKENS * D_MODEL * D_FFN / (a.elapsed_time(b) * 1e-3) / 1e12
    res["note"] = ("not part of `value`: v_mfma_f32_16x16x32_f16 in a register-only loop (512 workgroups x 4 wavefronts, 16 "
                   "independent accumulators) per operand kind -- the chip is power-limited, the rate depends on the "
                   "operand bits; and torch.matmul FP16 [8192,5120]x[5120,20480] on N(0,1) data")
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mxfp4", action="store_true", help="skip the MXFP4 comparison block")
    ap.add_argument("--no-rht-sweep", action="store_true", help="skip the rotation-size block")
    ap.add_argument("--no-context", action="store_true", help="skip the matrix-pipe context block")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2509_25149_amd import binding as nv
    nv.load_library()
    torch.cuda.set_device(0)
    x, w, dy = make_inputs(torch)

    RC = nv.LAYOUT_ROW | nv.LAYOUT_COL
    qx = nv.alloc_qtensor(TOKENS, D_MODEL, RC)
    qw = nv.alloc_qtensor(D_MODEL, D_FFN, RC)
    qdy = nv.alloc_qtensor(TOKENS, D_FFN, RC)
    y = torch.empty((TOKENS, D_FFN), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty((TOKENS, D_MODEL), dtype=torch.bfloat16, device="cuda")
    dw = torch.empty((D_MODEL, D_FFN), dtype=torch.float32, device="cuda")
    xd = torch.empty((TOKENS, D_MODEL), dtype=torch.bfloat16, device="cuda")
    # scratch for nvfp4_gemm's decode pass; the three GEMMs have the same M*K + N*K up to permutation
    gemm_ws = torch.empty(max(nv.gemm_workspace_bytes(TOKENS, D_FFN, D_MODEL), nv.gemm_workspace_bytes(TOKENS, D_MODEL, D_FFN),
                              nv.gemm_workspace_bytes(D_MODEL, D_FFN, TOKENS)), dtype=torch.uint8, device="cuda")
    RHT_SEED, SR_SEED = 2025, 0x5EED

    ev = lambda: torch.cuda.Event(enable_timing=True)
    gemm_events, quant_events = [], []

    def step(timed: bool, it: int):
        marks = [ev() for _ in range(8)] if timed else None
        rec = (lambda i: marks[i].record()) if timed else (lambda i: None)
        rec(0)
        nv.nvfp4_quantize(x, RC, nv.BLOCK_1x16, nv.ROUND_RNE, True, RHT_SEED, 0, out=qx)
        rec(1)
        nv.nvfp4_quantize(w, RC, nv.BLOCK_16x16, nv.ROUND_RNE, False, 0, 0, out=qw)
        rec(2)
        nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_BF16, out=y, workspace=gemm_ws)
        rec(3)
        nv.nvfp4_quantize(dy, RC, nv.BLOCK_1x16, nv.ROUND_SR, True, RHT_SEED, SR_SEED + it, out=qdy)
        rec(4)
        nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_BF16, out=dx, workspace=gemm_ws)
        rec(5)
        nv.nvfp4_gemm(qx, qdy, nv.OP_WGRAD, nv.OUT_F32, out=dw, workspace=gemm_ws)
        rec(6)
        nv.nvfp4_dequantize(qx, nv.COPY_ROW, False, nv.OUT_BF16, out=xd)
        rec(7)
        if timed:
            gemm_events.extend([(marks[2], marks[3]), (marks[4], marks[5]), (marks[5], marks[6])])
            quant_events.append([(marks[0], marks[1]), (marks[1], marks[2]), (marks[3], marks[4])])

    # A plain device copy of known size (1 GiB read + 1 GiB write), outside the timed region: under
    # rocprofv3 --pmc it calibrates FETCH_SIZE / WRITE_SIZE against known HBM traffic.
    cal_src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    # the same copy twice more, timed: the box's plain streaming bandwidth, to put beside the quantizer's
    ce0, ce1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ce0.record()
    cal_dst.copy_(cal_src)
    cal_dst.copy_(cal_src)
    ce1.record()
    torch.cuda.synchronize()
    copy_gbps = 2 * 2.0 * (1 << 30) / (ce0.elapsed_time(ce1) * 1e-3) / 1e9
    del cal_src, cal_dst

    for i in range(args.warmup):
        step(False, i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(True, args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gemm_flops = 2.0 * TOKENS * D_MODEL * D_FFN            # per GEMM launch
    step_flops = 3.0 * gemm_flops
    gemm_ms = [a.elapsed_time(b) for a, b in gemm_events]
    gemm_avg_ms = sum(gemm_ms) / len(gemm_ms)
    gemm_tflops = gemm_flops / (gemm_avg_ms * 1e-3) / 1e12
    per_op = {k: sum(gemm_ms[i::3]) / args.steps for i, k in enumerate(("fprop", "dgrad", "wgrad"))}

    n_x, n_w, n_dy = TOKENS * D_MODEL, D_MODEL * D_FFN, TOKENS * D_FFN
    q_ms = [[a.elapsed_time(b) for a, b in trio] for trio in quant_events]
    q_avg = [sum(t[i] for t in q_ms) / len(q_ms) for i in range(3)]
    q_bytes = [quant_bytes(n_x, 2), quant_bytes(n_w, 2), quant_bytes(n_dy, 2)]
    q_gbps = [b / (ms * 1e-3) / 1e9 for b, ms in zip(q_bytes, q_avg)]
    q_total_gbps = sum(q_bytes) / (sum(q_avg) * 1e-3) / 1e9

    out = {
        "metric": "NVFP4 quantize GB/s + block-scaled GEMM TFLOP/s at 12B linear shapes, %roofline",
        "value": step_flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 x f16 -> f32 MFMA on NVFP4 (e2m1 x e4m3) operands decoded exactly to f16", "data": "synthetic",
        "config": {"workload": "one NVFP4 linear layer fwd+bwd at the 12B MLP up-projection shape: 8192 tokens, "
                               "5120 -> 20480 (BASELINE configs 3+4+5 plus Wgrad at the same shape): quantize X, W, dY "
                               "(row + col copies, RHT on the Wgrad copies, SR on dY), Fprop/Dgrad/Wgrad GEMM, dequantize",
                   "tokens": TOKENS, "d_model": D_MODEL, "d_ffn": D_FFN},
        "value_definition": "3 GEMMs x 2*8192*5120*20480 flop divided by the whole step time (quantizers and dequantize included)",
        "gemm": {"TFLOPs_per_launch_avg": gemm_tflops, "ms": per_op,
                 "frac_of_f16_mfma_peak": gemm_tflops / PEAK_MFMA_F16_TFLOPS,
                 "frac_of_fp8_mfma_peak": gemm_tflops / PEAK_MFMA_F8_TFLOPS},
        "quantize": {"GBps_total_one_pass_accounting": q_total_gbps,
                     "per_tensor": {"X_8192x5120_rne_rht": {"ms": q_avg[0], "GBps": q_gbps[0]},
                                    "W_5120x20480_2d": {"ms": q_avg[1], "GBps": q_gbps[1]},
                                    "dY_8192x20480_sr_rht": {"ms": q_avg[2], "GBps": q_gbps[2]}},
                     "note": "call time = clear + amax pass + cast pass; bytes = bf16 read once + both copies written"},
        "roofline": {"kernel": "one nvfp4_gemm call = decode_f16_kernel (A, B) + gemm_f16_kernel (256x256 tiles, plus a "
                               "split-K launch for a partial last round of tiles)",
                     "bound": "mfma", "achieved": gemm_tflops, "peak": PEAK_MFMA_F16_TFLOPS,
                     "unit": "TFLOP/s", "frac": gemm_tflops / PEAK_MFMA_F16_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES["gemm_call"],
                     "flops_per_launch": gemm_flops, "avg_launch_ms": gemm_avg_ms,
                     "note": "peak is the published FP16 dense MFMA rate; what a register-only MFMA loop sustains on this "
                             "box under its power limit is measured in `matrix_pipe_context`"},
        "roofline_quantize": {"kernel": "three nvfp4_quantize calls = amax_kernel + amax_finalize_kernel + cast_kernel each",
                              "bound": "hbm", "achieved": q_total_gbps,
                              "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": q_total_gbps / PEAK_HBM_GBPS,
                              "traffic": MEASURED_TRAFFIC_BYTES["quantize_calls"],
                              "bytes_algorithmic_one_pass": sum(q_bytes),
                              "achieved_two_pass_accounting": (sum(q_bytes) + 2.0 * (n_x + n_w + n_dy)) / (sum(q_avg) * 1e-3) / 1e9,
                              "stream_copy_GBps_measured": copy_gbps,
                              "two_pass_frac_of_stream_copy": (sum(q_bytes) + 2.0 * (n_x + n_w + n_dy)) / (sum(q_avg) * 1e-3) / 1e9 / copy_gbps},
    }
    if not args.no_mxfp4:
        out["mxfp4_comparison"] = mxfp4_comparison(torch, nv, x, w, dy)
    if not args.no_rht_sweep:
        out["rht_size_sweep"] = rht_size_sweep(torch, nv, x, dy)
        out["quantize_with_known_amax"] = known_amax_block(torch, nv, x, w, dy)
    if not args.no_context:
        out["matrix_pipe_context"] = matrix_pipe_context(torch, nv)
        ctx = out["matrix_pipe_context"]
        out["roofline"]["frac_of_register_only_rate_nvfp4_like_values"] = gemm_tflops / ctx["register_only_mfma_nvfp4_like_values_TFLOPs"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(torch, nv, x, w)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
