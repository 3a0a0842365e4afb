"""GPU parity of the GEMM kernels bench.py times, at the shapes and in the launch configuration it times them.

bench.py's step runs three nvfp4_gemm calls with a lent workspace (decode pass + FP16 MFMA GEMM): Fprop
8192 x 20480 x 5120 to bf16 (2560 tiles of 256 x 256, ten full rounds), Dgrad 8192 x 5120 x 20480 to bf16 (640
tiles, the last 128 split in two along K) and Wgrad 5120 x 20480 x 8192 to FP32 (1600 tiles, the last 64 split in
four along K, non-temporal stores).  Here every element of each result is compared with the oracle's binary64
product of the dequantized operands (App. B.3 Eq. 5): relative Frobenius error over the whole matrix and over every
256 x 256 output tile on its own, so one misplaced tile cannot hide.  The operands are the tensors of BASELINE
configs 3 and 4, quantized the way the step quantizes them (both copies, rotation on the Wgrad copies, stochastic
rounding on dY) and compared bit for bit with the oracle first.  The MXFP4 comparison block of bench.py gets the same
treatment.  These tests are slow on the host side (about half a minute of oracle GEMM each).
"""
import functools

import numpy as np
import pytest
import torch

import oracle
from paper_2509_25149_amd import binding as nv, synth

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

GEMM_TOL = 1e-5
RHT_SEED, SR_SEED = 2025, 0x5EED
TOKENS, D_MODEL, D_FFN = 8192, 5120, 20480
RC = nv.LAYOUT_ROW | nv.LAYOUT_COL


def to_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def assert_copy(codes, scales, ts, ref, what, tensor_scale=True):
    torch.cuda.synchronize()
    if tensor_scale:
        t = ts.cpu().numpy()
        assert t[1].view(np.uint32) == ref.amax.view(np.uint32), f"{what}: amax"
        assert t[0].view(np.uint32) == ref.s_dec.view(np.uint32), f"{what}: s_dec"
    assert np.array_equal(scales.cpu().numpy(), ref.scales), f"{what}: scales differ"
    assert np.array_equal(codes.cpu().numpy(), ref.codes), f"{what}: codes differ"


@functools.lru_cache(maxsize=None)
def source(name):
    """The bf16 tensors of BASELINE configs 3 and 4 (same generators and seeds)."""
    if name == "X":
        return synth.normal_with_outliers(TOKENS, D_MODEL, 1.0, 301)
    if name == "W":
        return synth.normal(D_MODEL, D_FFN, 0.02, 302)
    return synth.student_t3(TOKENS, D_FFN, 1e-3, 401)


@functools.lru_cache(maxsize=None)
def nvfp4_operand(name):
    """(GPU tensor with both copies, oracle row copy, oracle col copy), quantized as bench.py's step does and
    checked bit for bit."""
    xb = source(name)
    if name == "X":
        q = nv.nvfp4_quantize(to_dev(xb), RC, nv.BLOCK_1x16, nv.ROUND_RNE, True, RHT_SEED, 0)
        row = oracle.quantize(xb, oracle.ROW)
        col = oracle.quantize(xb, oracle.COL, use_rht=True, rht_seed=RHT_SEED)
    elif name == "W":
        q = nv.nvfp4_quantize(to_dev(xb), RC, nv.BLOCK_16x16)
        row = oracle.quantize(xb, oracle.ROW, oracle.BLOCK_16x16)
        col = oracle.quantize(xb, oracle.COL, oracle.BLOCK_16x16)
    else:
        q = nv.nvfp4_quantize(to_dev(xb), RC, nv.BLOCK_1x16, nv.ROUND_SR, True, RHT_SEED, SR_SEED)
        row = oracle.quantize(xb, oracle.ROW, rounding=oracle.SR, sr_seed=SR_SEED)
        col = oracle.quantize(xb, oracle.COL, rounding=oracle.SR, use_rht=True, rht_seed=RHT_SEED, sr_seed=SR_SEED)
    assert_copy(q.row_codes, q.row_scales, q.row_ts, row, f"{name} row copy")
    assert_copy(q.col_codes, q.col_scales, q.col_ts, col, f"{name} col copy")
    return q, row, col


@functools.lru_cache(maxsize=None)
def mxfp4_operand(name):
    xb = source(name)
    rnd, ornd = (nv.ROUND_SR, oracle.SR) if name == "dY" else (nv.ROUND_RNE, oracle.RNE)
    rht = name != "W"
    q = nv.nvfp4_quantize(to_dev(xb), RC, nv.BLOCK_MX32, rnd, rht, RHT_SEED, SR_SEED)
    row = oracle.mx_quantize(xb, oracle.ROW, ornd, False, 0, SR_SEED)
    col = oracle.mx_quantize(xb, oracle.COL, ornd, rht, RHT_SEED, SR_SEED)
    assert_copy(q.row_codes, q.row_scales, None, row, f"MXFP4 {name} row copy", tensor_scale=False)
    assert_copy(q.col_codes, q.col_scales, None, col, f"MXFP4 {name} col copy", tensor_scale=False)
    return q, row, col


@functools.lru_cache(maxsize=None)
def step_workspace():
    """One scratch buffer for all three calls, sized as bench.py sizes it."""
    need = max(nv.gemm_workspace_bytes(TOKENS, D_FFN, D_MODEL), nv.gemm_workspace_bytes(TOKENS, D_MODEL, D_FFN),
               nv.gemm_workspace_bytes(D_MODEL, D_FFN, TOKENS))
    return torch.empty(need, dtype=torch.uint8, device="cuda")


def assert_whole_matrix(d_gpu, ref, what):
    """Relative Frobenius error over the whole matrix and over each 256 x 256 output tile."""
    torch.cuda.synchronize()
    got = d_gpu.float().cpu().numpy()
    M, N = ref.shape
    assert got.shape == (M, N)
    err2 = np.zeros((M // 256, N // 256))
    ref2 = np.zeros((M // 256, N // 256))
    for tm in range(M // 256):                              # a band of tile rows at a time keeps the host copies small
        diff = got[tm * 256:(tm + 1) * 256].astype(np.float64) - ref[tm * 256:(tm + 1) * 256]
        err2[tm] = (diff.reshape(256, N // 256, 256) ** 2).sum(axis=(0, 2))
        ref2[tm] = (ref[tm * 256:(tm + 1) * 256].reshape(256, N // 256, 256) ** 2).sum(axis=(0, 2))
    whole = float(np.sqrt(err2.sum() / ref2.sum()))
    worst = float(np.sqrt((err2 / ref2).max()))
    assert whole <= GEMM_TOL, f"{what}: relative Frobenius error over the whole matrix {whole}"
    assert worst <= GEMM_TOL, f"{what}: worst 256x256 tile {np.unravel_index(np.argmax(err2 / ref2), err2.shape)} at {worst}"
    return whole, worst


def bf16_matches_fp32(d16, d32):
    return torch.equal(d16, d32.to(torch.bfloat16))


# ---------------------------------------------------------------- NVFP4: the three calls of the timed step

def test_fprop_two_pass_whole_matrix():
    (qx, rx_row, _), (qw, _, rw_col) = nvfp4_operand("X"), nvfp4_operand("W")
    ws = step_workspace()
    ref = oracle.gemm_f64(rx_row, rw_col)
    y = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_F32, workspace=ws)
    assert_whole_matrix(y, ref, "Fprop FP32")
    y16 = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_BF16, workspace=ws)       # what the step stores
    assert bf16_matches_fp32(y16, y)
    del y16
    fused = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_F32)                     # the route without a workspace
    assert float((y - fused).double().norm() / fused.double().norm()) <= 2e-6
    assert_whole_matrix(fused, ref, "Fprop FP32, fused route")


def test_dgrad_two_pass_whole_matrix():
    (qdy, rdy_row, _), (qw, rw_row, _) = nvfp4_operand("dY"), nvfp4_operand("W")
    ws = step_workspace()
    ref = oracle.gemm_f64(rdy_row, rw_row)
    dx = nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_F32, workspace=ws)
    assert_whole_matrix(dx, ref, "Dgrad FP32")
    dx16 = nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_BF16, workspace=ws)
    assert bf16_matches_fp32(dx16, dx)
    assert torch.equal(nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_F32, workspace=ws), dx)   # split-K sums in a fixed order


def test_wgrad_two_pass_whole_matrix():
    (qx, _, rx_col), (qdy, _, rdy_col) = nvfp4_operand("X"), nvfp4_operand("dY")
    ws = step_workspace()
    ref = oracle.gemm_f64(rx_col, rdy_col)                                     # dW = X^T dY, [5120, 20480]
    dw = nv.nvfp4_gemm(qx, qdy, nv.OP_WGRAD, nv.OUT_F32, workspace=ws)
    assert_whole_matrix(dw, ref, "Wgrad FP32")
    assert torch.equal(nv.nvfp4_gemm(qx, qdy, nv.OP_WGRAD, nv.OUT_F32, workspace=ws), dw)
    # micro-batch accumulation (Sec. 4.1): the same gradient added into a buffer that already holds something
    g = torch.Generator(device="cuda").manual_seed(7)
    prev = torch.randn(dw.shape, generator=g, device="cuda") * float(np.abs(ref).mean())
    acc = prev.clone()
    nv.nvfp4_gemm(qx, qdy, nv.OP_WGRAD, nv.OUT_F32_ACCUMULATE, out=acc, workspace=ws)
    assert torch.equal(acc, prev + dw)
    ref += prev.cpu().numpy().astype(np.float64)
    assert_whole_matrix(acc, ref, "Wgrad FP32 accumulate")
    del acc, prev
    fused = nv.nvfp4_gemm(qx, qdy, nv.OP_WGRAD, nv.OUT_F32)
    assert float((dw - fused).double().norm() / fused.double().norm()) <= 2e-6


def test_bf16_output_with_padded_rows_on_the_two_pass_route():
    """bf16 results leave in 16-byte pieces, so the leading dimension must be a multiple of 8 elements; a padded
    one (N + 8) keeps its padding and equals the rounded FP32 result; N + 4 is refused."""
    M, N, K = 528, 304, 256
    ab, bb = synth.normal_with_outliers(M, K, 1.0, 71), synth.normal(N, K, 0.05, 72)
    qa, qb = nv.nvfp4_quantize(to_dev(ab), nv.LAYOUT_ROW), nv.nvfp4_quantize(to_dev(bb), nv.LAYOUT_ROW)
    ws = torch.empty(nv.gemm_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda")
    d32 = nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_F32, workspace=ws)
    ref = oracle.gemm_f64(oracle.quantize(ab, oracle.ROW), oracle.quantize(bb, oracle.ROW))
    assert float(np.linalg.norm(d32.cpu().numpy() - ref) / np.linalg.norm(ref)) <= GEMM_TOL
    for route_ws in (ws, None):
        buf = torch.full((M, N + 8), 3.0, dtype=torch.bfloat16, device="cuda")
        nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_BF16, out=buf[:, :N], workspace=route_ws)
        torch.cuda.synchronize()
        assert torch.all(buf[:, N:] == 3.0)
        if route_ws is not None:
            assert torch.equal(buf[:, :N], d32.to(torch.bfloat16))
        else:
            assert torch.equal(buf[:, :N], nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_F32).to(torch.bfloat16))
        bad = torch.empty((M, N + 4), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(nv.NVFP4Error) as e:
            nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_BF16, out=bad[:, :N], workspace=route_ws)
        assert e.value.status == -2
    # FP32 keeps the weaker rule (16-byte pieces are 4 elements)
    buf32 = torch.full((M, N + 4), 3.0, dtype=torch.float32, device="cuda")
    nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_F32, out=buf32[:, :N], workspace=ws)
    assert torch.equal(buf32[:, :N], d32) and torch.all(buf32[:, N:] == 3.0)


# ---------------------------------------------------------------- MXFP4: the comparison block at the same shapes

def test_mxfp4_fprop_whole_matrix():
    (qx, rx_row, _), (qw, _, rw_col) = mxfp4_operand("X"), mxfp4_operand("W")
    y = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_F32)
    assert_whole_matrix(y, oracle.mx_gemm_f64(rx_row, rw_col), "MXFP4 Fprop")
    assert bf16_matches_fp32(nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_BF16), y)


def test_mxfp4_dgrad_whole_matrix():
    (qdy, rdy_row, _), (qw, rw_row, _) = mxfp4_operand("dY"), mxfp4_operand("W")
    dx = nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_F32)
    assert_whole_matrix(dx, oracle.mx_gemm_f64(rdy_row, rw_row), "MXFP4 Dgrad")
    assert bf16_matches_fp32(nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_BF16), dx)


def test_mxfp4_wgrad_whole_matrix():
    (qx, _, rx_col), (qdy, _, rdy_col) = mxfp4_operand("X"), mxfp4_operand("dY")
    dw = nv.nvfp4_gemm(qx, qdy, nv.OP_WGRAD, nv.OUT_F32)
    assert_whole_matrix(dw, oracle.mx_gemm_f64(rx_col, rdy_col), "MXFP4 Wgrad")
