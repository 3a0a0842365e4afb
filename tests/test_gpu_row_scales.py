"""GPU parity of the quantizer / dequantizer / GEMM with one tensor-level scale per row of each copy
(NVFP4_LAYOUT_ROW_SCALES; App. B.1, last sentence) against the oracle: codes, block scales, the s_dec and amax vectors
bit for bit; dequantize bit for bit; GEMM within 1e-5 relative Frobenius error of the binary64 product."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2509_25149_amd import binding as nv, synth

pytestmark = pytest.mark.gpu

GEMM_TOL = 1e-5
RS = nv.LAYOUT_ROW_SCALES
RHT_SEED, SR_SEED = 2025, 0x5EED


def to_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def assert_copy(codes, scales, ts, ref, what):
    torch.cuda.synchronize()
    t = ts.cpu().numpy()
    n = ref.outer
    assert t.shape == (2 * n,)
    assert np.array_equal(t[n:].view(np.uint32), ref.amax.view(np.uint32)), f"{what}: amax vector"
    assert np.array_equal(t[:n].view(np.uint32), ref.s_dec.view(np.uint32)), f"{what}: s_dec vector"
    assert np.array_equal(scales.cpu().numpy(), ref.scales), f"{what}: scales differ"
    assert np.array_equal(codes.cpu().numpy(), ref.codes), f"{what}: codes differ"


def check(xb, layout, rounding=nv.ROUND_RNE, rht=False):
    orr = oracle.SR if rounding == nv.ROUND_SR else oracle.RNE
    q = nv.nvfp4_quantize(to_dev(xb), layout | RS, rounding=rounding, rht_on_col=rht, rht_seed=RHT_SEED, sr_seed=SR_SEED)
    assert q.desc.scale_per_row == 1 and q.desc.layout_mask == layout
    refs = {}
    if layout & nv.LAYOUT_ROW:
        refs["row"] = oracle.quantize_row_scales(xb, oracle.ROW, orr, False, 0, SR_SEED)
        assert_copy(q.row_codes, q.row_scales, q.row_ts, refs["row"], "row copy")
    if layout & nv.LAYOUT_COL:
        refs["col"] = oracle.quantize_row_scales(xb, oracle.COL, orr, rht, RHT_SEED, SR_SEED)
        assert_copy(q.col_codes, q.col_scales, q.col_ts, refs["col"], "col copy")
    return q, refs


# 16 x 16: one block; 144 x 2064: ragged in both directions (a second column tile of one block); 128 x 4096: two
# register chunks per thread on the one-pass route; 48 x 20480: ten; 32 x 32768: sixteen, its limit; 32 x 34816:
# past it, so the row copy alone takes the two-pass route too
SHAPES = [(16, 16), (144, 2064), (128, 4096), (48, 20480), (32, 32768), (32, 34816), (272, 528)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("rounding", [nv.ROUND_RNE, nv.ROUND_SR])
def test_row_copy_alone_in_one_pass(shape, rounding):
    xb = synth.normal_with_outliers(shape[0], shape[1], 1.0, 1000 + shape[1], frac=0.01)
    xb[min(3, shape[0] - 1)] = 0                      # an all-zero row: scale vector entry 1, codes 0
    check(xb, nv.LAYOUT_ROW, rounding)


@pytest.mark.parametrize("shape", [(16, 16), (144, 2064), (272, 528), (1024, 1536)])
@pytest.mark.parametrize("layout", [nv.LAYOUT_COL, nv.LAYOUT_ROW | nv.LAYOUT_COL])
@pytest.mark.parametrize("rounding,rht", [(nv.ROUND_RNE, False), (nv.ROUND_RNE, True), (nv.ROUND_SR, True), (nv.ROUND_SR, False)])
def test_col_copy_and_both_copies(shape, layout, rounding, rht):
    xb = synth.student_t3(shape[0], shape[1], 0.02, 1100 + shape[0])
    xb[:, min(5, shape[1] - 1)] = 0                   # an all-zero column
    check(xb, layout, rounding, rht)


def test_rows_of_very_different_magnitude_keep_their_precision():
    """The point of the finer granularity: a row 2^-20 times smaller than the largest still uses the whole FP4 range."""
    xb = synth.normal(64, 256, 1.0, 1200)
    x = synth.bf16_bits_to_f32(xb) * np.exp2(-np.arange(64) % 24)[:, None].astype(np.float32)
    xb = synth.f32_to_bf16_bits(x)
    q, refs = check(xb, nv.LAYOUT_ROW)
    d = nv.nvfp4_dequantize(q, nv.COPY_ROW).cpu().numpy()
    rel = np.linalg.norm(d - x, axis=1) / np.linalg.norm(x, axis=1)
    assert rel.max() < 0.15
    # one scale per tensor: the small rows drown
    qt = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW)
    dt = nv.nvfp4_dequantize(qt, nv.COPY_ROW).cpu().numpy()
    assert (np.linalg.norm(dt - x, axis=1) / np.linalg.norm(x, axis=1)).max() > 0.9


def test_dequantize_matches_the_oracle_bitwise():
    xb = synth.normal_with_outliers(160, 288, 1.0, 1300, frac=0.02)
    q, refs = check(xb, nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.ROUND_RNE, True)
    for copy, ref, undo in ((nv.COPY_ROW, refs["row"], False), (nv.COPY_COL, refs["col"], False), (nv.COPY_COL, refs["col"], True)):
        got = nv.nvfp4_dequantize(q, copy, undo).cpu().numpy()
        want = oracle.dequantize(ref, undo_rht=undo, rht_seed=RHT_SEED)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        got16 = nv.nvfp4_dequantize(q, copy, undo, nv.OUT_BF16)
        assert np.array_equal(got16.view(torch.int16).cpu().numpy().view(np.uint16), synth.f32_to_bf16_bits(want))


def rel_fro(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref) / np.linalg.norm(ref))


def gemm_all_routes(a, b, op, ref):
    m, n = ref.shape
    k = a.rows if op == nv.OP_WGRAD else a.cols
    ws = torch.empty(nv.gemm_workspace_bytes(m, n, k), dtype=torch.uint8, device="cuda")
    fused = nv.nvfp4_gemm(a, b, op, nv.OUT_F32)
    two = nv.nvfp4_gemm(a, b, op, nv.OUT_F32, workspace=ws)
    assert rel_fro(fused.cpu().numpy(), ref) <= GEMM_TOL
    assert rel_fro(two.cpu().numpy(), ref) <= GEMM_TOL
    # entry by entry too: a wrong scale on one small row would vanish in the whole-matrix norm
    row_err = np.linalg.norm(two.cpu().numpy() - ref, axis=1) / np.maximum(np.linalg.norm(ref, axis=1), 1e-300)
    assert row_err.max() <= 4 * GEMM_TOL
    assert torch.equal(nv.nvfp4_gemm(a, b, op, nv.OUT_BF16, workspace=ws), two.to(torch.bfloat16))
    assert torch.equal(nv.nvfp4_gemm(a, b, op, nv.OUT_BF16), fused.to(torch.bfloat16))
    acc = two.clone()
    nv.nvfp4_gemm(a, b, op, nv.OUT_F32_ACCUMULATE, out=acc, workspace=ws)
    assert torch.equal(acc, two + two)


@pytest.mark.parametrize("mnk", [(16, 16, 16), (272, 144, 176), (528, 304, 256), (384, 512, 1024)])
def test_gemm_with_row_scales_all_ops(mnk):
    M, N, K = mnk
    x = synth.bf16_bits_to_f32(synth.normal_with_outliers(M, K, 1.0, 1400 + M, frac=0.01))
    x *= np.exp2(-(np.arange(M) % 12))[:, None].astype(np.float32)             # rows of different magnitude
    xb = synth.f32_to_bf16_bits(x)
    wb = synth.normal(K, N, 0.02, 1500 + N)
    dyb = synth.student_t3(M, N, 1e-3, 1600 + M)
    qx, rx = check(xb, nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.ROUND_RNE, True)
    qd, rd = check(dyb, nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.ROUND_SR, True)
    # the weight keeps its per-tensor 16x16 scale (Sec. 4.3): mixed granularity in Fprop and Dgrad
    qw = nv.nvfp4_quantize(to_dev(wb), nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16)
    rw_col, rw_row = oracle.quantize(wb, oracle.COL, oracle.BLOCK_16x16), oracle.quantize(wb, oracle.ROW, oracle.BLOCK_16x16)
    gemm_all_routes(qx, qw, nv.OP_FPROP, oracle.gemm_f64(rx["row"], rw_col))
    gemm_all_routes(qd, qw, nv.OP_DGRAD, oracle.gemm_f64(rd["row"], rw_row))
    gemm_all_routes(qx, qd, nv.OP_WGRAD, oracle.gemm_f64(rx["col"], rd["col"]))   # per-feature scales on both sides
    # a per-row weight (1x16 blocks) on the B side of Dgrad
    qw1, rw1 = check(wb, nv.LAYOUT_ROW)
    gemm_all_routes(qd, qw1, nv.OP_DGRAD, oracle.gemm_f64(rd["row"], rw1["row"]))


@pytest.mark.parametrize("mnk", [(4112, 4368, 128), (4352, 4096, 1024)])
def test_gemm_with_row_scales_and_more_tiles_than_compute_units(mnk):
    """The per-row output stage in the two launch forms the small shapes above do not reach: 306 tiles (ragged last
    row and column) run as streams of tiles by one workgroup per CU; 272 tiles = one whole round + 16 tiles split
    two ways along K, whose partial tiles the sum launch scales per row."""
    M, N, K = mnk
    x = synth.bf16_bits_to_f32(synth.normal_with_outliers(M, K, 1.0, 1700 + M, frac=0.01))
    x *= np.exp2(-(np.arange(M) % 12))[:, None].astype(np.float32)             # rows of different magnitude
    qx, rx = check(synth.f32_to_bf16_bits(x), nv.LAYOUT_ROW, nv.ROUND_RNE, False)
    wb = synth.normal(K, N, 0.02, 1800 + N)
    qw = nv.nvfp4_quantize(to_dev(wb), nv.LAYOUT_COL, nv.BLOCK_16x16)
    gemm_all_routes(qx, qw, nv.OP_FPROP, oracle.gemm_f64(rx["row"], oracle.quantize(wb, oracle.COL, oracle.BLOCK_16x16)))


def test_bad_combinations_are_refused():
    x = to_dev(synth.normal(64, 64, 1.0, 1700))
    for kw in (dict(block_dim=nv.BLOCK_16x16), dict(block_dim=nv.BLOCK_MX32), dict(rht_on_col=4), dict(rht_on_col=128)):
        with pytest.raises(nv.NVFP4Error) as e:
            nv.nvfp4_quantize(x, nv.LAYOUT_ROW | nv.LAYOUT_COL | RS, **kw)
        assert e.value.status == -1, kw
    with pytest.raises(nv.NVFP4Error):
        nv.nvfp4_quantize(x, nv.LAYOUT_ROW | nv.LAYOUT_ROW_RHT | RS, rht_seed=1)
    # a later per-tensor call into the same descriptor clears the mark
    q = nv.nvfp4_quantize(x, nv.LAYOUT_ROW | RS)
    assert q.desc.scale_per_row == 1
    nv.nvfp4_quantize(x, nv.LAYOUT_ROW, out=q)
    assert q.desc.scale_per_row == 0


@pytest.mark.parametrize("name", ["X", "dY"])
def test_full_size_row_copies_in_one_pass(name):
    """The row copies of the 12B layer's activations and gradients (8192 x 5120 RNE, 8192 x 20480 SR)."""
    if name == "X":
        xb, rounding = synth.normal_with_outliers(8192, 5120, 1.0, 301), nv.ROUND_RNE
    else:
        xb, rounding = synth.student_t3(8192, 20480, 1e-3, 401), nv.ROUND_SR
    check(xb, nv.LAYOUT_ROW, rounding)


def test_full_size_both_copies_of_the_gradient():
    xb = synth.student_t3(8192, 20480, 1e-3, 401)
    check(xb, nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.ROUND_SR, True)
