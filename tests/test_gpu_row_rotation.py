"""GPU parity for the rotated row copy (NVFP4_LAYOUT_ROW_RHT: the random Hadamard transform on the operands of Fprop
and Dgrad, App. E.4.1), through the C ABI, against the CPU oracle: codes, block scales, tensor scale and amax
bit-exact for both copies, dequantize with the inverse rotation bit-exact, Fprop and Dgrad on operands rotated alike
within the GEMM bar, operands rotated differently refused.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_25149_amd import binding as nv, synth

pytestmark = pytest.mark.gpu

GEMM_TOL = 1e-5
ROW, COL, ROT = nv.LAYOUT_ROW, nv.LAYOUT_COL, nv.LAYOUT_ROW_RHT


def to_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def assert_copy_equal(codes, scales, ts, ref, what):
    torch.cuda.synchronize()
    c, s, t = codes.cpu().numpy(), scales.cpu().numpy(), ts.cpu().numpy()
    assert t[1].view(np.uint32) == ref.amax.view(np.uint32), f"{what}: amax {t[1]} vs {ref.amax}"
    assert t[0].view(np.uint32) == ref.s_dec.view(np.uint32), f"{what}: s_dec {t[0]} vs {ref.s_dec}"
    bad_s = np.argwhere(s != ref.scales)
    assert bad_s.size == 0, f"{what}: {len(bad_s)} scale bytes differ, first at {bad_s[0]}"
    bad_c = np.argwhere(c != ref.codes)
    assert bad_c.size == 0, f"{what}: {len(bad_c)} code bytes differ, first at {bad_c[0]}"


def check(xb, col, rounding=nv.ROUND_RNE, rht_seed=0, sr_seed=0):
    """col: None (row copy only), 0 (plain col copy) or 16 (rotated col copy)."""
    layout = ROW | ROT | (COL if col is not None else 0)
    q = nv.nvfp4_quantize(to_dev(xb), layout, nv.BLOCK_1x16, rounding, col or 0, rht_seed, sr_seed)
    assert q.desc.row_has_rht == 16 and q.desc.col_has_rht == (col or 0) and q.desc.rht_seed == rht_seed
    assert q.desc.layout_mask == (layout & 3)
    orr = oracle.SR if rounding == nv.ROUND_SR else oracle.RNE
    ref_row = oracle.quantize(xb, oracle.ROW, oracle.BLOCK_1x16, orr, True, rht_seed, sr_seed)
    assert_copy_equal(q.row_codes, q.row_scales, q.row_ts, ref_row, f"rotated row copy (col={col})")
    ref_col = None
    if col is not None:
        ref_col = oracle.quantize(xb, oracle.COL, oracle.BLOCK_1x16, orr, bool(col), rht_seed, sr_seed)
        assert_copy_equal(q.col_codes, q.col_scales, q.col_ts, ref_col, f"col copy (col={col}) beside a rotated row copy")
    return q, ref_row, ref_col


# one tile, several tiles, partly filled last tiles in both directions
SHAPES = [(16, 16), (128, 512), (384, 1040), (160, 528), (208, 48), (32, 2064)]
COLS = [None, 0, 16]


@pytest.mark.parametrize("col", COLS, ids=["row", "row+plain col", "row+rotated col"])
def test_quantize_rne(col):
    for rows, cols in SHAPES:
        check(synth.normal_with_outliers(rows, cols, 1.0, rows + cols, frac=0.01), col, rht_seed=2025)
        check(synth.student_t3(rows, cols, 1e-3, 7 + rows + cols), col, rht_seed=rows)


@pytest.mark.parametrize("col", COLS, ids=["row", "row+plain col", "row+rotated col"])
def test_quantize_sr(col):
    for rows, cols in SHAPES:
        check(synth.normal_with_outliers(rows, cols, 1.0, 3 * rows + cols, frac=0.01), col, nv.ROUND_SR, rht_seed=77,
              sr_seed=2 ** 63 + 17 + cols)


def test_strided_input():
    base = synth.normal_with_outliers(144, 600, 1.0, 4, frac=0.01)
    view = to_dev(base)[:, 8:8 + 528]
    q = nv.nvfp4_quantize(view, ROW | COL | ROT, nv.BLOCK_1x16, nv.ROUND_SR, 16, 5, 6)
    xb = np.ascontiguousarray(base[:, 8:8 + 528])
    assert_copy_equal(q.row_codes, q.row_scales, q.row_ts, oracle.quantize(xb, oracle.ROW, oracle.BLOCK_1x16, oracle.SR, True, 5, 6),
                      "strided rotated row copy")
    assert_copy_equal(q.col_codes, q.col_scales, q.col_ts, oracle.quantize(xb, oracle.COL, oracle.BLOCK_1x16, oracle.SR, True, 5, 6),
                      "strided rotated col copy")


def test_outlier_spreads_along_the_row():
    rows, cols = 128, 64
    x = np.zeros((rows, cols), dtype=np.float32)
    for r in range(rows):
        x[r, (r * 5) % cols] = 512.0
    q, _, _ = check(synth.f32_to_bf16_bits(x), 0, rht_seed=3)
    assert q.row_ts.cpu().numpy()[1] == np.float32(128.0)
    assert q.col_ts.cpu().numpy()[1] == np.float32(512.0)


def test_zero_tensor():
    check(np.zeros((128, 64), dtype=np.uint16), 16, rht_seed=1)
    check(np.zeros((16, 16), dtype=np.uint16), None, rht_seed=1)


@pytest.mark.parametrize("out_dtype", [nv.OUT_F32, nv.OUT_BF16], ids=["f32", "bf16"])
def test_dequantize_undoes_the_rotation(out_dtype):
    xb = synth.normal_with_outliers(96, 272, 1.0, 500, frac=0.01)
    q, ref, _ = check(xb, 16, rht_seed=40)
    got = nv.nvfp4_dequantize(q, nv.COPY_ROW, True, out_dtype)
    torch.cuda.synchronize()
    want = oracle.dequantize(ref, True, 40)
    if out_dtype == nv.OUT_BF16:
        assert np.array_equal(got.view(torch.int16).cpu().numpy().view(np.uint16), synth.f32_to_bf16_bits(want))
    else:
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))
    x = synth.bf16_bits_to_f32(xb)
    assert np.linalg.norm(want.astype(np.float64) - x) / np.linalg.norm(x) < 0.2
    # without the inverse: the rotated values as stored
    plain = nv.nvfp4_dequantize(q, nv.COPY_ROW, False, nv.OUT_F32)
    torch.cuda.synchronize()
    assert np.array_equal(plain.cpu().numpy().view(np.uint32), oracle.dequantize(ref).view(np.uint32))
    # a copy that is not rotated has nothing to undo
    q2 = nv.nvfp4_quantize(to_dev(xb), ROW | COL, rht_on_col=16, rht_seed=40)
    with pytest.raises(nv.NVFP4Error):
        nv.nvfp4_dequantize(q2, nv.COPY_ROW, True, nv.OUT_F32)


def gemm_close(qa, qb, op, ra, rb, m, n, k):
    want = oracle.gemm_f64(ra, rb)
    for ws in (False, True):
        workspace = torch.empty(nv.gemm_workspace_bytes(m, n, k), dtype=torch.uint8, device="cuda") if ws else None
        got = nv.nvfp4_gemm(qa, qb, op, nv.OUT_F32, workspace=workspace)
        torch.cuda.synchronize()
        g = got.cpu().numpy().astype(np.float64)
        assert np.linalg.norm(g - want) / np.linalg.norm(want) <= GEMM_TOL
    return want


def test_fprop_and_dgrad_on_operands_rotated_alike():
    tokens, d_in, d_out = 256, 192, 320
    xb = synth.normal_with_outliers(tokens, d_in, 1.0, 600, frac=0.01)
    wb = synth.normal(d_in, d_out, 0.02, 601)
    gb = synth.student_t3(tokens, d_out, 1e-3, 602)
    x, w, g = (synth.bf16_bits_to_f32(t).astype(np.float64) for t in (xb, wb, gb))
    qx, rx_row, rx_col = check(xb, 16, rht_seed=9)
    qw, rw_row, rw_col = check(wb, 16, rht_seed=9)                 # 1x16 blocks: a rotated weight has no 16x16 form
    qg, rg_row, rg_col = check(gb, 16, nv.ROUND_SR, rht_seed=9, sr_seed=5)
    y = gemm_close(qx, qw, nv.OP_FPROP, rx_row, rw_col, tokens, d_out, d_in)
    assert np.linalg.norm(y - x @ w) / np.linalg.norm(x @ w) < 0.25
    dx = gemm_close(qg, qw, nv.OP_DGRAD, rg_row, rw_row, tokens, d_in, d_out)
    assert np.linalg.norm(dx - g @ w.T) / np.linalg.norm(g @ w.T) < 0.25
    dw = gemm_close(qx, qg, nv.OP_WGRAD, rx_col, rg_col, d_in, d_out, tokens)
    assert np.linalg.norm(dw - x.T @ g) / np.linalg.norm(x.T @ g) < 0.25


def test_operands_rotated_differently_are_refused():
    xb, wb = synth.normal(128, 64, 1.0, 1), synth.normal(64, 32, 1.0, 2)
    qx = nv.nvfp4_quantize(to_dev(xb), ROW | ROT, rht_seed=4)
    qw_plain = nv.nvfp4_quantize(to_dev(wb), ROW | COL, nv.BLOCK_16x16)
    qw_other = nv.nvfp4_quantize(to_dev(wb), COL, rht_on_col=16, rht_seed=5)
    qw_good = nv.nvfp4_quantize(to_dev(wb), COL, rht_on_col=16, rht_seed=4)
    for bad in (qw_plain, qw_other):
        with pytest.raises(nv.NVFP4Error):
            nv.nvfp4_gemm(qx, bad, nv.OP_FPROP, nv.OUT_F32)
    nv.nvfp4_gemm(qx, qw_good, nv.OP_FPROP, nv.OUT_F32)
    # Dgrad: dY row copy rotated, W row copy not
    qg = nv.nvfp4_quantize(to_dev(synth.normal(128, 32, 1.0, 3)), ROW | ROT, rht_seed=4)
    with pytest.raises(nv.NVFP4Error):
        nv.nvfp4_gemm(qg, qw_plain, nv.OP_DGRAD, nv.OUT_F32)
    # what the flag does not combine with
    for kwargs in (dict(layout_mask=COL | ROT, rht_on_col=16), dict(layout_mask=ROW | ROT, block_dim=nv.BLOCK_16x16),
                   dict(layout_mask=ROW | ROT, block_dim=nv.BLOCK_MX32), dict(layout_mask=ROW | COL | ROT, rht_on_col=4),
                   dict(layout_mask=ROT)):
        with pytest.raises(nv.NVFP4Error):
            nv.nvfp4_quantize(to_dev(xb), **kwargs)
    amax = nv.nvfp4_amax(to_dev(xb))
    with pytest.raises(nv.NVFP4Error):
        nv.nvfp4_quantize_with_amax(to_dev(xb), amax, ROW | ROT)
    torch.cuda.synchronize()


def test_a_later_plain_call_clears_the_mark():
    xb = synth.normal(64, 64, 1.0, 1)
    q = nv.nvfp4_quantize(to_dev(xb), ROW | ROT, rht_seed=4)
    assert q.desc.row_has_rht == 16
    nv.nvfp4_quantize(to_dev(xb), ROW, out=q)
    assert q.desc.row_has_rht == 0 and q.desc.rht_seed == 0
    assert_copy_equal(q.row_codes, q.row_scales, q.row_ts, oracle.quantize(xb, oracle.ROW), "plain row copy")
