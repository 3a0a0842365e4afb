"""GPU parity for the other rotation sizes (2, 4, 32, 128 points; Sec. 4.2 "Hadamard matrix size", App. E.4),
through the C ABI, against the CPU oracle: codes, block scales, tensor scale and amax bit-exact, dequantize with the
inverse rotation bit-exact, Wgrad on two operands rotated the same way within the GEMM bar.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_25149_amd import binding as nv, synth

pytestmark = pytest.mark.gpu

GEMM_TOL = 1e-5
SIZES = (2, 4, 32, 128)


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


def check(xb, d, layout, rounding=nv.ROUND_RNE, rht_seed=0, sr_seed=0):
    q = nv.nvfp4_quantize(to_dev(xb), layout, nv.BLOCK_1x16, rounding, d, rht_seed, sr_seed)
    assert q.desc.col_has_rht == d
    orr = oracle.SR if rounding == nv.ROUND_SR else oracle.RNE
    if layout & nv.LAYOUT_ROW:   # the row copy is never rotated
        ref = oracle.quantize(xb, oracle.ROW, oracle.BLOCK_1x16, orr, False, 0, sr_seed)
        assert_copy_equal(q.row_codes, q.row_scales, q.row_ts, ref, f"d={d} row copy")
    ref = oracle.quantize(xb, oracle.COL, oracle.BLOCK_1x16, orr, True, rht_seed, sr_seed, rht_dim=d)
    assert_copy_equal(q.col_codes, q.col_scales, q.col_ts, ref, f"d={d} col copy")
    return q, ref


# rows: one tile, several tiles, and (for the sizes that allow it) a partly filled last tile; columns with a ragged tail
def shapes_for(d):
    rows = [128, 384] + ([32, 160, 208] if d <= 16 else [32, 160] if d == 32 else [])
    return [(r, c) for r in rows if r % d == 0 for c in (16, 528, 1040)]


@pytest.mark.parametrize("d", SIZES)
@pytest.mark.parametrize("both", [False, True], ids=["col", "row+col"])
def test_quantize_rne(d, both):
    layout = nv.LAYOUT_COL | (nv.LAYOUT_ROW if both else 0)
    for rows, cols in shapes_for(d):
        check(synth.normal_with_outliers(rows, cols, 1.0, 10 * d + rows + cols, frac=0.01), d, layout, rht_seed=2025 + d)
        check(synth.student_t3(rows, cols, 1e-3, 20 * d + rows + cols), d, layout, rht_seed=d)


@pytest.mark.parametrize("d", SIZES)
@pytest.mark.parametrize("both", [False, True], ids=["col", "row+col"])
def test_quantize_sr(d, both):
    layout = nv.LAYOUT_COL | (nv.LAYOUT_ROW if both else 0)
    for rows, cols in shapes_for(d):
        check(synth.normal_with_outliers(rows, cols, 1.0, 30 * d + rows + cols, frac=0.01), d, layout, nv.ROUND_SR,
              rht_seed=77, sr_seed=2 ** 63 + 17 + d)


@pytest.mark.parametrize("d", SIZES)
def test_outlier_spread_names_the_size(d):
    # one outlier per rotation group: every rotated entry has magnitude outlier / sqrt(d)
    rows, cols = 256, 32
    x = np.zeros((rows, cols), dtype=np.float32)
    for g in range(rows // d):
        x[g * d + (g % d), :] = 512.0
    q, _ = check(synth.f32_to_bf16_bits(x), d, nv.LAYOUT_COL, rht_seed=3)
    assert q.col_ts.cpu().numpy()[1] == np.float32(512.0) * np.float32(1.0 / np.sqrt(float(d)))


@pytest.mark.parametrize("d", SIZES)
def test_zero_tensor(d):
    check(np.zeros((128, 64), dtype=np.uint16), d, nv.LAYOUT_ROW | nv.LAYOUT_COL, rht_seed=1)


@pytest.mark.parametrize("d", SIZES)
@pytest.mark.parametrize("out_dtype", [nv.OUT_F32, nv.OUT_BF16], ids=["f32", "bf16"])
def test_dequantize_undoes_the_rotation(d, out_dtype):
    rows, cols = 256, 80
    xb = synth.normal_with_outliers(rows, cols, 1.0, 500 + d, frac=0.01)
    q, ref = check(xb, d, nv.LAYOUT_COL, rht_seed=40 + d)
    got = nv.nvfp4_dequantize(q, nv.COPY_COL, True, out_dtype)
    torch.cuda.synchronize()
    want = oracle.dequantize(ref, True, 40 + d, rht_dim=d)
    if out_dtype == nv.OUT_BF16:
        assert np.array_equal(got.view(torch.int16).cpu().numpy().view(np.uint16), synth.f32_to_bf16_bits(want))
    else:
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))
    # and the rotation really is undone: close to x within the FP4 quantisation error of the rotated tensor
    x = synth.bf16_bits_to_f32(xb)
    err = np.linalg.norm(want.T.astype(np.float64) - x) / np.linalg.norm(x)
    assert err < 0.2


@pytest.mark.parametrize("d", SIZES)
def test_wgrad_on_operands_rotated_alike(d):
    tokens, d_in, d_out = 256, 96, 160
    xb = synth.normal_with_outliers(tokens, d_in, 1.0, 600 + d, frac=0.01)
    gb = synth.student_t3(tokens, d_out, 1e-3, 700 + d)
    qx, rx = check(xb, d, nv.LAYOUT_COL, rht_seed=9)
    qg, rg = check(gb, d, nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.ROUND_SR, rht_seed=9, sr_seed=5)
    want = oracle.gemm_f64(rx, rg)                      # [d_in, d_out]
    for ws in (False, True):
        workspace = (torch.empty(nv.gemm_workspace_bytes(d_in, d_out, tokens), dtype=torch.uint8, device="cuda")
                     if ws else None)
        got = nv.nvfp4_gemm(qx, qg, nv.OP_WGRAD, nv.OUT_F32, workspace=workspace)
        torch.cuda.synchronize()
        g = got.cpu().numpy().astype(np.float64)
        assert np.linalg.norm(g - want) / np.linalg.norm(want) <= GEMM_TOL
    # the rotation cancels in the product: close to the unquantised x^T dy
    x, gy = synth.bf16_bits_to_f32(xb).astype(np.float64), synth.bf16_bits_to_f32(gb).astype(np.float64)
    exact = x.T @ gy
    assert np.linalg.norm(want - exact) / np.linalg.norm(exact) < 0.25


def test_operands_rotated_differently_are_refused():
    xb = synth.normal(128, 64, 1.0, 1)
    gb = synth.normal(128, 32, 1.0, 2)
    qx = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_COL, rht_on_col=128, rht_seed=4)
    qg = nv.nvfp4_quantize(to_dev(gb), nv.LAYOUT_COL, rht_on_col=16, rht_seed=4)
    with pytest.raises(nv.NVFP4Error):
        nv.nvfp4_gemm(qx, qg, nv.OP_WGRAD, nv.OUT_F32)
    with pytest.raises(nv.NVFP4Error):
        nv.nvfp4_quantize(to_dev(synth.normal(160, 64, 1.0, 3)), nv.LAYOUT_COL, rht_on_col=128)   # 160 rows: no whole groups
    with pytest.raises(nv.NVFP4Error):
        nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_COL, rht_on_col=8)
    with pytest.raises(nv.NVFP4Error):
        nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_COL, nv.BLOCK_MX32, rht_on_col=16)
    torch.cuda.synchronize()


def test_layer_backward_follows_the_rotation_size_of_x():
    tokens, d_in, d_out = 256, 128, 192
    xb = synth.normal_with_outliers(tokens, d_in, 1.0, 11, frac=0.01)
    wb = synth.normal(d_in, d_out, 0.02, 12)
    gb = synth.student_t3(tokens, d_out, 1e-3, 13)
    qw = nv.nvfp4_quantize(to_dev(wb), nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16)
    qx = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW | nv.LAYOUT_COL, rht_on_col=128, rht_seed=21)
    ws = torch.empty(nv.linear_workspace_bytes(tokens, d_in, d_out), dtype=torch.uint8, device="cuda")
    dw = torch.zeros((d_in, d_out), dtype=torch.float32, device="cuda")
    dx, qdy = nv.nvfp4_linear_backward(to_dev(gb), qx, qw, dw, ws, sr_seed=8)
    torch.cuda.synchronize()
    assert qdy.desc.col_has_rht == 128 and qdy.desc.rht_seed == 21
    rx = oracle.quantize(xb, oracle.COL, use_rht=True, rht_seed=21, rht_dim=128)
    rg = oracle.quantize(gb, oracle.COL, rounding=oracle.SR, use_rht=True, rht_seed=21, sr_seed=8, rht_dim=128)
    assert_copy_equal(qdy.col_codes, qdy.col_scales, qdy.col_ts, rg, "dY col copy")
    want = oracle.gemm_f64(rx, rg)
    g = dw.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(g - want) / np.linalg.norm(want) <= GEMM_TOL
