"""GPU parity of the MXFP4 mode (the paper's comparison format: Sec. 2, App. B.4, Sec. 5) through the C ABI:
quantizer bit-exact against the oracle, dequantize bitwise, GEMM on the block-scaled FP4 matrix instruction
within 1e-5 relative Frobenius error of the oracle's binary64 result."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_25149_amd import binding as nv, synth

pytestmark = pytest.mark.gpu
RHT_SEED, SR_SEED = 20250929, 0xC0FFEE
GEMM_TOL = 1e-5


def to_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def assert_mx_copy(codes, scales, ref, what):
    torch.cuda.synchronize()
    assert np.array_equal(scales.cpu().numpy(), ref.scales), f"{what}: scales differ"
    assert np.array_equal(codes.cpu().numpy(), ref.codes), f"{what}: codes differ"


MODES = {
    "rne": dict(),
    "rne_rht": dict(rht=True),
    "sr": dict(rounding=nv.ROUND_SR),
    "sr_rht": dict(rounding=nv.ROUND_SR, rht=True),
}


@pytest.mark.parametrize("shape", [(128, 512), (32, 32), (160, 608), (384, 1056)])
@pytest.mark.parametrize("mode", sorted(MODES))
def test_mx_quantize_matches_the_oracle(shape, mode):
    m = MODES[mode]
    rounding, rht = m.get("rounding", nv.ROUND_RNE), m.get("rht", False)
    xb = synth.normal_with_outliers(shape[0], shape[1], 1.0, 900 + shape[0], frac=0.01)
    q = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_MX32, rounding, rht_on_col=rht,
                          rht_seed=RHT_SEED, sr_seed=SR_SEED)
    o_round = oracle.SR if rounding == nv.ROUND_SR else oracle.RNE
    r_row = oracle.mx_quantize(xb, oracle.ROW, o_round, False, 0, SR_SEED)
    r_col = oracle.mx_quantize(xb, oracle.COL, o_round, rht, RHT_SEED, SR_SEED)
    assert q.row_scales.shape == (shape[0], shape[1] // 32) and q.col_scales.shape == (shape[1], shape[0] // 32)
    assert_mx_copy(q.row_codes, q.row_scales, r_row, f"row copy {mode}")
    assert_mx_copy(q.col_codes, q.col_scales, r_col, f"col copy {mode}")
    assert q.row_ts.cpu().tolist() == [1.0, 0.0] and q.col_ts.cpu().tolist() == [1.0, 0.0]
    # single copies go through their own kernel instantiations
    q1 = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_COL, nv.BLOCK_MX32, rounding, rht_on_col=rht, rht_seed=RHT_SEED, sr_seed=SR_SEED)
    assert_mx_copy(q1.col_codes, q1.col_scales, r_col, f"col only {mode}")
    if not rht:
        q2 = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW, nv.BLOCK_MX32, rounding, sr_seed=SR_SEED)
        assert_mx_copy(q2.row_codes, q2.row_scales, r_row, f"row only {mode}")
    # decode: bitwise, and the rotated copy comes back through the inverse rotation
    d = nv.nvfp4_dequantize(q, nv.COPY_ROW, False, nv.OUT_F32)
    assert np.array_equal(d.cpu().numpy().view(np.uint32), oracle.mx_dequantize(r_row).view(np.uint32))
    dc = nv.nvfp4_dequantize(q, nv.COPY_COL, rht, nv.OUT_F32)
    assert np.array_equal(dc.cpu().numpy().view(np.uint32), oracle.mx_dequantize(r_col, rht, RHT_SEED).view(np.uint32))
    d16 = nv.nvfp4_dequantize(q, nv.COPY_ROW, False, nv.OUT_BF16)
    assert np.array_equal(d16.view(torch.int16).cpu().numpy().view(np.uint16), synth.f32_to_bf16_bits(d.cpu().numpy()))


def test_mx_degenerate_blocks():
    """All-zero blocks store the smallest scale; powers of two sit exactly on the rounding boundary of the scale."""
    x = np.zeros((32, 128), dtype=np.float32)
    x[0, 0:32] = 6.0            # amax / 6 = 1 exactly -> e = 0, the block maximum encodes as 6
    x[1, 32:64] = 6.03125       # just above -> e = 1
    x[2, 64:96] = 2.0 ** -120
    x[3, :] = -0.0
    xb = synth.f32_to_bf16_bits(x)
    q = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_MX32)
    assert_mx_copy(q.row_codes, q.row_scales, oracle.mx_quantize(xb, oracle.ROW), "row")
    assert_mx_copy(q.col_codes, q.col_scales, oracle.mx_quantize(xb, oracle.COL), "col")
    sc = q.row_scales.cpu().numpy()
    assert sc[0, 0] == 127 and sc[1, 1] == 128 and sc[5, 0] == 0


def rel_fro(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref) / np.linalg.norm(ref))


# K a multiple of 512 takes the kernel with full-line loads (two K steps per stage, scales four steps at a time),
# any other multiple of 128 the general one (with an odd number of K steps for 384 and 640)
@pytest.mark.parametrize("mnk", [(256, 256, 128), (288, 160, 384), (512, 768, 1024), (32, 32, 128), (288, 160, 512),
                                 (544, 96, 1536), (32, 32, 2048), (160, 288, 640)])
def test_mx_gemm_all_ops(mnk):
    M, N, K = mnk
    ab = synth.normal_with_outliers(M, K, 1.0, 910, frac=0.01)
    bb = synth.normal(N, K, 0.05, 911)
    qa = nv.nvfp4_quantize(to_dev(ab), nv.LAYOUT_ROW, nv.BLOCK_MX32)
    qb = nv.nvfp4_quantize(to_dev(bb), nv.LAYOUT_ROW, nv.BLOCK_MX32)
    ra, rb = oracle.mx_quantize(ab, oracle.ROW), oracle.mx_quantize(bb, oracle.ROW)
    ref = oracle.mx_gemm_f64(ra, rb)
    d = nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_F32)                       # D = A B^T, both row copies
    assert d.shape == (M, N) and rel_fro(d.cpu().numpy(), ref) <= GEMM_TOL
    d16 = nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_BF16)
    assert torch.equal(d16, d.to(torch.bfloat16))
    acc = d.clone()
    nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_F32_ACCUMULATE, out=acc)
    assert torch.equal(acc, d + d)
    # Fprop form: B given as the col copy of its transpose [K, N]
    qbt = nv.nvfp4_quantize(to_dev(np.ascontiguousarray(bb.T)), nv.LAYOUT_COL, nv.BLOCK_MX32)
    assert torch.equal(nv.nvfp4_gemm(qa, qbt, nv.OP_FPROP, nv.OUT_F32), d)
    # Wgrad form with the 32-point rotation on both operands (Sec. 5): the rotation cancels in exact arithmetic,
    # the quantized result matches the oracle's for the same rotated operands
    qat = nv.nvfp4_quantize(to_dev(np.ascontiguousarray(ab.T)), nv.LAYOUT_COL, nv.BLOCK_MX32, rht_on_col=True, rht_seed=RHT_SEED)
    qbt2 = nv.nvfp4_quantize(to_dev(np.ascontiguousarray(bb.T)), nv.LAYOUT_COL, nv.BLOCK_MX32, rht_on_col=True, rht_seed=RHT_SEED)
    rat = oracle.mx_quantize(np.ascontiguousarray(ab.T), oracle.COL, use_rht=True, rht_seed=RHT_SEED)
    rbt = oracle.mx_quantize(np.ascontiguousarray(bb.T), oracle.COL, use_rht=True, rht_seed=RHT_SEED)
    dw = nv.nvfp4_gemm(qat, qbt2, nv.OP_WGRAD, nv.OUT_F32)
    assert rel_fro(dw.cpu().numpy(), oracle.mx_gemm_f64(rat, rbt)) <= GEMM_TOL


@pytest.mark.parametrize("K", [512, 1536])
def test_mx_gemm_with_more_tiles_than_compute_units(K):
    """17 x 18 tiles of 256 x 256, the last row and column of them ragged: the kernel for K % 512 == 0 is launched with
    one workgroup per CU, 50 of which run two tiles as one stream of stages (K = 512: one scale chunk per tile, the
    shortest tile; K = 1536: an odd number of chunks, so the scale ring's phase differs from tile to tile)."""
    M, N = 4128, 4384
    ab = synth.normal_with_outliers(M, K, 1.0, 920 + K, frac=0.01)
    bb = synth.normal(N, K, 0.05, 921 + K)
    qa = nv.nvfp4_quantize(to_dev(ab), nv.LAYOUT_ROW, nv.BLOCK_MX32)
    qb = nv.nvfp4_quantize(to_dev(bb), nv.LAYOUT_ROW, nv.BLOCK_MX32)
    ra, rb = oracle.mx_quantize(ab, oracle.ROW), oracle.mx_quantize(bb, oracle.ROW)
    d = nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_F32)
    assert d.shape == (M, N) and rel_fro(d.cpu().numpy(), oracle.mx_gemm_f64(ra, rb)) <= GEMM_TOL
    d16 = nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_BF16)
    assert torch.equal(d16, d.to(torch.bfloat16))


def test_mx_and_nvfp4_operands_do_not_mix():
    xb = synth.normal(128, 128, 1.0, 920)
    a = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW, nv.BLOCK_MX32)
    b = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW)
    with pytest.raises(nv.NVFP4Error) as e:
        nv.nvfp4_gemm(a, b, nv.OP_DGRAD)
    assert e.value.status == -4
    c = nv.nvfp4_quantize(to_dev(synth.normal(64, 96, 1.0, 921)), nv.LAYOUT_ROW, nv.BLOCK_MX32)
    with pytest.raises(nv.NVFP4Error) as e:                      # K = 96 is not a multiple of 128
        nv.nvfp4_gemm(c, c, nv.OP_DGRAD)
    assert e.value.status == -2
