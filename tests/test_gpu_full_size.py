"""GPU parity at the full sizes of the BASELINE configs 2-5 (the shapes bench.py times).

Quantizer outputs are compared with the CPU oracle in full (bit-exact).  The big
GEMMs are compared on a seeded sample of output entries the oracle computes one
by one in binary64 (full rows, full columns and tiles), relative Frobenius error
over the sample <= 1e-5; properties that hold at any size (bf16 output equals the
rounded FP32 output, determinism) are checked on the whole matrix.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_25149_amd import binding as nv, synth

pytestmark = pytest.mark.gpu

GEMM_TOL = 1e-5
RHT_SEED, SR_SEED = 2025, 0x5EED5EED5EED


def to_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def assert_copy(codes, scales, ts, ref, what):
    torch.cuda.synchronize()
    t = ts.cpu().numpy()
    assert t[1].view(np.uint32) == ref.amax.view(np.uint32), f"{what}: amax"
    assert t[0].view(np.uint32) == ref.s_dec.view(np.uint32), f"{what}: s_dec"
    assert np.array_equal(scales.cpu().numpy(), ref.scales), f"{what}: scales differ"
    assert np.array_equal(codes.cpu().numpy(), ref.codes), f"{what}: codes differ"


def sample_entries(M, N, seed, rows=4, cols=4, tile=32):
    """Seeded sample: a few full rows, full columns and two tiles (one touching the last row/column)."""
    rng = np.random.default_rng(seed)
    m_list, n_list = [], []
    for r in rng.choice(M, rows, replace=False):
        m_list.append(np.full(N, r)); n_list.append(np.arange(N))
    for c in rng.choice(N, cols, replace=False):
        m_list.append(np.arange(M)); n_list.append(np.full(M, c))
    for (r0, c0) in ((M - tile, N - tile), (int(rng.integers(0, M - tile)), int(rng.integers(0, N - tile)))):
        mm, nn = np.meshgrid(np.arange(r0, r0 + tile), np.arange(c0, c0 + tile), indexing="ij")
        m_list.append(mm.ravel()); n_list.append(nn.ravel())
    return np.concatenate(m_list), np.concatenate(n_list)


def ws_for(m, n, k):
    return torch.empty(nv.gemm_workspace_bytes(m, n, k), dtype=torch.uint8, device="cuda")


def check_gemm_sample(d_gpu, a_ref, b_ref, seed):
    M, N = d_gpu.shape
    m, n = sample_entries(M, N, seed)
    want = oracle.gemm_f64_entries(a_ref, b_ref, m, n)
    got = d_gpu[torch.from_numpy(m).cuda(), torch.from_numpy(n).cuda()].double().cpu().numpy()
    err = np.linalg.norm(got - want) / np.linalg.norm(want)
    assert err <= GEMM_TOL, f"relative Frobenius error over {m.size} sampled entries: {err}"
    return err


@pytest.fixture(scope="module")
def weight():
    """W 5120x20480 of configs 3 and 4, quantized once with 16x16 blocks, both orientations."""
    wb = synth.normal(5120, 20480, 0.02, 302)
    qw = nv.nvfp4_quantize(to_dev(wb), nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16)
    ref_col = oracle.quantize(wb, oracle.COL, oracle.BLOCK_16x16)
    ref_row = oracle.quantize(wb, oracle.ROW, oracle.BLOCK_16x16)
    assert_copy(qw.col_codes, qw.col_scales, qw.col_ts, ref_col, "W col copy")
    assert_copy(qw.row_codes, qw.row_scales, qw.row_ts, ref_row, "W row copy")
    return qw, ref_row, ref_col


def test_config2_wgrad_rht_sr():
    t = synth.config_tensors(2)
    qdy = nv.nvfp4_quantize(to_dev(t["dY"]), nv.LAYOUT_COL, rounding=nv.ROUND_SR, rht_on_col=True,
                            rht_seed=RHT_SEED, sr_seed=SR_SEED)
    qx = nv.nvfp4_quantize(to_dev(t["X"]), nv.LAYOUT_COL, rht_on_col=True, rht_seed=RHT_SEED)
    rdy = oracle.quantize(t["dY"], oracle.COL, rounding=oracle.SR, use_rht=True, rht_seed=RHT_SEED, sr_seed=SR_SEED)
    rx = oracle.quantize(t["X"], oracle.COL, use_rht=True, rht_seed=RHT_SEED)
    assert_copy(qdy.col_codes, qdy.col_scales, qdy.col_ts, rdy, "dY col copy (RHT, SR)")
    assert_copy(qx.col_codes, qx.col_scales, qx.col_ts, rx, "X col copy (RHT, RNE)")
    ws = ws_for(5120, 5120, 4096)
    dw = nv.nvfp4_gemm(qdy, qx, nv.OP_WGRAD, nv.OUT_F32, workspace=ws)     # the route bench.py times
    assert dw.shape == (5120, 5120)
    check_gemm_sample(dw, rdy, rx, 22)
    again = nv.nvfp4_gemm(qdy, qx, nv.OP_WGRAD, nv.OUT_F32, workspace=ws)
    assert torch.equal(dw, again)
    fused = nv.nvfp4_gemm(qdy, qx, nv.OP_WGRAD, nv.OUT_F32)                 # the fused route, no workspace
    check_gemm_sample(fused, rdy, rx, 23)
    # gradient accumulation over micro-batches (Sec. 4.1): the same micro-batch added twice into an FP32 buffer
    acc = torch.zeros_like(dw)
    nv.nvfp4_gemm(qdy, qx, nv.OP_WGRAD, nv.OUT_F32_ACCUMULATE, out=acc, workspace=ws)
    assert torch.equal(acc, dw)
    nv.nvfp4_gemm(qdy, qx, nv.OP_WGRAD, nv.OUT_F32_ACCUMULATE, out=acc, workspace=ws)
    assert torch.equal(acc, dw + dw)


def test_config3_fprop(weight):
    qw, _, ref_col = weight
    xb = synth.normal_with_outliers(8192, 5120, 1.0, 301)
    qx = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW)
    rx = oracle.quantize(xb, oracle.ROW)
    assert_copy(qx.row_codes, qx.row_scales, qx.row_ts, rx, "X row copy")
    ws = ws_for(8192, 20480, 5120)
    y = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_F32, workspace=ws)
    assert y.shape == (8192, 20480)
    check_gemm_sample(y, rx, ref_col, 33)
    y16 = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_BF16, workspace=ws)
    assert torch.equal(y16, y.to(torch.bfloat16))          # bf16 output = RNE of the FP32 output
    del y16
    fused = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_F32)
    check_gemm_sample(fused, rx, ref_col, 34)


def test_config4_dgrad(weight):
    qw, ref_row, _ = weight
    dyb = synth.student_t3(8192, 20480, 1e-3, 401)
    qdy = nv.nvfp4_quantize(to_dev(dyb), nv.LAYOUT_ROW, rounding=nv.ROUND_SR, sr_seed=SR_SEED)
    rdy = oracle.quantize(dyb, oracle.ROW, rounding=oracle.SR, sr_seed=SR_SEED)
    assert_copy(qdy.row_codes, qdy.row_scales, qdy.row_ts, rdy, "dY row copy (SR)")
    dx = nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_F32, workspace=ws_for(8192, 5120, 20480))
    assert dx.shape == (8192, 5120)                            # same quantized W, transposed, no requantization
    check_gemm_sample(dx, rdy, ref_row, 44)
    fused = nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_F32)
    check_gemm_sample(fused, rdy, ref_row, 45)
    # 640 tiles of 256x256: the last 128 run split in two along K; every entry must agree with the fused route
    assert float((dx - fused).double().norm() / fused.double().norm()) <= 2e-6


@pytest.mark.parametrize("name,mode", [
    ("T1", dict(rounding=nv.ROUND_RNE, rht_on_col=True)),                    # activation: row RNE + col RHT RNE
    ("T2", dict(rounding=nv.ROUND_SR, rht_on_col=True)),                     # gradient: row SR + col RHT SR
    ("T3", dict(block_dim=nv.BLOCK_16x16)),                                  # weight: 16x16, both orientations
])
def test_config5_quantize_sweep(name, mode):
    shapes = {"T1": (8192, 5120, 501), "T2": (8192, 20480, 502), "T3": (5120, 20480, 503)}
    rows, cols, seed = shapes[name]
    xb = synth.student_t3(rows, cols, 0.02, seed)
    q = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW | nv.LAYOUT_COL, rht_seed=RHT_SEED, sr_seed=SR_SEED, **mode)
    ob = oracle.BLOCK_16x16 if mode.get("block_dim") == nv.BLOCK_16x16 else oracle.BLOCK_1x16
    orr = oracle.SR if mode.get("rounding") == nv.ROUND_SR else oracle.RNE
    rht = bool(mode.get("rht_on_col"))
    row = oracle.quantize(xb, oracle.ROW, ob, orr, False, 0, SR_SEED)
    assert_copy(q.row_codes, q.row_scales, q.row_ts, row, f"{name} row copy")
    del row
    col = oracle.quantize(xb, oracle.COL, ob, orr, rht, RHT_SEED, SR_SEED)
    assert_copy(q.col_codes, q.col_scales, q.col_ts, col, f"{name} col copy")


@pytest.mark.parametrize("name,d,rounding", [("activation", 4, nv.ROUND_RNE), ("activation", 32, nv.ROUND_RNE),
                                             ("gradient", 128, nv.ROUND_SR)])
def test_other_rotation_sizes_at_full_size(name, d, rounding):
    """The Wgrad copies of the 12B shapes with the rotation sizes ablated in Sec. 4.2 / App. E.4."""
    rows, cols, seed = {"activation": (8192, 5120, 511), "gradient": (8192, 20480, 512)}[name]
    xb = synth.student_t3(rows, cols, 0.02, seed)
    q = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW | nv.LAYOUT_COL, rounding=rounding, rht_on_col=d, rht_seed=RHT_SEED,
                          sr_seed=SR_SEED)
    orr = oracle.SR if rounding == nv.ROUND_SR else oracle.RNE
    row = oracle.quantize(xb, oracle.ROW, oracle.BLOCK_1x16, orr, False, 0, SR_SEED)
    assert_copy(q.row_codes, q.row_scales, q.row_ts, row, f"{name} d={d} row copy")
    del row
    col = oracle.quantize(xb, oracle.COL, oracle.BLOCK_1x16, orr, True, RHT_SEED, SR_SEED, rht_dim=d)
    assert_copy(q.col_codes, q.col_scales, q.col_ts, col, f"{name} d={d} col copy")


@pytest.mark.parametrize("name,rounding", [("activation", nv.ROUND_RNE), ("gradient", nv.ROUND_SR)])
def test_rotated_row_copy_at_full_size(name, rounding):
    """Both copies of the 12B shapes with the row copy rotated too (the Fprop / Dgrad operands of App. E.4.1)."""
    rows, cols, seed = {"activation": (8192, 5120, 521), "gradient": (8192, 20480, 522)}[name]
    xb = synth.student_t3(rows, cols, 0.02, seed)
    q = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW | nv.LAYOUT_COL | nv.LAYOUT_ROW_RHT, rounding=rounding, rht_on_col=16,
                          rht_seed=RHT_SEED, sr_seed=SR_SEED)
    orr = oracle.SR if rounding == nv.ROUND_SR else oracle.RNE
    row = oracle.quantize(xb, oracle.ROW, oracle.BLOCK_1x16, orr, True, RHT_SEED, SR_SEED)
    assert_copy(q.row_codes, q.row_scales, q.row_ts, row, f"{name} rotated row copy")
    del row
    col = oracle.quantize(xb, oracle.COL, oracle.BLOCK_1x16, orr, True, RHT_SEED, SR_SEED)
    assert_copy(q.col_codes, q.col_scales, q.col_ts, col, f"{name} col copy")


def test_contraction_too_long_for_the_two_pass_kernel():
    """K = 2^21: the FP16 GEMM kernel's 32-bit byte offsets inside a block of rows stop there, so the call must take
    the fused route even when a workspace is lent; results as usual."""
    M, N, K = 32, 48, 1 << 21
    ab = synth.normal_with_outliers(M, K, 1.0, 901, frac=0.001)
    bb = synth.normal(N, K, 0.02, 902)
    qa = nv.nvfp4_quantize(to_dev(ab), nv.LAYOUT_ROW)
    qb = nv.nvfp4_quantize(to_dev(bb), nv.LAYOUT_ROW)
    ra, rb = oracle.quantize(ab, oracle.ROW), oracle.quantize(bb, oracle.ROW)
    assert_copy(qa.row_codes, qa.row_scales, qa.row_ts, ra, "A")
    want = oracle.gemm_f64(ra, rb)
    for ws in (None, ws_for(M, N, K)):
        got = nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_F32, workspace=ws)
        torch.cuda.synchronize()
        err = np.linalg.norm(got.cpu().numpy().astype(np.float64) - want) / np.linalg.norm(want)
        assert err <= GEMM_TOL, err


def test_indexing_beyond_2_31_elements():
    """A tensor of 2^31 + 2^27 elements (4.5 GB of bf16): the small tensor it is tiled from fixes the expected
    bytes, since tiling by whole 16-row groups changes neither the amax nor any block (RNE)."""
    base_rows, cols, reps = 128, 16384, 1088          # 128*1088 = 139264 rows; 139264*16384 = 2^31 + 2^27
    xb = synth.normal_with_outliers(base_rows, cols, 1.0, 777, frac=0.01)
    small = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW | nv.LAYOUT_COL, rht_on_col=True, rht_seed=RHT_SEED)
    big_x = to_dev(xb).repeat(reps, 1)
    assert big_x.numel() > 2 ** 31
    big = nv.nvfp4_quantize(big_x, nv.LAYOUT_ROW | nv.LAYOUT_COL, rht_on_col=True, rht_seed=RHT_SEED)
    torch.cuda.synchronize()
    del big_x
    assert torch.equal(big.row_ts, small.row_ts) and torch.equal(big.col_ts, small.col_ts)
    assert torch.equal(big.row_codes.view(reps, base_rows, cols // 2), small.row_codes.expand(reps, -1, -1))
    assert torch.equal(big.row_scales.view(reps, base_rows, cols // 16), small.row_scales.expand(reps, -1, -1))
    assert torch.equal(big.col_codes.view(cols, reps, base_rows // 2), small.col_codes.unsqueeze(1).expand(-1, reps, -1))
    assert torch.equal(big.col_scales.view(cols, reps, base_rows // 16), small.col_scales.unsqueeze(1).expand(-1, reps, -1))
    # decode goes through the same 64-bit offsets
    d_small = nv.nvfp4_dequantize(small, nv.COPY_ROW, False, nv.OUT_BF16)
    d_big = nv.nvfp4_dequantize(big, nv.COPY_ROW, False, nv.OUT_BF16)
    assert torch.equal(d_big.view(reps, base_rows, cols), d_small.expand(reps, -1, -1))
    del d_big
    # GEMM with M = 139264 rows of A (2^31 + 2^27 elements): every block of 128 output rows repeats
    wq = nv.nvfp4_quantize(to_dev(synth.normal(cols, 256, 0.02, 778)), nv.LAYOUT_COL, nv.BLOCK_16x16)
    y_small = nv.nvfp4_gemm(small, wq, nv.OP_FPROP, nv.OUT_F32)
    ws = ws_for(base_rows * reps, 256, cols)
    y_big = nv.nvfp4_gemm(big, wq, nv.OP_FPROP, nv.OUT_F32, workspace=ws)
    torch.cuda.synchronize()
    err = (y_big.view(reps, base_rows, 256) - y_small).double().norm() / (y_small.double().norm() * reps ** 0.5)
    assert float(err) <= 2e-6      # same products, FP32 summation order may differ between tile positions
    y_big_fused = nv.nvfp4_gemm(big, wq, nv.OP_FPROP, nv.OUT_F32)
    err = (y_big_fused.view(reps, base_rows, 256) - y_small).double().norm() / (y_small.double().norm() * reps ** 0.5)
    assert float(err) <= 2e-6


@pytest.mark.parametrize("M,N,K,splits", [(4352, 4096, 4096, 8), (4208, 4304, 2048, 4), (8192, 5120, 1024, 2)])
def test_split_k_last_round(M, N, K, splits):
    """Shapes whose last round of 256x256 tiles is partial (272, 289 and 640 tiles), ragged edges included: the
    split-K launch and the launch that adds its partial tiles against the oracle on a sample, against the fused route
    everywhere, and bit-for-bit against itself (the partial sums are added in a fixed order)."""
    tiles = -(-M // 256) * -(-N // 256)                                        # partial tiles are in the workspace
    assert nv.gemm_workspace_bytes(M, N, K) == (((M + N) * K * 2 + 255) // 256) * 256 + (tiles % 256) * splits * 2 ** 18
    ab = synth.normal_with_outliers(M, K, 1.0, 901)
    bb = synth.normal(N, K, 0.05, 902)
    qa = nv.nvfp4_quantize(to_dev(ab), nv.LAYOUT_ROW)
    qb = nv.nvfp4_quantize(to_dev(bb), nv.LAYOUT_ROW)
    ra, rb = oracle.quantize(ab, oracle.ROW), oracle.quantize(bb, oracle.ROW)
    ws = ws_for(M, N, K)
    ws.fill_(0xA5)                                                              # the call must not rely on its contents
    d = nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_F32, workspace=ws)
    check_gemm_sample(d, ra, rb, 91)
    fused = nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_F32)
    assert float((d - fused).double().norm() / fused.double().norm()) <= 2e-6
    for _ in range(3):
        again = nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_F32, workspace=ws)
        assert torch.equal(again, d)
    d16 = nv.nvfp4_gemm(qa, qb, nv.OP_DGRAD, nv.OUT_BF16, workspace=ws)
    assert torch.equal(d16, d.to(torch.bfloat16))
