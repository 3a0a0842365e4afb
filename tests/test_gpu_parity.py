"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle.

Bar: codes, block scales, tensor scale and amax bit-exact (also under stochastic
rounding with the same Philox counters and under the rotation with the fixed
butterfly order); dequantize bit-exact; GEMM relative Frobenius error <= 1e-5
against the binary64 reference on the dequantized operands.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2509_25149_amd import binding as nv, synth

pytestmark = pytest.mark.gpu

GEMM_TOL = 1e-5


def to_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def assert_copy_equal(codes, scales, ts, ref: oracle.QCopy, what: str):
    torch.cuda.synchronize()
    c, s, t = codes.cpu().numpy(), scales.cpu().numpy(), ts.cpu().numpy()
    assert t[1].view(np.uint32) == ref.amax.view(np.uint32), f"{what}: amax {t[1]} vs {ref.amax}"
    assert t[0].view(np.uint32) == ref.s_dec.view(np.uint32), f"{what}: s_dec {t[0]} vs {ref.s_dec}"
    bad_s = np.argwhere(s != ref.scales)
    assert bad_s.size == 0, f"{what}: {len(bad_s)} scale bytes differ, first at {bad_s[0]}"
    bad_c = np.argwhere(c != ref.codes)
    assert bad_c.size == 0, f"{what}: {len(bad_c)} code bytes differ, first at {bad_c[0]}"


def check_quantize(xb, layout, block_dim=nv.BLOCK_1x16, rounding=nv.ROUND_RNE, rht=False, rht_seed=0, sr_seed=0,
                   x_dev=None):
    x = to_dev(xb) if x_dev is None else x_dev
    q = nv.nvfp4_quantize(x, layout, block_dim, rounding, rht, rht_seed, sr_seed)
    ob = oracle.BLOCK_16x16 if block_dim == nv.BLOCK_16x16 else oracle.BLOCK_1x16
    orr = oracle.SR if rounding == nv.ROUND_SR else oracle.RNE
    refs = {}
    if layout & nv.LAYOUT_ROW:
        refs["row"] = oracle.quantize(xb, oracle.ROW, ob, orr, False, 0, sr_seed)
        assert_copy_equal(q.row_codes, q.row_scales, q.row_ts, refs["row"], "row copy")
    if layout & nv.LAYOUT_COL:
        refs["col"] = oracle.quantize(xb, oracle.COL, ob, orr, rht, rht_seed, sr_seed)
        assert_copy_equal(q.col_codes, q.col_scales, q.col_ts, refs["col"], "col copy")
    return q, refs


def test_conversion_instructions_selftest():
    assert nv.nvfp4_selftest_conversions() == [0, 0, 0, 0, 0]


@pytest.mark.parametrize("name", ["handworked_A.txt", "handworked_B.txt"])
def test_handworked_tensors(golden_dir, name):
    g = {}
    for line in open(os.path.join(golden_dir, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split(":")
            g[k.strip()] = v.split()
    x = np.array([float(t) for t in g["x"]], dtype=np.float32)
    xb = np.tile(synth.f32_to_bf16_bits(x).reshape(1, -1), (16, 1))
    q, _ = check_quantize(xb, nv.LAYOUT_ROW)
    codes = q.row_codes.cpu().numpy()[0]
    c4 = np.stack([codes & 15, codes >> 4], -1).ravel()
    assert [int(v) for v in c4] == [int(t, 16) for t in g["codes"]]
    assert [int(v) for v in q.row_scales.cpu().numpy()[0]] == [int(t, 16) for t in g["scales"]]
    assert q.row_ts.cpu().numpy()[0].view(np.uint32) == int(g["s_dec_bits"][0], 16)


SHAPES = [(16, 16), (16, 1040), (80, 528), (144, 2064)]   # several 512-column tiles plus ragged tails
MODES = [
    dict(layout=nv.LAYOUT_ROW),
    dict(layout=nv.LAYOUT_COL),
    dict(layout=nv.LAYOUT_ROW | nv.LAYOUT_COL),
    dict(layout=nv.LAYOUT_COL, rht=True, rht_seed=2025),
    dict(layout=nv.LAYOUT_ROW | nv.LAYOUT_COL, rht=True, rht_seed=7),
    dict(layout=nv.LAYOUT_ROW, rounding=nv.ROUND_SR, sr_seed=0xC0FFEE1234),
    dict(layout=nv.LAYOUT_COL, rounding=nv.ROUND_SR, sr_seed=99),
    dict(layout=nv.LAYOUT_ROW | nv.LAYOUT_COL, rounding=nv.ROUND_SR, rht=True, rht_seed=11, sr_seed=2 ** 63 + 17),
    dict(layout=nv.LAYOUT_ROW | nv.LAYOUT_COL, block_dim=nv.BLOCK_16x16),
    dict(layout=nv.LAYOUT_COL, block_dim=nv.BLOCK_16x16),
    dict(layout=nv.LAYOUT_ROW | nv.LAYOUT_COL, block_dim=nv.BLOCK_16x16, rounding=nv.ROUND_SR, sr_seed=3),
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("mode", MODES, ids=lambda m: "-".join(f"{k}{v}" for k, v in m.items()))
def test_quantize_modes(shape, mode):
    rows, cols = shape
    gen = [synth.normal_with_outliers(rows, cols, 1.0, 1000 + rows + cols, frac=0.01),
           synth.student_t3(rows, cols, 1e-3, 2000 + rows + cols)]
    for xb in gen:
        check_quantize(xb, **mode)


def test_quantize_with_leading_dimension():
    xb = synth.normal(48, 96, 1.0, 77)
    big = torch.zeros((48, 128), dtype=torch.bfloat16, device="cuda")
    big[:, :96] = to_dev(xb)
    check_quantize(xb, nv.LAYOUT_ROW | nv.LAYOUT_COL, rht=True, rht_seed=5, x_dev=big[:, :96])


def test_quantize_degenerate_inputs():
    z = np.zeros((32, 64), dtype=np.float32)
    check_quantize(synth.f32_to_bf16_bits(z), nv.LAYOUT_ROW | nv.LAYOUT_COL)
    z[3, 7] = -0.0
    z[0, 16] = 1.0
    z[1, 0] = -1e-6
    z[1, 1] = 1e-7
    z[20, 40] = -3.0
    for kw in (dict(), dict(rht=True, rht_seed=1), dict(block_dim=nv.BLOCK_16x16), dict(rounding=nv.ROUND_SR, sr_seed=4)):
        check_quantize(synth.f32_to_bf16_bits(z), nv.LAYOUT_ROW | nv.LAYOUT_COL, **kw)
    # subnormal-range tensors: 2688/amax overflows and is clamped; s_dec is subnormal
    t = np.zeros((16, 32), dtype=np.float32)
    t[0, 0] = 1e-38
    t[5, 20] = -3e-39
    t[9, 9] = 1e-40
    check_quantize(synth.f32_to_bf16_bits(t), nv.LAYOUT_ROW | nv.LAYOUT_COL)
    # huge values
    h = synth.bf16_bits_to_f32(synth.normal(32, 32, 1.0, 5)) * np.float32(1e37)
    check_quantize(synth.f32_to_bf16_bits(h), nv.LAYOUT_ROW | nv.LAYOUT_COL, rht=True, rht_seed=3)


def test_nonfinite_input_is_flagged_in_amax():
    x = synth.bf16_bits_to_f32(synth.normal(16, 32, 1.0, 6))
    x[3, 3] = np.inf
    q = nv.nvfp4_quantize(to_dev(synth.f32_to_bf16_bits(x)), nv.LAYOUT_ROW)
    torch.cuda.synchronize()
    assert not np.isfinite(q.row_ts.cpu().numpy()[1])


@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
def test_nonfinite_input_is_flagged_in_every_copy(bad):
    # the maxima of rotated values skip NaNs, so the raw maximum is what carries a NaN into a rotated copy's amax
    x = synth.bf16_bits_to_f32(synth.normal(256, 48, 1.0, 6))
    x[131, 17] = bad
    xd = to_dev(synth.f32_to_bf16_bits(x))
    for d in (2, 4, 16, 32, 128):
        q = nv.nvfp4_quantize(xd, nv.LAYOUT_COL, rht_on_col=d, rht_seed=3)            # a rotated copy alone
        assert not np.isfinite(q.col_ts.cpu().numpy()[1]), d
        q = nv.nvfp4_quantize(xd, nv.LAYOUT_ROW | nv.LAYOUT_COL, rht_on_col=d, rht_seed=3)
        assert not np.isfinite(q.col_ts.cpu().numpy()[1]) and not np.isfinite(q.row_ts.cpu().numpy()[1]), d
    for col in (0, 16):
        q = nv.nvfp4_quantize(xd, nv.LAYOUT_ROW | nv.LAYOUT_COL | nv.LAYOUT_ROW_RHT, rht_on_col=col, rht_seed=3)
        assert not np.isfinite(q.col_ts.cpu().numpy()[1]) and not np.isfinite(q.row_ts.cpu().numpy()[1]), col
    q = nv.nvfp4_quantize(xd, nv.LAYOUT_ROW | nv.LAYOUT_ROW_RHT, rht_seed=3)
    assert not np.isfinite(q.row_ts.cpu().numpy()[1])
    q = nv.nvfp4_quantize(xd, nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16)
    assert not np.isfinite(q.col_ts.cpu().numpy()[1]) and not np.isfinite(q.row_ts.cpu().numpy()[1])
    amax = nv.nvfp4_amax(xd, 16, 3).cpu().numpy()
    assert not np.isfinite(amax[0]) and not np.isfinite(amax[1])
    # and a finite tensor is not flagged
    q = nv.nvfp4_quantize(to_dev(synth.normal(256, 48, 1.0, 6)), nv.LAYOUT_COL, rht_on_col=16, rht_seed=3)
    assert np.isfinite(q.col_ts.cpu().numpy()[1])


def test_two_d_weight_copies_are_transposes():
    wb = synth.normal(96, 160, 0.02, 8)
    q, _ = check_quantize(wb, nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16)
    r, c = q.row_codes.cpu().numpy(), q.col_codes.cpu().numpy()
    un = lambda b: np.stack([b & 15, b >> 4], -1).reshape(b.shape[0], -1)
    assert np.array_equal(un(r), un(c).T)


def test_quantize_is_deterministic():
    xb = synth.student_t3(64, 1024, 1e-3, 9)
    x = to_dev(xb)
    a = nv.nvfp4_quantize(x, 3, rounding=nv.ROUND_SR, rht_on_col=True, rht_seed=1, sr_seed=2)
    b = nv.nvfp4_quantize(x, 3, rounding=nv.ROUND_SR, rht_on_col=True, rht_seed=1, sr_seed=2)
    torch.cuda.synchronize()
    assert torch.equal(a.row_codes, b.row_codes) and torch.equal(a.col_codes, b.col_codes)
    assert torch.equal(a.col_scales, b.col_scales)


# ---------------------------------------------------------------- dequantize

def test_dequantize_matches_oracle_bitwise():
    xb = synth.normal_with_outliers(48, 160, 1.0, 21, frac=0.01)
    q, refs = check_quantize(xb, nv.LAYOUT_ROW | nv.LAYOUT_COL, rht=True, rht_seed=31)
    for copy, key, undo in ((nv.COPY_ROW, "row", False), (nv.COPY_COL, "col", False), (nv.COPY_COL, "col", True)):
        got = nv.nvfp4_dequantize(q, copy, undo).cpu().numpy()
        want = oracle.dequantize(refs[key], undo, 31)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (key, undo)
        got16 = nv.nvfp4_dequantize(q, copy, undo, nv.OUT_BF16).view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got16, synth.f32_to_bf16_bits(want))
    back = nv.nvfp4_dequantize(q, nv.COPY_COL, True).cpu().numpy().T
    x = synth.bf16_bits_to_f32(xb)
    assert np.linalg.norm(back - x) < 0.15 * np.linalg.norm(x)


# ---------------------------------------------------------------- GEMM

def rel_fro(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref) / np.linalg.norm(ref))


def gemm_ws(m, n, k):
    """Workspace that lets nvfp4_gemm take its decode-pass + FP16-GEMM route."""
    return torch.empty(nv.gemm_workspace_bytes(m, n, k), dtype=torch.uint8, device="cuda")


def gemm_both_routes(a, b, op, ref):
    """Run the fused route (no workspace) and the two-pass route; both must meet the tolerance."""
    fused = nv.nvfp4_gemm(a, b, op, nv.OUT_F32)
    m, n = fused.shape
    k = a.rows if op == nv.OP_WGRAD else a.cols
    two = nv.nvfp4_gemm(a, b, op, nv.OUT_F32, workspace=gemm_ws(m, n, k))
    assert rel_fro(fused.cpu().numpy(), ref) <= GEMM_TOL
    assert rel_fro(two.cpu().numpy(), ref) <= GEMM_TOL
    two16 = nv.nvfp4_gemm(a, b, op, nv.OUT_BF16, workspace=gemm_ws(m, n, k))
    assert torch.equal(two16, two.to(torch.bfloat16))
    # FP32 accumulate-into (Sec. 4.1): D <- D + result, against the oracle's binary64 sum, and exactly one
    # FP32 addition on top of the plain result
    g = torch.Generator(device="cuda").manual_seed(1000 + m + n)
    d_prev = torch.randn((m, n), generator=g, device="cuda") * float(np.abs(ref).mean())
    want = d_prev.cpu().numpy().astype(np.float64) + ref
    for ws, plain in ((None, fused), (gemm_ws(m, n, k), two)):
        d = d_prev.clone()
        nv.nvfp4_gemm(a, b, op, nv.OUT_F32_ACCUMULATE, out=d, workspace=ws)
        assert rel_fro(d.cpu().numpy(), want) <= GEMM_TOL
        assert torch.equal(d, d_prev + plain)
    return fused


def test_config1_fprop_full():
    t = synth.config_tensors(1)
    qx, rx = check_quantize(t["X"], nv.LAYOUT_ROW)
    qw, rw = check_quantize(t["W"], nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16)
    ref = oracle.gemm_f64(rx["row"], rw["col"])
    y = gemm_both_routes(qx, qw, nv.OP_FPROP, ref)
    assert y.shape == (256, 256)
    y16 = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_BF16)
    assert np.array_equal(y16.view(torch.int16).cpu().numpy().view(np.uint16), synth.f32_to_bf16_bits(y.cpu().numpy()))
    # Dgrad reuses the same quantized weight, transposed, without requantizing (Sec. 4.3)
    dyb = synth.student_t3(256, 256, 1e-3, 103)
    qd, rd = check_quantize(dyb, nv.LAYOUT_ROW, rounding=nv.ROUND_SR, sr_seed=1)
    dx = gemm_both_routes(qd, qw, nv.OP_DGRAD, oracle.gemm_f64(rd["row"], rw["row"]))
    assert dx.shape == (256, 512)


@pytest.mark.parametrize("mnk", [(16, 16, 16), (80, 48, 80), (272, 144, 176), (128, 384, 1040), (80, 48, 64), (272, 528, 192)])
def test_gemm_ragged_shapes_all_ops(mnk):
    M, N, K = mnk
    xb = synth.normal_with_outliers(M, K, 1.0, 300 + M, frac=0.01)
    wb = synth.normal(K, N, 0.02, 400 + N)
    qx, rx = check_quantize(xb, nv.LAYOUT_ROW | nv.LAYOUT_COL, rht=True, rht_seed=12)
    qw, rw = check_quantize(wb, nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16)
    gemm_both_routes(qx, qw, nv.OP_FPROP, oracle.gemm_f64(rx["row"], rw["col"]))
    dyb = synth.student_t3(M, N, 1e-3, 500 + M)
    qd, rd = check_quantize(dyb, nv.LAYOUT_ROW | nv.LAYOUT_COL, rounding=nv.ROUND_SR, rht=True, rht_seed=12, sr_seed=8)
    dx = gemm_both_routes(qd, qw, nv.OP_DGRAD, oracle.gemm_f64(rd["row"], rw["row"]))
    assert dx.shape == (M, K)
    ref = oracle.gemm_f64(rd["col"], rx["col"])
    dw = gemm_both_routes(qd, qx, nv.OP_WGRAD, ref)                # dY^T X : [N, K]
    assert dw.shape == (N, K)
    # the rotation cancels: the result approximates the unquantized product
    exact = synth.bf16_bits_to_f32(dyb).astype(np.float64).T @ synth.bf16_bits_to_f32(xb).astype(np.float64)
    if M >= 80:
        assert np.linalg.norm(ref - exact) <= 0.3 * np.linalg.norm(exact)


@pytest.mark.parametrize("K", [64, 128, 192])
def test_gemm_with_more_tiles_than_compute_units(K):
    """17 x 18 tiles of 256 x 256, the last row and column of them ragged: with a workspace the FP16 kernel is launched
    with one workgroup per CU, 50 of which run two tiles as one stream of K steps (K = 128: the shortest tile that
    allows it; K = 192: an odd number of steps, so the LDS stage parity differs from tile to tile; K = 64: one step,
    launched with a workgroup per tile instead)."""
    M, N = 4112, 4368
    xb = synth.normal_with_outliers(M, K, 1.0, 900 + K, frac=0.01)
    wb = synth.normal(K, N, 0.02, 901 + K)
    qx, rx = check_quantize(xb, nv.LAYOUT_ROW)
    qw, rw = check_quantize(wb, nv.LAYOUT_COL, nv.BLOCK_16x16)
    y = gemm_both_routes(qx, qw, nv.OP_FPROP, oracle.gemm_f64(rx["row"], rw["col"]))
    assert y.shape == (M, N)


def test_gemm_output_with_leading_dimension():
    xb, wb = synth.normal(32, 64, 1.0, 61), synth.normal(64, 48, 0.02, 62)
    qx, rx = check_quantize(xb, nv.LAYOUT_ROW)
    qw, rw = check_quantize(wb, nv.LAYOUT_COL, nv.BLOCK_16x16)
    buf = torch.full((32, 64), 7.0, dtype=torch.float32, device="cuda")
    nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, out=buf[:, :48])
    got = buf.cpu().numpy()
    assert np.all(got[:, 48:] == 7.0)
    assert rel_fro(got[:, :48], oracle.gemm_f64(rx["row"], rw["col"])) <= GEMM_TOL


def test_linear_layer_calls_equal_the_call_sequence():
    """nvfp4_linear_forward / nvfp4_linear_backward (Sec. 4.1 flow) against the oracle and, bit for bit, against
    the same steps issued one by one; two micro-batches accumulate into one FP32 dW."""
    tokens, d_in, d_out = 384, 512, 640
    rht_seed, sr_seed = 77, 4242
    wb = synth.normal(d_in, d_out, 0.02, 801)
    qw = nv.nvfp4_quantize(to_dev(wb), nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16)
    rw_col = oracle.quantize(wb, oracle.COL, oracle.BLOCK_16x16)
    rw_row = oracle.quantize(wb, oracle.ROW, oracle.BLOCK_16x16)
    ws = torch.empty(nv.linear_workspace_bytes(tokens, d_in, d_out), dtype=torch.uint8, device="cuda")
    dw = torch.zeros((d_in, d_out), dtype=torch.float32, device="cuda")
    dw_ref = np.zeros((d_in, d_out), dtype=np.float64)
    for mb in range(2):
        xb = synth.normal_with_outliers(tokens, d_in, 1.0, 810 + mb)
        dyb = synth.student_t3(tokens, d_out, 1e-3, 820 + mb)
        y, qx = nv.nvfp4_linear_forward(to_dev(xb), qw, ws, True, rht_seed, nv.OUT_F32)
        rx_row = oracle.quantize(xb, oracle.ROW)
        rx_col = oracle.quantize(xb, oracle.COL, use_rht=True, rht_seed=rht_seed)
        assert_copy_equal(qx.row_codes, qx.row_scales, qx.row_ts, rx_row, "X row")
        assert_copy_equal(qx.col_codes, qx.col_scales, qx.col_ts, rx_col, "X col (RHT)")
        assert rel_fro(y.cpu().numpy(), oracle.gemm_f64(rx_row, rw_col)) <= GEMM_TOL
        dw_before = dw.clone()
        dx, qdy = nv.nvfp4_linear_backward(to_dev(dyb), qx, qw, dw, ws, True, sr_seed + mb, nv.OUT_F32)
        rdy_row = oracle.quantize(dyb, oracle.ROW, rounding=oracle.SR, sr_seed=sr_seed + mb)
        rdy_col = oracle.quantize(dyb, oracle.COL, rounding=oracle.SR, use_rht=True, rht_seed=rht_seed, sr_seed=sr_seed + mb)
        assert_copy_equal(qdy.row_codes, qdy.row_scales, qdy.row_ts, rdy_row, "dY row (SR)")
        assert_copy_equal(qdy.col_codes, qdy.col_scales, qdy.col_ts, rdy_col, "dY col (RHT, SR)")
        assert rel_fro(dx.cpu().numpy(), oracle.gemm_f64(rdy_row, rw_row)) <= GEMM_TOL
        dw_ref = oracle.gemm_f64(rx_col, rdy_col, d_prev=dw_before.cpu().numpy())
        assert rel_fro(dw.cpu().numpy(), dw_ref) <= GEMM_TOL
        # the same steps one by one give the same bits
        qx2 = nv.nvfp4_quantize(to_dev(xb), nv.LAYOUT_ROW | nv.LAYOUT_COL, rht_on_col=True, rht_seed=rht_seed)
        y2 = nv.nvfp4_gemm(qx2, qw, nv.OP_FPROP, nv.OUT_F32, workspace=ws)
        qdy2 = nv.nvfp4_quantize(to_dev(dyb), nv.LAYOUT_ROW | nv.LAYOUT_COL, rounding=nv.ROUND_SR, rht_on_col=True,
                                 rht_seed=rht_seed, sr_seed=sr_seed + mb)
        dx2 = nv.nvfp4_gemm(qdy2, qw, nv.OP_DGRAD, nv.OUT_F32, workspace=ws)
        dw2 = dw_before.clone()
        nv.nvfp4_gemm(qx2, qdy2, nv.OP_WGRAD, nv.OUT_F32_ACCUMULATE, out=dw2, workspace=ws)
        assert torch.equal(y, y2) and torch.equal(dx, dx2) and torch.equal(dw, dw2)
    # inference-style forward keeps no column copy, and backward refuses such a descriptor
    y3, qx3 = nv.nvfp4_linear_forward(to_dev(xb), qw, ws, False, 0, nv.OUT_BF16)
    assert qx3.col_codes is None and torch.equal(y3, y.to(torch.bfloat16))
    with pytest.raises(nv.NVFP4Error) as e:
        nv.nvfp4_linear_backward(to_dev(dyb), qx3, qw, dw, ws)
    assert e.value.status == -3


def test_layer_step_replays_from_a_hip_graph():
    """A whole layer step (quantize + three GEMMs through the per-layer entry points, caller-owned buffers only) is
    captured into a HIP graph and replayed with eager work in between; every replay must reproduce the eager
    result bit for bit.  Shapes with a split-K last round."""
    tokens, d_in, d_out = 4352, 1024, 4096          # Fprop: 17 x 16 = 272 tiles -> the last 16 are split along K
    wb = synth.normal(d_in, d_out, 0.02, 951)
    xb = synth.normal_with_outliers(tokens, d_in, 1.0, 952)
    dyb = synth.student_t3(tokens, d_out, 1e-3, 953)
    x, dy = to_dev(xb), to_dev(dyb)
    qw = nv.nvfp4_quantize(to_dev(wb), nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16)
    ws = torch.empty(nv.linear_workspace_bytes(tokens, d_in, d_out), dtype=torch.uint8, device="cuda")
    RC = nv.LAYOUT_ROW | nv.LAYOUT_COL
    qx, qdy = nv.alloc_qtensor(tokens, d_in, RC), nv.alloc_qtensor(tokens, d_out, RC)
    y = torch.empty((tokens, d_out), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty((tokens, d_in), dtype=torch.bfloat16, device="cuda")
    dw = torch.zeros((d_in, d_out), dtype=torch.float32, device="cuda")

    def step():
        nv.nvfp4_linear_forward(x, qw, ws, True, 7, nv.OUT_BF16, qx=qx, y=y)
        nv.nvfp4_linear_backward(dy, qx, qw, dw, ws, False, 99, nv.OUT_BF16, qdy=qdy, dx=dx)

    step()                                           # eager: also sets the kernels' launch attributes
    torch.cuda.synchronize()
    want = [t.clone() for t in (y, dx, dw, qx.col_codes, qdy.row_codes, qdy.col_scales)]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    for rep in range(3):
        for t in (y, dx, dw):
            t.fill_(float(rep + 1))                  # eager work between the replays; stale outputs must be overwritten
        ws.random_(0, 255)                           # and the scratch contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (y, dx, dw, qx.col_codes, qdy.row_codes, qdy.col_scales)
        for g, w_ in zip(got, want):
            assert torch.equal(g, w_), f"replay {rep} differs from the eager result"


# ---------------------------------------------------------------- the two passes as separate calls (App. B.1)

@pytest.mark.parametrize("mode", [
    dict(layout=nv.LAYOUT_ROW | nv.LAYOUT_COL, rht=16),
    dict(layout=nv.LAYOUT_ROW | nv.LAYOUT_COL, rht=128, rounding=nv.ROUND_SR, sr_seed=7),
    dict(layout=nv.LAYOUT_COL, rht=4),
    dict(layout=nv.LAYOUT_ROW | nv.LAYOUT_COL, rht=0, block_dim=nv.BLOCK_16x16),
    dict(layout=nv.LAYOUT_ROW, rht=0, rounding=nv.ROUND_SR, sr_seed=9),
], ids=lambda m: "-".join(f"{k}{v}" for k, v in m.items()))
def test_amax_then_quantize_with_amax_equals_quantize(mode):
    rows, cols = 384, 1040
    xb = synth.normal_with_outliers(rows, cols, 1.0, 4242, frac=0.01)
    x = to_dev(xb)
    kw = dict(block_dim=mode.get("block_dim", nv.BLOCK_1x16), rounding=mode.get("rounding", nv.ROUND_RNE),
              rht_on_col=mode["rht"], rht_seed=31, sr_seed=mode.get("sr_seed", 0))
    whole = nv.nvfp4_quantize(x, mode["layout"], **kw)
    amax = nv.nvfp4_amax(x, mode["rht"], 31)
    split = nv.nvfp4_quantize_with_amax(x, amax, mode["layout"], **kw)
    torch.cuda.synchronize()
    ob = oracle.BLOCK_16x16 if kw["block_dim"] == nv.BLOCK_16x16 else oracle.BLOCK_1x16
    orr = oracle.SR if kw["rounding"] == nv.ROUND_SR else oracle.RNE
    am = amax.cpu().numpy()
    raw = oracle.quantize(xb, oracle.ROW, ob, orr, False, 0, kw["sr_seed"])
    assert am[0].view(np.uint32) == raw.amax.view(np.uint32)
    if mode["rht"]:
        rot = oracle.quantize(xb, oracle.COL, ob, orr, True, 31, kw["sr_seed"], rht_dim=mode["rht"])
        assert am[1].view(np.uint32) == rot.amax.view(np.uint32)
    else:
        assert am[1] == 0.0
    assert split.desc.col_has_rht == whole.desc.col_has_rht and split.desc.layout_mask == whole.desc.layout_mask
    if mode["layout"] & nv.LAYOUT_ROW:
        assert torch.equal(split.row_codes, whole.row_codes) and torch.equal(split.row_scales, whole.row_scales)
        assert torch.equal(split.row_ts, whole.row_ts)
    if mode["layout"] & nv.LAYOUT_COL:
        assert torch.equal(split.col_codes, whole.col_codes) and torch.equal(split.col_scales, whole.col_scales)
        assert torch.equal(split.col_ts, whole.col_ts)


@pytest.mark.parametrize("factor", [4.0, 1.0 / 64.0])
def test_quantize_with_a_supplied_amax_matches_the_oracle(factor):
    """A larger amax (as after a max over shards) and a far too small one (block scales and codes saturate)."""
    rows, cols = 144, 528
    xb = synth.normal_with_outliers(rows, cols, 1.0, 4343, frac=0.01)
    x = to_dev(xb)
    own = nv.nvfp4_amax(x, 16, 5).cpu().numpy()
    given = torch.tensor(own * np.float32(factor), dtype=torch.float32, device="cuda")
    q = nv.nvfp4_quantize_with_amax(x, given, nv.LAYOUT_ROW | nv.LAYOUT_COL, rht_on_col=16, rht_seed=5)
    g = given.cpu().numpy()
    assert_copy_equal(q.row_codes, q.row_scales, q.row_ts, oracle.quantize(xb, oracle.ROW, amax=float(g[0])), "row copy")
    assert_copy_equal(q.col_codes, q.col_scales, q.col_ts,
                      oracle.quantize(xb, oracle.COL, use_rht=True, rht_seed=5, amax=float(g[1])), "col copy")


def test_predecoded_operands_give_the_same_bits():
    """nvfp4_predecode: a weight decoded to FP16 once serves Fprop and Dgrad of every micro-batch (Sec. 4.3, Sec. 4.1);
    the GEMM on the decoded copy runs the same kernel on the same FP16 values, so the results are identical.  Shapes
    with a split-K last round; a workspace sized only for the operands still to decode must be enough."""
    tokens, d_in, d_out = 4352, 1024, 4096
    wb = synth.normal(d_in, d_out, 0.02, 2101)
    qw = nv.nvfp4_quantize(to_dev(wb), nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16)
    qx = nv.nvfp4_quantize(to_dev(synth.normal_with_outliers(tokens, d_in, 1.0, 2102)), nv.LAYOUT_ROW | nv.LAYOUT_COL,
                           rht_on_col=True, rht_seed=3)
    qdy = nv.nvfp4_quantize(to_dev(synth.student_t3(tokens, d_out, 1e-3, 2103)), nv.LAYOUT_ROW | nv.LAYOUT_COL,
                            rounding=nv.ROUND_SR, rht_on_col=True, rht_seed=3, sr_seed=5)
    ws = gemm_ws(tokens, d_out, d_in)
    ws2 = gemm_ws(tokens, d_in, d_out)
    y0 = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_F32, workspace=ws)
    dx0 = nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_F32, workspace=ws2)
    w_col16 = nv.nvfp4_predecode(qw, nv.COPY_COL)
    w_row16 = nv.nvfp4_predecode(qw, nv.COPY_ROW)
    assert w_col16.shape == (d_out, d_in) and w_row16.shape == (d_in, d_out)
    # The decoded copy is value * block scale (no tensor scale): times s_dec it is the dequantized tensor, up to FP32
    # rounding -- once its elements are put back in row order.  The buffer holds them as the GEMM loads them: 16-row
    # blocks, within a block the steps of 32 k, and within a step (1 KiB) the 16-byte chunks chunk-major: the 16 rows'
    # first 8 k, then their second, third and fourth.
    tiled = w_col16.view(d_out // 16, d_in // 32, 4, 16, 8)          # [block][step][chunk][row in block][8 elements]
    row_major = tiled.permute(0, 3, 1, 2, 4).reshape(d_out, d_in)
    deq = nv.nvfp4_dequantize(qw, nv.COPY_COL)
    assert torch.allclose(row_major.float() * qw.col_ts[0], deq, rtol=1e-6, atol=0)
    # less scratch is enough now: only X (or dY) and the partial tiles
    small = torch.empty(nv.gemm_workspace_bytes(tokens, d_out, d_in) - d_out * d_in * 2, dtype=torch.uint8, device="cuda")
    y1 = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_F32, workspace=small)
    assert torch.equal(y1, y0)
    small2 = torch.empty(nv.gemm_workspace_bytes(tokens, d_in, d_out) - d_in * d_out * 2, dtype=torch.uint8, device="cuda")
    dx1 = nv.nvfp4_gemm(qdy, qw, nv.OP_DGRAD, nv.OUT_F32, workspace=small2)
    assert torch.equal(dx1, dx0)
    # both operands decoded beforehand (Wgrad): only partial tiles remain in the workspace, here none: no workspace at all
    dw0 = nv.nvfp4_gemm(qx, qdy, nv.OP_WGRAD, nv.OUT_F32, workspace=gemm_ws(d_in, d_out, tokens))
    nv.nvfp4_predecode(qx, nv.COPY_COL)
    nv.nvfp4_predecode(qdy, nv.COPY_COL)
    tiny = torch.empty(nv.gemm_workspace_bytes(d_in, d_out, tokens) - (d_in + d_out) * tokens * 2, dtype=torch.uint8, device="cuda")
    assert torch.equal(nv.nvfp4_gemm(qx, qdy, nv.OP_WGRAD, nv.OUT_F32, workspace=tiny), dw0)
    # the fused route ignores decoded copies
    assert torch.equal(nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_F32), nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_F32))
    # requantizing into the descriptor drops the decoded copies (they would be stale)
    nv.nvfp4_quantize(to_dev(wb), nv.LAYOUT_ROW | nv.LAYOUT_COL, nv.BLOCK_16x16, out=qw)
    assert qw.desc.row_fp16 is None and qw.desc.col_fp16 is None and qw.row_fp16 is None
    y2 = nv.nvfp4_gemm(qx, qw, nv.OP_FPROP, nv.OUT_F32, workspace=ws)
    assert torch.equal(y2, y0)
