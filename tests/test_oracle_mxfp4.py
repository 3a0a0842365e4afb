"""Pins of the MXFP4 part of the oracle (comparison format: Sec. 2, App. B.4, Sec. 5) against what the paper and
the mathematics fix.  CPU only."""
import math

import numpy as np
import pytest

import oracle
from paper_2509_25149_amd import synth

GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def bf16(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def unpack(codes):
    lo, hi = codes & 15, codes >> 4
    return np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1)


def code_values(c):
    return np.where(c & 8, -GRID[c & 7], GRID[c & 7])


def test_scale_is_the_next_power_of_two_at_or_above_amax_over_6():
    """Sec. 2: UE8M0 scales are powers of two; App. B.4: rounded up.  Exact rational check, no float log."""
    rng = np.random.default_rng(5)
    vals = np.concatenate([np.float32(2.0) ** rng.integers(-120, 120, 200), rng.random(500).astype(np.float32) * 1000,
                           np.float32([1.0, 0.5, 0.25, 6.0, 3.0, 3.0000002, 2.9999998])])
    for s in vals.astype(np.float32):
        e = oracle.ue8m0_exponent_round_up(float(s))
        from fractions import Fraction
        assert Fraction(2) ** e >= Fraction(float(s))
        if e > -127:
            assert Fraction(2) ** (e - 1) < Fraction(float(s))
    assert oracle.ue8m0_exponent_round_up(0.0) == -127
    assert oracle.ue8m0_exponent_round_up(float(np.float32(2.0) ** -140)) == -127       # clamped to the UE8M0 range


def test_worked_example_of_appendix_b4():
    """App. B.4: a block whose amax is 3 + delta gets decode scale 0.5 + delta/6 -> rounded up to 1, and its amax
    then quantizes to 3: the samples 4 and 6 go unused.  With amax exactly 3 the scale is 0.5 and 3 maps to 6."""
    x = np.zeros((1, 64), dtype=np.float32)
    x[0, :32] = np.linspace(-3.0, 3.0, 32)
    x[0, 7] = 3.0625                      # 3 + delta, exact in bf16
    x[0, 32:] = np.linspace(-3.0, 3.0, 32)
    x[0, 32 + 31] = 3.0
    q = oracle.mx_quantize(bf16(x), oracle.ROW)
    assert q.scales.shape == (1, 2)
    assert int(q.scales[0, 0]) - 127 == 0 and int(q.scales[0, 1]) - 127 == -1
    c = unpack(q.codes)[0]
    assert code_values(c[7:8])[0] == 3.0                       # 3.0625 / 1 -> 3
    assert np.abs(code_values(c[:32])).max() == 3.0            # 4 and 6 unused in the first block
    assert code_values(c[63:64])[0] == 6.0                     # 3 / 0.5 -> 6 in the second
    d = oracle.mx_dequantize(q)
    assert d[0, 7] == 3.0 and d[0, 63] == 3.0


def reference_mx_quantize_rne(x):
    """Independent numpy formulation for one row copy (RNE): exponents through np.frexp on float64."""
    rows, cols = x.shape
    codes = np.zeros((rows, cols), dtype=np.uint8)
    scales = np.zeros((rows, cols // 32), dtype=np.uint8)
    for r in range(rows):
        for b in range(cols // 32):
            blk = x[r, 32 * b:32 * b + 32].astype(np.float32)
            amax = np.abs(blk).max()
            s = np.float32(amax) / np.float32(6.0)
            if s == 0:
                e = -127
            else:
                m, ex = math.frexp(float(s))
                e = ex - 1 if m == 0.5 else ex
                e = min(max(e, -127), 127)
            scales[r, b] = e + 127
            v = blk.astype(np.float64) * 2.0 ** (-e)            # exact: power-of-two scaling of binary32 values
            for k in range(32):
                a = abs(v[k])
                if a >= 6:
                    idx = 7
                else:
                    lo = np.searchsorted(GRID, a, side="right") - 1
                    hi = lo + 1
                    mid = (GRID[lo] + GRID[hi]) / 2
                    if a < mid:
                        idx = lo
                    elif a > mid:
                        idx = hi
                    else:
                        idx = lo if lo % 2 == 0 else hi         # ties to the code with mantissa bit 0
                codes[r, 32 * b + k] = idx | (8 if np.signbit(v[k]) else 0)
    return codes, scales


def test_row_copy_against_an_independent_numpy_formulation():
    xb = synth.normal_with_outliers(8, 128, 1.0, 61, frac=0.02)
    x = synth.bf16_bits_to_f32(xb)
    q = oracle.mx_quantize(xb, oracle.ROW)
    codes, scales = reference_mx_quantize_rne(x)
    assert np.array_equal(q.scales, scales)
    assert np.array_equal(unpack(q.codes), codes)
    # the col copy is the row copy of the transpose
    xb2 = synth.normal(64, 32, 0.3, 62)
    a = oracle.mx_quantize(xb2, oracle.COL)
    b = oracle.mx_quantize(np.ascontiguousarray(xb2.T), oracle.ROW)
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.scales, b.scales)
    assert a.codes.shape == (32, 32) and a.scales.shape == (32, 2)


def test_nothing_saturates_and_the_error_is_within_half_a_step():
    """App. B.4: rounding the scale up prevents saturation, so |x| / 2^e <= 6 and RNE is off by at most half of the
    local grid step (0.25, 0.5 or 1, times 2^e)."""
    xb = synth.student_t3(64, 256, 0.02, 63)
    x = synth.bf16_bits_to_f32(xb).astype(np.float64)
    q = oracle.mx_quantize(xb, oracle.ROW)
    e = q.scales.astype(np.int64) - 127
    scale = np.repeat(2.0 ** e, 32, axis=1)
    v = np.abs(x) / scale
    assert v.max() <= 6.0
    d = oracle.mx_dequantize(q).astype(np.float64)
    step = np.where(v < 2, 0.5, np.where(v < 4, 1.0, 2.0))
    assert np.all(np.abs(d - x) <= step / 2 * scale + 1e-300)
    # every block's amax lands in (3, 6] after scaling unless the block is all zero (the lost binade of App. B.4)
    blk_max = v.reshape(64, -1, 32).max(axis=2)
    assert np.all((blk_max > 3.0) | (blk_max == 0.0)) and np.all(blk_max <= 6.0)


def sylvester(n):
    h = np.array([[1.0]])
    while h.shape[0] < n:
        h = np.kron(np.array([[1.0, 1.0], [1.0, -1.0]]), h)
    return h


def test_rht32_is_the_normalised_sylvester_matrix_with_a_sign_diagonal():
    mask = oracle.rht_sign_mask32(2025)
    assert mask & 0xFFFF == oracle.rht_sign_mask(2025)                   # the 16-point mask is its low half
    s = np.array([-1.0 if (mask >> i) & 1 else 1.0 for i in range(32)])
    h = sylvester(32) / math.sqrt(32.0)
    rng = np.random.default_rng(9)
    for _ in range(20):
        v = rng.standard_normal(32).astype(np.float32)
        y = oracle.rht32_forward(v, mask).astype(np.float64)
        want = h @ (s * v.astype(np.float64))
        assert np.allclose(y, want, rtol=0, atol=8 * 2.0 ** -24 * np.abs(v).sum())
        back = oracle.rht32_inverse(y.astype(np.float32), mask)
        assert np.allclose(back, v, rtol=0, atol=2e-6 * np.abs(v).sum())
    # small integers go through the butterfly exactly: only the final 1/sqrt(32) multiply rounds
    v = rng.integers(-8, 9, 32).astype(np.float32)
    y = oracle.rht32_forward(v, 0)
    exact = sylvester(32) @ v.astype(np.float64)
    assert np.array_equal(y, (np.float32(0.176776695296636893) * exact.astype(np.float32)).astype(np.float32))
    # orthogonality: rotating both operands leaves the dot product unchanged (App. C)
    a, b = rng.standard_normal(32).astype(np.float32), rng.standard_normal(32).astype(np.float32)
    assert abs(float(oracle.rht32_forward(a, mask) @ oracle.rht32_forward(b, mask)) - float(a @ b)) < 1e-4


def test_sr_draws_and_unbiasedness():
    """Row copy: the NVFP4 draws.  Col copy: its own counters (documented convention).  SR is unbiased (Sec. 4.4)."""
    xb = bf16(np.full((32, 32), 0.8125, dtype=np.float32))
    x = 0.8125
    # block amax 0.8125 -> s = 0.1354 -> e = -2 -> scaled 3.25, between 3 and 4: P(up) = 0.25
    ups_row = ups_col = 0
    n = 0
    for seed in range(300):
        qr = oracle.mx_quantize(xb, oracle.ROW, rounding=oracle.SR, sr_seed=seed)
        qc = oracle.mx_quantize(xb, oracle.COL, rounding=oracle.SR, sr_seed=seed)
        assert int(qr.scales[0, 0]) - 127 == -2
        cr, cc = unpack(qr.codes), unpack(qc.codes)
        assert set(np.unique(cr)) <= {5, 6} and set(np.unique(cc)) <= {5, 6}
        ups_row += int((cr == 6).sum()); ups_col += int((cc == 6).sum()); n += cr.size
        if seed < 3:
            for (i, j) in ((0, 0), (5, 17), (31, 30)):
                want_r = 6 if (int(0.25 * 65536) + oracle.sr_random16(seed, i, j)) >= 65536 else 5
                want_c = 6 if (int(0.25 * 65536) + oracle.mx_col_random16(seed, i, j)) >= 65536 else 5
                assert cr[i, j] == want_r and cc[j, i] == want_c
    for ups in (ups_row, ups_col):
        p = ups / n
        assert abs(p - 0.25) < 4 * math.sqrt(0.25 * 0.75 / n)
    assert x == 0.8125


def test_gemm_reference_is_the_plain_dot_product_of_the_decoded_values():
    ab, bb = synth.normal(16, 64, 1.0, 64), synth.normal(24, 64, 0.05, 65)
    qa, qb = oracle.mx_quantize(ab, oracle.ROW), oracle.mx_quantize(bb, oracle.ROW)
    d = oracle.mx_gemm_f64(qa, qb)
    da, db = oracle.mx_dequantize(qa).astype(np.float64), oracle.mx_dequantize(qb).astype(np.float64)
    assert np.array_equal(d, np.stack([[float(np.dot(da[m], db[n])) for n in range(24)] for m in range(16)])) or \
        np.allclose(d, da @ db.T, rtol=1e-13, atol=0)
    m_idx, n_idx = np.array([0, 3, 15]), np.array([1, 23, 0])
    assert np.array_equal(oracle.mx_gemm_f64_entries(qa, qb, m_idx, n_idx), d[m_idx, n_idx])
