"""Pins for the oracle's quantizer with one tensor-level scale per row of the copy (CPU only): App. B.1, last
sentence, with Eq. 1 evaluated per row and Eq. 2-5 unchanged."""
import os

import numpy as np
import pytest

import oracle
from paper_2509_25149_amd import synth
from test_oracle_quantize import bits, unpack, read_golden, e4m3_values, code_values


def test_handworked_three_row_tensor(golden_dir):
    g = read_golden(os.path.join(golden_dir, "handworked_row_scales.txt"))
    x = np.array([[float(t) for t in g[f"x{r}"]] for r in range(3)], dtype=np.float32)
    xb = bits(x)
    assert np.array_equal(synth.bf16_bits_to_f32(xb), x), "fixture must be bf16-exact"
    q = oracle.quantize_row_scales(xb, oracle.ROW)
    assert [int(v) for v in q.amax.view(np.uint32)] == [int(t, 16) for t in g["amax_bits"]]
    assert [int(v) for v in q.s_dec.view(np.uint32)] == [int(t, 16) for t in g["s_dec_bits"]]
    assert [int(v) for v in q.scales.ravel()] == [int(t, 16) for t in g["scales"]]
    for r in range(3):
        assert [int(v) for v in unpack(q.codes)[r]] == [int(t, 16) for t in g[f"codes{r}"]], r
    # the per-tensor scale gives row 1 something else (its first block would store 0.5 = 0x30)
    assert oracle.quantize(xb, oracle.ROW).scales[1, 0] == 0x30
    # the same tensor as columns: the col copy of the transpose, scales per logical column
    qc = oracle.quantize_row_scales(np.ascontiguousarray(xb.T), oracle.COL)
    assert np.array_equal(qc.codes, q.codes) and np.array_equal(qc.scales, q.scales)
    assert np.array_equal(qc.s_dec.view(np.uint32), q.s_dec.view(np.uint32))


@pytest.mark.parametrize("copy", [oracle.ROW, oracle.COL])
@pytest.mark.parametrize("mode", [dict(), dict(rounding=oracle.SR, sr_seed=9), dict(use_rht=True, rht_seed=3),
                                  dict(rounding=oracle.SR, sr_seed=9, use_rht=True, rht_seed=3)])
def test_every_row_is_quantized_as_a_tensor_of_its_own(copy, mode):
    """Row o of the copy must come out exactly as the per-tensor routine (pinned by the hand-worked cases and the
    App. B.2 invariants) quantizes that row alone -- except for the stochastic-rounding draws, which belong to the
    element's position in the whole tensor."""
    rows, cols = (48, 160) if copy == oracle.ROW else (160, 48)
    xb = synth.normal_with_outliers(rows, cols, 1.0, 31, frac=0.02)
    xb[5 if copy == oracle.ROW else slice(None), slice(None) if copy == oracle.ROW else 5] = 0          # an all-zero row of the copy
    q = oracle.quantize_row_scales(xb, copy, **mode)
    view = xb if copy == oracle.ROW else np.ascontiguousarray(xb.T)
    assert q.per_row and q.s_dec.shape == (view.shape[0],)
    for o in range(view.shape[0]):
        alone = view[o:o + 1] if copy == oracle.ROW else np.ascontiguousarray(view[o:o + 1].T)
        if mode.get("rounding") == oracle.SR:
            # same draws: quantize the whole tensor per tensor with this row's amax supplied
            ref_all = oracle.quantize(xb, copy, amax=float(q.amax[o]), **mode)
            ref_codes, ref_scales, ref_sdec = ref_all.codes[o], ref_all.scales[o], ref_all.s_dec
        else:
            ref = oracle.quantize(alone, copy, **mode)
            ref_codes, ref_scales, ref_sdec = ref.codes[0], ref.scales[0], ref.s_dec
            assert ref.amax.view(np.uint32) == q.amax[o].view(np.uint32)
        assert np.array_equal(q.codes[o], ref_codes), o
        assert np.array_equal(q.scales[o], ref_scales), o
        assert q.s_dec[o].view(np.uint32) == ref_sdec.view(np.uint32), o
    assert q.amax[5] == 0 and q.s_dec[5] == 1 and not q.codes[5].any() and not q.scales[5].any()


def test_each_rows_amax_block_stores_the_e4m3_maximum():
    xb = synth.normal_with_outliers(64, 256, 1.0, 32, frac=0.01)
    x = synth.bf16_bits_to_f32(xb)
    q = oracle.quantize_row_scales(xb, oracle.ROW)
    assert np.array_equal(q.amax, np.abs(x).max(axis=1))
    k = np.abs(x).argmax(axis=1)
    assert np.all(q.scales[np.arange(64), k // 16] == 0x7E)              # App. B.2: the amax block maps to 448
    assert np.all((unpack(q.codes)[np.arange(64), k] & 7) == 7)         # and the amax element to +-6
    # per-tensor scaling only does that for the one row holding the tensor's amax
    assert (oracle.quantize(xb, oracle.ROW).scales == 0x7E).sum() < 8


def test_equal_row_amaxes_give_the_per_tensor_result():
    xb = synth.normal(32, 128, 1.0, 33)
    x = synth.bf16_bits_to_f32(xb).copy()
    x[:, 7] = 8.0                                                       # every row's (and the tensor's) amax
    x = np.clip(x, -8, 8)
    xb = bits(x)
    a, b = oracle.quantize_row_scales(xb, oracle.ROW), oracle.quantize(xb, oracle.ROW)
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.scales, b.scales)
    assert np.all(a.s_dec.view(np.uint32) == b.s_dec.view(np.uint32)) and np.all(a.amax == b.amax)


def test_codes_do_not_change_when_single_rows_are_scaled_by_powers_of_two():
    """What the finer granularity buys: a row's codes and block scales depend on that row alone, so scaling row i by
    2^k_i only moves s_dec[i] (exactly); with one scale per tensor the small rows would lose their low bits."""
    xb = synth.normal_with_outliers(24, 96, 1.0, 34, frac=0.02)
    x = synth.bf16_bits_to_f32(xb)
    k = np.arange(24) - 12
    xs = bits(x * np.exp2(k)[:, None].astype(np.float32))
    a, b = oracle.quantize_row_scales(xb, oracle.ROW), oracle.quantize_row_scales(xs, oracle.ROW)
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.scales, b.scales)
    assert np.array_equal(b.s_dec, a.s_dec * np.exp2(k).astype(np.float32))
    assert np.array_equal(oracle.dequantize(b), oracle.dequantize(a) * np.exp2(k)[:, None].astype(np.float32))
    assert not np.array_equal(oracle.quantize(xb, oracle.ROW).codes, oracle.quantize(xs, oracle.ROW).codes)


def test_dequantize_applies_the_rows_own_scale():
    xb = synth.normal_with_outliers(16, 64, 1.0, 35, frac=0.05)
    q = oracle.quantize_row_scales(xb, oracle.ROW)
    want = (code_values(unpack(q.codes)) * np.repeat(e4m3_values(q.scales), 16, axis=1)) * q.s_dec[:, None]
    assert np.array_equal(oracle.dequantize(q), want)
    x = synth.bf16_bits_to_f32(xb)
    assert np.all(np.abs(oracle.dequantize(q) - x) <= np.abs(x).max(axis=1, keepdims=True) / 6 * 1.07)   # half a step of the coarsest block
    # rotated col copy: undoing the rotation recovers the tensor to the same accuracy
    xc = synth.normal(64, 16, 1.0, 36)
    qc = oracle.quantize_row_scales(xc, oracle.COL, use_rht=True, rht_seed=8)
    back = oracle.dequantize(qc, undo_rht=True, rht_seed=8).T
    assert np.linalg.norm(back - synth.bf16_bits_to_f32(xc)) <= 0.12 * np.linalg.norm(synth.bf16_bits_to_f32(xc))


def test_gemm_with_row_scales():
    # closed form: all-ones operands with per-row magnitudes 2^i and 2^-j: D[i, j] = K * 2^(i - j), exactly
    M, N, K = 8, 6, 64
    a = bits(np.exp2(np.arange(M))[:, None] * np.ones((M, K)))
    b = bits(np.exp2(-np.arange(N))[:, None] * np.ones((N, K)))
    qa, qb = oracle.quantize_row_scales(a, oracle.ROW), oracle.quantize_row_scales(b, oracle.ROW)
    d = oracle.gemm_f64(qa, qb)
    want = K * np.exp2(np.arange(M))[:, None] * np.exp2(-np.arange(N))[None, :]
    assert np.allclose(d, want, rtol=3e-7, atol=0)           # s_dec = fl(1 / fl(2688 / amax)) carries two roundings
    # against the product of the dequantized operands (a library matmul), mixed granularity included
    xb, wb = synth.normal_with_outliers(40, 96, 1.0, 37, frac=0.02), synth.normal(24, 96, 0.02, 38)
    for qa, qb in ((oracle.quantize_row_scales(xb, oracle.ROW), oracle.quantize_row_scales(wb, oracle.ROW)),
                   (oracle.quantize_row_scales(xb, oracle.ROW), oracle.quantize(wb, oracle.ROW)),
                   (oracle.quantize(xb, oracle.ROW), oracle.quantize_row_scales(wb, oracle.ROW))):
        ref = oracle.dequantize(qa).astype(np.float64) @ oracle.dequantize(qb).astype(np.float64).T
        # (the FP32 dequantized values carry one rounding each, the binary64 reference none)
        assert np.linalg.norm(oracle.gemm_f64(qa, qb) - ref) <= 1e-6 * np.linalg.norm(ref)
    # rotated Wgrad operands with per-feature scales still approximate the unrotated product (App. C)
    xw, dyw = synth.normal(256, 32, 1.0, 39), synth.student_t3(256, 48, 1e-3, 40)
    qx = oracle.quantize_row_scales(xw, oracle.COL, use_rht=True, rht_seed=6)
    qd = oracle.quantize_row_scales(dyw, oracle.COL, use_rht=True, rht_seed=6)
    exact = synth.bf16_bits_to_f32(xw).astype(np.float64).T @ synth.bf16_bits_to_f32(dyw).astype(np.float64)
    assert np.linalg.norm(oracle.gemm_f64(qx, qd) - exact) <= 0.15 * np.linalg.norm(exact)


def test_bad_arguments():
    xb = synth.normal(32, 32, 1.0, 41)
    with pytest.raises(ValueError):
        oracle.quantize_row_scales(xb[:, :24], oracle.ROW)
    with pytest.raises(ValueError):
        oracle.quantize_row_scales(xb, oracle.ROW, use_rht=True, rht_dim=3)
