"""Pins for the oracle's GEMM references (CPU only): App. B.3 Eq. 5 and Sec. 2."""
import numpy as np

import oracle
from paper_2509_25149_amd import synth

E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def pack(c4):
    c4 = np.asarray(c4, dtype=np.uint8)
    return (c4[:, 0::2] | (c4[:, 1::2] << 4)).astype(np.uint8)


def make(c4, scales, s_dec):
    c4 = np.asarray(c4, dtype=np.uint8)
    return oracle.QCopy(pack(c4), np.asarray(scales, dtype=np.uint8), np.float32(s_dec), np.float32(0),
                        c4.shape[0], c4.shape[1])


def values(c4):
    c4 = np.asarray(c4)
    return np.where(c4 & 8, -E2M1[c4 & 7], E2M1[c4 & 7])


def test_single_block_by_hand():
    # one 16-block per operand: A = [6,-4,3,.5, 0...] scale 1.5 (0x3C), B = [1,2,-6,1.5, 0...] scale 0.25 (0x28)
    # dot = 6 - 8 - 18 + 0.75 = -19.25 ; * 1.5 * 0.25 = -7.21875 ; * s_decA 0.5 * s_decB 4 = -14.4375
    a = np.zeros((1, 16), dtype=np.uint8)
    b = np.zeros((1, 16), dtype=np.uint8)
    a[0, :4] = [7, 8 | 6, 5, 1]
    b[0, :4] = [2, 4, 8 | 7, 3]
    A, B = make(a, [[0x3C]], 0.5), make(b, [[0x28]], 4.0)
    assert oracle.e4m3_decode(0x3C) == 1.5 and oracle.e4m3_decode(0x28) == 0.25
    assert oracle.gemm_f64(A, B)[0, 0] == -14.4375
    assert oracle.gemm_f32_blockscaled(A, B)[0, 0] == np.float32(-14.4375)


def test_all_ones_closed_form():
    M, N, K = 5, 7, 96
    a = np.full((M, K), 2, dtype=np.uint8)              # code 2 = 1.0
    A = make(a, np.full((M, K // 16), 0x38), 1.0)        # scale 1.0
    B = make(np.full((N, K), 2, dtype=np.uint8), np.full((N, K // 16), 0x40), 0.75)   # scale 2.0
    want = K * 1.0 * 2.0 * 0.75
    assert np.all(oracle.gemm_f64(A, B) == want)
    assert np.all(oracle.gemm_f32_blockscaled(A, B) == np.float32(want))


def test_unit_scales_reduce_to_an_integer_matmul():
    rng = np.random.default_rng(21)
    M, N, K = 9, 11, 64
    a, b = rng.integers(0, 16, (M, K)), rng.integers(0, 16, (N, K))
    A = make(a, np.full((M, K // 16), 0x38), 1.0)
    B = make(b, np.full((N, K // 16), 0x38), 1.0)
    ai, bi = (values(a) * 2).astype(np.int64), (values(b) * 2).astype(np.int64)
    want = (ai @ bi.T) / 4.0
    assert np.array_equal(oracle.gemm_f64(A, B), want)
    assert np.array_equal(oracle.gemm_f32_blockscaled(A, B).astype(np.float64), want)


def test_operand_order_and_transposition():
    # D[m, n] = sum_k A[m, k] B[n, k]: a one-hot A row picks a B column
    K = 32
    a = np.zeros((3, K), dtype=np.uint8)
    a[1, 17] = 2                                          # A[1, 17] = 1
    b = np.random.default_rng(2).integers(0, 16, (4, K))
    A = make(a, np.full((3, 2), 0x38), 1.0)
    B = make(b, np.full((4, 2), 0x38), 1.0)
    D = oracle.gemm_f64(A, B)
    assert D.shape == (3, 4)
    assert np.array_equal(D[1], values(b)[:, 17]) and not D[0].any() and not D[2].any()


def test_f64_reference_equals_numpy_on_dequantized_operands_and_eq5_form():
    xb = synth.normal_with_outliers(48, 256, 1.0, 31, frac=0.01)
    wb = synth.normal(256, 80, 0.02, 32)
    A = oracle.quantize(xb, oracle.ROW)
    B = oracle.quantize(wb, oracle.COL, oracle.BLOCK_16x16)
    D = oracle.gemm_f64(A, B)
    da, db = oracle.dequantize(A).astype(np.float64), oracle.dequantize(B).astype(np.float64)
    # binary32 dequantization rounds twice; compare against an exact-in-double decode instead
    ea = values(np.stack([A.codes & 15, A.codes >> 4], -1).reshape(48, 256)) * \
        np.repeat([[oracle.e4m3_decode(int(v)) for v in r] for r in A.scales], 16, axis=1) * float(A.s_dec)
    eb = values(np.stack([B.codes & 15, B.codes >> 4], -1).reshape(80, 256)) * \
        np.repeat([[oracle.e4m3_decode(int(v)) for v in r] for r in B.scales], 16, axis=1) * float(B.s_dec)
    ref = ea @ eb.T
    assert np.linalg.norm(D - ref) <= 1e-13 * np.linalg.norm(ref)
    assert np.linalg.norm(D - da @ db.T) <= 1e-6 * np.linalg.norm(ref)
    # Eq. 5 with binary32 accumulation agrees to binary32 accuracy
    S = oracle.gemm_f32_blockscaled(A, B)
    assert np.linalg.norm(S - D) <= 1e-6 * np.linalg.norm(D)
    # and the quantized product approximates the unquantized one (sanity of the whole path)
    x, w = synth.bf16_bits_to_f32(xb).astype(np.float64), synth.bf16_bits_to_f32(wb).astype(np.float64)
    assert np.linalg.norm(D - x @ w) <= 0.2 * np.linalg.norm(x @ w)


def test_entries_variant_matches_full():
    xb = synth.normal(32, 64, 1.0, 41)
    yb = synth.normal(48, 64, 1.0, 42)
    A, B = oracle.quantize(xb, oracle.ROW), oracle.quantize(yb, oracle.ROW)
    D = oracle.gemm_f64(A, B)
    m = np.array([0, 5, 31, 17]); n = np.array([47, 0, 3, 17])
    assert np.array_equal(oracle.gemm_f64_entries(A, B, m, n), D[m, n])


def test_wgrad_with_rotation_approximates_the_plain_product():
    # Sec. 4.2 / App. C: rotating both Wgrad operands along the token dimension
    # cancels inside the dot product (up to quantization error).
    dyb = synth.student_t3(128, 48, 1e-3, 51)
    xb = synth.normal_with_outliers(128, 64, 1.0, 52, frac=0.01)
    seed = 4242
    A = oracle.quantize(dyb, oracle.COL, use_rht=True, rht_seed=seed, rounding=oracle.SR, sr_seed=1)
    B = oracle.quantize(xb, oracle.COL, use_rht=True, rht_seed=seed)
    D = oracle.gemm_f64(A, B)                              # [48, 64] = dY^T X
    ref = synth.bf16_bits_to_f32(dyb).astype(np.float64).T @ synth.bf16_bits_to_f32(xb).astype(np.float64)
    assert np.linalg.norm(D - ref) <= 0.25 * np.linalg.norm(ref)
    # a mismatched sign diagonal on one operand breaks the cancellation
    B2 = oracle.quantize(xb, oracle.COL, use_rht=True, rht_seed=seed + 1)
    if oracle.rht_sign_mask(seed) != oracle.rht_sign_mask(seed + 1):
        assert np.linalg.norm(oracle.gemm_f64(A, B2) - ref) > 0.5 * np.linalg.norm(ref)


def test_accumulate_into_is_a_plain_sum():
    """Sec. 4.1 gradient accumulation: the K range split into two micro-batches and accumulated equals the GEMM
    over the whole K range (the tensor scales are shared by construction: both halves are cut from one
    quantized tensor), and adding into zeros is the product itself."""
    xb = synth.normal(32, 64, 1.0, 71)
    wb = synth.normal(48, 64, 0.02, 72)
    qa, qb = oracle.quantize(xb, oracle.ROW), oracle.quantize(wb, oracle.ROW)
    whole = oracle.gemm_f64(qa, qb)
    assert np.array_equal(oracle.gemm_f64(qa, qb, d_prev=np.zeros((32, 48), np.float32)), whole)

    def half(q, lo, hi):
        return oracle.QCopy(np.ascontiguousarray(q.codes[:, lo // 2:hi // 2]), np.ascontiguousarray(q.scales[:, lo // 16:hi // 16]),
                            q.s_dec, q.amax, q.outer, hi - lo)
    first = oracle.gemm_f64(half(qa, 0, 32), half(qb, 0, 32))
    d32 = first.astype(np.float32)
    both = oracle.gemm_f64(half(qa, 32, 64), half(qb, 32, 64), d_prev=d32)
    # d32 carries one FP32 rounding of the first half: error at most 2^-24 relative to it
    assert np.all(np.abs(both - whole) <= np.abs(first) * 2.0 ** -24 + 1e-300)
    assert np.linalg.norm(both - whole) / np.linalg.norm(whole) < 1e-7
