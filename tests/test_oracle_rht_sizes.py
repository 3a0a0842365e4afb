"""Pins for the oracle's rotations of other sizes (CPU only).

Sec. 4.2 ("Hadamard matrix size") and App. E.4 ablate d = 2, 4 and 128 against the
chosen d = 16; App. C fixes H_d = (1/sqrt 2) H_2 (x) H_{d/2} and H = S_d H_d.  Checked
here against the dense matrix built from that recursion, the closed-form entries, an
outlier's known spread, and the quantizer's reported amax.
"""
import numpy as np
import pytest

import oracle
from paper_2509_25149_amd import synth

SIZES = (2, 4, 16, 32, 128)


def sylvester(d):
    h2 = np.array([[1.0, 1.0], [1.0, -1.0]])
    h = np.array([[1.0]])
    while h.shape[0] < d:
        h = np.kron(h2, h)
    return h / np.sqrt(float(d))


@pytest.mark.parametrize("d", SIZES)
def test_signs_are_the_first_d_bits_of_the_philox_call(d):
    for seed in (0, 9, 2 ** 63 + 5):
        w = oracle.philox4x32_10([0, 0, 0, 0xFFFFFFFF], [seed & 0xFFFFFFFF, seed >> 32])
        want = [(int(w[i // 32]) >> (i % 32)) & 1 for i in range(d)]
        assert oracle.rht_signs(seed, d).tolist() == want
    # the 16- and 32-point masks are the same bits
    m16 = oracle.rht_sign_mask(9)
    assert oracle.rht_signs(9, 16).tolist() == [(m16 >> i) & 1 for i in range(16)]
    m32 = oracle.rht_sign_mask32(9)
    assert oracle.rht_signs(9, 32).tolist() == [(m32 >> i) & 1 for i in range(32)]


@pytest.mark.parametrize("d", SIZES)
def test_matrix_entries_closed_form(d):
    h = sylvester(d)
    i, j = np.meshgrid(np.arange(d), np.arange(d), indexing="ij")
    pop = np.vectorize(lambda t: bin(t).count("1"))(i & j)
    assert np.allclose(h, (-1.0) ** pop / np.sqrt(d), rtol=0, atol=1e-15)
    assert np.allclose(h @ h.T, np.eye(d), atol=1e-12)


@pytest.mark.parametrize("d", SIZES)
def test_butterfly_equals_dense_matrix(d):
    rng = np.random.default_rng(d)
    h = sylvester(d)
    norm = np.float32(1.0 / np.sqrt(float(d)))
    for neg in (np.zeros(d, np.uint8), np.ones(d, np.uint8), oracle.rht_signs(2025, d)):
        s = 1.0 - 2.0 * neg.astype(np.float64)
        for _ in range(20):
            v = rng.integers(-64, 65, d).astype(np.float32)
            got = oracle.rht_forward(v, neg).astype(np.float64)
            # small integers: the unnormalised sums are exact, so the only rounding is the final multiply
            exact_sums = (v.astype(np.float64) * s) @ (h * np.sqrt(float(d)))
            want = (exact_sums.astype(np.float32) * norm).astype(np.float64)
            assert np.array_equal(got, want)
            assert np.allclose(got, (v.astype(np.float64) * s) @ h, rtol=1e-6, atol=1e-6)
            back = oracle.rht_inverse(got.astype(np.float32), neg)
            assert np.allclose(back, v, atol=1e-4)


def test_sixteen_point_case_is_the_original_routine():
    rng = np.random.default_rng(1)
    mask = oracle.rht_sign_mask(31)
    neg = oracle.rht_signs(31, 16)
    for _ in range(20):
        v = rng.standard_normal(16).astype(np.float32)
        assert np.array_equal(oracle.rht_forward(v, neg), oracle.rht16_forward(v, mask))
        assert np.array_equal(oracle.rht_inverse(v, neg), oracle.rht16_inverse(v, mask))
    mask = oracle.rht_sign_mask32(31)
    neg = oracle.rht_signs(31, 32)
    for _ in range(20):
        v = rng.standard_normal(32).astype(np.float32)
        assert np.array_equal(oracle.rht_forward(v, neg), oracle.rht32_forward(v, mask))


@pytest.mark.parametrize("d", SIZES)
def test_an_outlier_spreads_evenly_over_its_group(d):
    # one outlier of magnitude 2^k in a group of d becomes d values of magnitude 2^k / sqrt(d)
    v = np.zeros(d, dtype=np.float32)
    v[d // 2 + 1 if d > 2 else 1] = 1024.0
    got = oracle.rht_forward(v, np.zeros(d, np.uint8))
    assert np.array_equal(np.abs(got), np.full(d, np.float32(1024.0) * np.float32(1.0 / np.sqrt(float(d))), np.float32))
    assert abs(float(np.abs(got)[0]) - 1024.0 / np.sqrt(d)) < 1e-4


@pytest.mark.parametrize("d", SIZES)
def test_quantizer_reports_the_rotated_amax_and_rotates_groups_of_d(d):
    # Column j of x holds one outlier per aligned group of d rows; after the rotation along rows every entry of the
    # col copy has magnitude outlier / sqrt(d), so amax says which d was used and every block scale is the same.
    rows, cols = 256, 32
    x = np.zeros((rows, cols), dtype=np.float32)
    for g in range(rows // d):
        x[g * d + (g % d), :] = 512.0
    q = oracle.quantize(synth.f32_to_bf16_bits(x), oracle.COL, use_rht=True, rht_seed=3, rht_dim=d)
    want = np.float32(512.0) * np.float32(1.0 / np.sqrt(float(d)))
    assert q.amax == want
    assert len(set(q.scales.ravel().tolist())) == 1
    assert np.all((q.codes & 7) == 7) and np.all(((q.codes >> 4) & 7) == 7)       # every magnitude is the block's amax: code 6
    back = oracle.dequantize(q, undo_rht=True, rht_seed=3, rht_dim=d)             # [cols, rows]
    assert np.allclose(back.T, x, rtol=0, atol=512.0 * 2e-6 * d)


@pytest.mark.parametrize("d", SIZES)
def test_rotating_both_operands_leaves_the_product_unchanged(d):
    rng = np.random.default_rng(5 + d)
    neg = oracle.rht_signs(77, d)
    k = 2 * d if d >= 16 else 32
    a = rng.integers(-8, 9, (6, k)).astype(np.float32)
    b = rng.integers(-8, 9, (5, k)).astype(np.float32)
    rot = lambda m: np.stack([np.concatenate([oracle.rht_forward(r[g:g + d], neg) for g in range(0, k, d)]) for r in m])
    want = a.astype(np.float64) @ b.astype(np.float64).T
    got = rot(a).astype(np.float64) @ rot(b).astype(np.float64).T
    assert np.max(np.abs(got - want)) < 1e-3


def test_rejects_sizes_outside_the_list_and_ragged_groups():
    with pytest.raises(ValueError):
        oracle.rht_signs(1, 8)
    x = np.zeros((48, 16), dtype=np.uint16)
    with pytest.raises(ValueError):
        oracle.quantize(x, oracle.COL, use_rht=True, rht_dim=32)      # 48 rows are not whole groups of 32
    with pytest.raises(ValueError):
        oracle.quantize(x, oracle.COL, use_rht=True, rht_dim=64)
