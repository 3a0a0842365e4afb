"""Pins for the oracle's random bits and Hadamard rotation (CPU only).

Philox4x32-10: the published known-answer vectors (tests/golden).  Rotation:
App. C of the paper -- normalised Sylvester matrix, orthogonality, and the
identity C = (A H)(H^T B) = A B.
"""
import os

import numpy as np

import oracle


def test_philox_known_answers(golden_dir):
    n = 0
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            out = oracle.philox4x32_10(w[0:4], w[4:6])
            assert [int(v) for v in out] == w[6:10]
            n += 1
    assert n == 3


def test_sr_random16_counter_layout():
    seed = 0x0123456789ABCDEF
    key = [seed & 0xFFFFFFFF, seed >> 32]
    for i, j in [(0, 0), (0, 7), (0, 8), (5, 13), (4095, 5119), (70000, 3)]:
        w = oracle.philox4x32_10([j >> 3, i, 0, 0], key)
        word = int(w[(j & 7) >> 1])
        want = (word >> 16) if (j & 1) else (word & 0xFFFF)
        assert oracle.sr_random16(seed, i, j) == want


def test_sr_random16_is_roughly_uniform():
    r = np.array([oracle.sr_random16(99, i, j) for i in range(64) for j in range(256)], dtype=np.float64)
    n = r.size
    assert abs(r.mean() - 32767.5) < 4 * 65536 / np.sqrt(12 * n)
    hist = np.bincount((r // 4096).astype(int), minlength=16)
    assert hist.min() > 0.85 * n / 16 and hist.max() < 1.15 * n / 16


def test_sign_mask_definition_and_balance():
    for seed in (0, 1, 2025, 2 ** 63 + 5):
        w = oracle.philox4x32_10([0, 0, 0, 0xFFFFFFFF], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.rht_sign_mask(seed) == int(w[0]) & 0xFFFF
    bits = sum(bin(oracle.rht_sign_mask(s)).count("1") for s in range(400))
    assert abs(bits - 3200) < 4 * np.sqrt(6400 * 0.25)


def sylvester16():
    h2 = np.array([[1.0, 1.0], [1.0, -1.0]])
    h = np.array([[1.0]])
    for _ in range(4):
        h = np.kron(h2, h)                         # App. C: H_d = (1/sqrt 2) H_2 (x) H_{d/2}
    return h / 4.0                                 # four factors of 1/sqrt 2, applied exactly


def test_sylvester_matrix_entries():
    h = sylvester16()
    for i in range(16):
        for j in range(16):
            assert h[i, j] == (-1.0) ** bin(i & j).count("1") / 4.0
    assert np.array_equal(h, h.T)
    assert np.array_equal(h @ h.T, np.eye(16))


def test_butterfly_equals_dense_matrix_on_small_integers():
    rng = np.random.default_rng(3)
    h = sylvester16()
    for mask in (0, 0xFFFF, 0x5A3C, oracle.rht_sign_mask(2025)):
        s = np.array([-1.0 if (mask >> i) & 1 else 1.0 for i in range(16)])
        for _ in range(50):
            v = rng.integers(-64, 65, 16).astype(np.float32)
            want = (v.astype(np.float64) * s) @ h            # (v .* s) H, exact for small ints
            got = oracle.rht16_forward(v, mask)
            assert np.array_equal(got.astype(np.float64), want)
            back = oracle.rht16_inverse(got, mask)
            assert np.array_equal(back, v)


def test_unit_impulse():
    v = np.zeros(16, dtype=np.float32)
    v[3] = 16.0
    got = oracle.rht16_forward(v, 0)
    want = np.array([4.0 * (-1.0) ** bin(i & 3).count("1") for i in range(16)], dtype=np.float32)
    assert np.array_equal(got, want)
    got = oracle.rht16_forward(v, 1 << 3)
    assert np.array_equal(got, -want)


def test_rotation_is_orthogonal_for_any_mask():
    rng = np.random.default_rng(4)
    for mask in (0, 0x8001, 0xBEEF):
        v = rng.standard_normal(16).astype(np.float32)
        y = oracle.rht16_forward(v, mask)
        assert abs(float(np.dot(y.astype(np.float64), y.astype(np.float64))) -
                   float(np.dot(v.astype(np.float64), v.astype(np.float64)))) < 1e-5
        assert np.allclose(oracle.rht16_inverse(y, mask), v, atol=1e-6)


def test_rotating_both_operands_leaves_the_product_unchanged():
    # C = (A H)(H^T B) = A B (App. C), here along a contraction of 64 = 4 groups of 16.
    rng = np.random.default_rng(5)
    mask = oracle.rht_sign_mask(77)
    a = rng.integers(-8, 9, (6, 64)).astype(np.float32)      # [m, k]
    b = rng.integers(-8, 9, (5, 64)).astype(np.float32)      # [n, k]
    ar = np.stack([np.concatenate([oracle.rht16_forward(r[g:g + 16], mask) for g in range(0, 64, 16)]) for r in a])
    br = np.stack([np.concatenate([oracle.rht16_forward(r[g:g + 16], mask) for g in range(0, 64, 16)]) for r in b])
    want = a.astype(np.float64) @ b.astype(np.float64).T
    got = ar.astype(np.float64) @ br.astype(np.float64).T
    assert np.max(np.abs(got - want)) < 1e-9
