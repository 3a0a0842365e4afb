"""Pins for the oracle's number formats (CPU only).

E2M1 value set: Sec. 2 of the paper.  E4M3 maximum 448: App. B.1.  The encoders
are checked against brute-force nearest-neighbour searches over the whole code
space, and the E4M3/bf16 routines against PyTorch's own CPU casts.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

E2M1_VALUES = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]   # Sec. 2


def f32(x):
    return np.float32(x)


def neighbours(x):
    x = f32(x)
    return [np.nextafter(x, f32(-np.inf)), x, np.nextafter(x, f32(np.inf))]


# ---------------------------------------------------------------- E2M1

def test_e2m1_decode_is_the_papers_value_set():
    for code in range(16):
        want = E2M1_VALUES[code & 7] * (-1.0 if code & 8 else 1.0)
        got = oracle.e2m1_decode(code)
        assert got == want and np.signbit(got) == bool(code & 8)


def brute_e2m1_rne(v):
    a = Fraction(abs(float(v)))
    best = None
    for idx, g in enumerate(E2M1_VALUES):
        d = abs(a - Fraction(g))
        if best is None or d < best[0] or (d == best[0] and idx % 2 == 0 and best[1] % 2 == 1):
            best = (d, idx)
    return (8 if np.signbit(v) else 0) | best[1]


def e2m1_probe_values():
    vals = []
    for g in E2M1_VALUES:
        vals += neighbours(g)
    for lo, hi in zip(E2M1_VALUES[:-1], E2M1_VALUES[1:]):
        vals += neighbours((lo + hi) / 2)
    vals += [f32(6.5), f32(7.0), f32(1e30), f32(3.4e38), f32(1e-30), f32(1e-45), f32(0.1), f32(0.26)]
    rng = np.random.default_rng(7)
    vals += list(rng.uniform(0, 7, 2000).astype(np.float32))
    vals += list((rng.standard_normal(2000) * 2).astype(np.float32))
    return [f32(s * v) for v in vals for s in (1, -1)]


def test_e2m1_rne_matches_bruteforce_nearest_with_even_ties():
    for v in e2m1_probe_values():
        assert oracle.e2m1_encode_rne(float(v)) == brute_e2m1_rne(v), float(v)


def test_e2m1_rne_tie_table_and_saturation():
    # midpoints listed with the value they must reach (mantissa-even neighbour)
    ties = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    for mid, want in ties.items():
        assert oracle.e2m1_decode(oracle.e2m1_encode_rne(mid)) == want
        assert oracle.e2m1_decode(oracle.e2m1_encode_rne(-mid)) == -want
    for big in (6.0, 6.0000005, 6.4, 100.0, 3e38):
        assert oracle.e2m1_encode_rne(big) == 7 and oracle.e2m1_encode_rne(-big) == 15


def test_e2m1_codes_roundtrip_and_negative_zero():
    for code in range(16):
        assert oracle.e2m1_encode_rne(oracle.e2m1_decode(code)) == code
    assert oracle.e2m1_encode_rne(-0.0) == 8
    assert oracle.e2m1_encode_rne(-0.1) == 8      # rounds to zero, keeps its sign bit


# ---------------------------------------------------------------- E4M3

def torch_e4m3_decode_table():
    codes = torch.arange(0, 127, dtype=torch.uint8)
    return codes.view(torch.float8_e4m3fn).to(torch.float32).numpy()


def test_e4m3_decode_matches_torch_and_max_is_448():
    table = torch_e4m3_decode_table()
    for code in range(127):
        assert oracle.e4m3_decode(code) == table[code]
    assert oracle.e4m3_decode(0x7E) == 448.0                       # App. B.1
    assert np.isnan(oracle.e4m3_decode(0x7F))
    assert oracle.e4m3_decode(0x01) == 2.0 ** -9 and oracle.e4m3_decode(0x08) == 2.0 ** -6


def brute_e4m3_rne_sat(u, table):
    a = Fraction(float(u))
    best = None
    for code in range(127):
        d = abs(a - Fraction(float(table[code])))
        if best is None or d < best[0] or (d == best[0] and code % 2 == 0 and best[1] % 2 == 1):
            best = (d, code)
    return best[1]


def test_e4m3_encode_bruteforce_all_codes_midpoints_and_random():
    table = torch_e4m3_decode_table()
    probes = []
    for code in range(127):
        probes += neighbours(table[code])
    for code in range(126):
        probes += neighbours((float(table[code]) + float(table[code + 1])) / 2)
    rng = np.random.default_rng(11)
    probes += list(np.exp(rng.uniform(np.log(1e-4), np.log(460.0), 4000)).astype(np.float32))
    for u in probes:
        if u < 0:
            continue
        assert oracle.e4m3_encode_rne_sat(float(u)) == brute_e4m3_rne_sat(u, table), float(u)


def test_e4m3_encode_matches_torch_cast_below_overflow():
    rng = np.random.default_rng(12)
    u = np.exp(rng.uniform(np.log(1e-4), np.log(447.0), 20000)).astype(np.float32)
    want = torch.from_numpy(u).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode_rne_sat(float(v)) for v in u], dtype=np.uint8)
    assert np.array_equal(got, want)


def test_e4m3_encode_edges():
    assert oracle.e4m3_encode_rne_sat(0.0) == 0
    assert oracle.e4m3_encode_rne_sat(448.0) == 0x7E
    for big in (449.0, 463.9, 464.0, 480.0, 1e9, 3e38):
        assert oracle.e4m3_encode_rne_sat(big) == 0x7E           # saturates, never the NaN code
    assert oracle.e4m3_encode_rne_sat(2.0 ** -10) == 0            # tie between 0 and 2^-9 -> even
    assert oracle.e4m3_encode_rne_sat(float(np.nextafter(f32(2.0 ** -10), f32(1)))) == 1
    assert oracle.e4m3_encode_rne_sat(3 * 2.0 ** -10) == 2        # tie between codes 1 and 2
    assert oracle.e4m3_encode_rne_sat(2.0 ** -6) == 0x08
    assert oracle.e4m3_encode_rne_sat(13.44) == 0x55              # 13
    assert oracle.e4m3_encode_rne_sat(13.5) == 0x56               # tie 13 | 14 -> even code (14)


# ---------------------------------------------------------------- bf16

def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(13)
    x = (rng.standard_normal(5000) * np.exp(rng.uniform(-20, 20, 5000))).astype(np.float32)
    x = np.concatenate([x, np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    got = np.array([oracle.f32_to_bf16_rne(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)
