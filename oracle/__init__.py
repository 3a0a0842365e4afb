"""ctypes front end of the NVFP4 CPU oracle -- TEST INFRASTRUCTURE ONLY.

The arithmetic lives in ``nvfp4_oracle.cpp`` (plain C++, built with
``-ffp-contract=off``); this module only marshals numpy arrays.  It must never be
imported by the product package: only the tests, ``__graft_entry__.smoke()`` and
the ``cpu_baseline`` leg of ``bench.py`` use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nvfp4_oracle.cpp")
_LIB = os.path.join(_HERE, "libnvfp4_oracle.so")

ROW, COL = 0, 1
RNE, SR = 0, 1
BLOCK_1x16, BLOCK_16x16 = 1, 16


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler; returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u32, u64, i64, f32 = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int64, ctypes.c_float
        vp = ctypes.c_void_p
        L.orc_e2m1_decode.restype = f32
        L.orc_e2m1_decode.argtypes = [u32]
        L.orc_e2m1_encode_rne.restype = u32
        L.orc_e2m1_encode_rne.argtypes = [f32]
        L.orc_e2m1_encode_sr.restype = u32
        L.orc_e2m1_encode_sr.argtypes = [f32, u32]
        L.orc_e4m3_decode.restype = f32
        L.orc_e4m3_decode.argtypes = [u32]
        L.orc_e4m3_encode_rne_sat.restype = u32
        L.orc_e4m3_encode_rne_sat.argtypes = [f32]
        L.orc_f32_to_bf16_rne.restype = u32
        L.orc_f32_to_bf16_rne.argtypes = [f32]
        L.orc_philox4x32_10.restype = None
        L.orc_philox4x32_10.argtypes = [vp, vp, vp]
        L.orc_sr_random16.restype = u32
        L.orc_sr_random16.argtypes = [u64, u64, u64]
        L.orc_rht_sign_mask.restype = u32
        L.orc_rht_sign_mask.argtypes = [u64]
        L.orc_rht16_forward.restype = None
        L.orc_rht16_forward.argtypes = [vp, u32]
        L.orc_rht16_inverse.restype = None
        L.orc_rht16_inverse.argtypes = [vp, u32]
        L.orc_rht_signs.restype = ctypes.c_int
        L.orc_rht_signs.argtypes = [u64, ctypes.c_int, vp]
        L.orc_rht_forward_d.restype = ctypes.c_int
        L.orc_rht_forward_d.argtypes = [vp, ctypes.c_int, vp]
        L.orc_rht_inverse_d.restype = ctypes.c_int
        L.orc_rht_inverse_d.argtypes = [vp, ctypes.c_int, vp]
        L.orc_num_threads.restype = ctypes.c_int
        L.orc_quantize.restype = ctypes.c_int
        L.orc_quantize.argtypes = [vp, i64, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_int, u64, u64, vp, vp, vp, vp]
        L.orc_quantize_row_scales.restype = ctypes.c_int
        L.orc_quantize_row_scales.argtypes = [vp, i64, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int, u64, u64, vp, vp, vp]
        L.orc_dequantize_row_scales.restype = ctypes.c_int
        L.orc_dequantize_row_scales.argtypes = [vp, vp, vp, i64, i64, ctypes.c_int, u64, vp]
        L.orc_gemm_f64_row_scales.restype = ctypes.c_int
        L.orc_gemm_f64_row_scales.argtypes = [vp, vp, vp, ctypes.c_int, vp, vp, vp, ctypes.c_int, i64, i64, i64, vp]
        L.orc_dequantize.restype = ctypes.c_int
        L.orc_dequantize.argtypes = [vp, vp, f32, i64, i64, ctypes.c_int, u64, vp]
        gemm_head = [vp, vp, f32, vp, vp, f32]
        L.orc_gemm_f64.restype = ctypes.c_int
        L.orc_gemm_f64.argtypes = gemm_head + [i64, i64, i64, vp]
        L.orc_gemm_f64_entries.restype = ctypes.c_int
        L.orc_gemm_f64_entries.argtypes = gemm_head + [i64, i64, vp, vp, vp]
        L.orc_gemm_f32_blockscaled.restype = ctypes.c_int
        L.orc_gemm_f32_blockscaled.argtypes = gemm_head + [i64, i64, i64, vp]
        # MXFP4 (comparison format)
        L.orc_rht_sign_mask32.restype = u32
        L.orc_rht_sign_mask32.argtypes = [u64]
        L.orc_rht32_forward.restype = None
        L.orc_rht32_forward.argtypes = [vp, u32]
        L.orc_rht32_inverse.restype = None
        L.orc_rht32_inverse.argtypes = [vp, u32]
        L.orc_ue8m0_exponent_round_up.restype = ctypes.c_int
        L.orc_ue8m0_exponent_round_up.argtypes = [f32]
        L.orc_mx_col_random16.restype = u32
        L.orc_mx_col_random16.argtypes = [u64, u64, u64]
        L.orc_mx_quantize.restype = ctypes.c_int
        L.orc_mx_quantize.argtypes = [vp, i64, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int, u64, u64, vp, vp, vp]
        L.orc_mx_dequantize.restype = ctypes.c_int
        L.orc_mx_dequantize.argtypes = [vp, vp, i64, i64, ctypes.c_int, u64, vp]
        L.orc_mx_gemm_f64.restype = ctypes.c_int
        L.orc_mx_gemm_f64.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp]
        L.orc_mx_gemm_f64_entries.restype = ctypes.c_int
        L.orc_mx_gemm_f64_entries.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp, vp]
        _lib = L
    return _lib


def _p(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


# ------------------------------------------------------------------ scalars

def e2m1_decode(code: int) -> float:
    return float(lib().orc_e2m1_decode(code))


def e2m1_encode_rne(v: float) -> int:
    return int(lib().orc_e2m1_encode_rne(v))


def e2m1_encode_sr(v: float, r16: int) -> int:
    return int(lib().orc_e2m1_encode_sr(v, r16))


def e4m3_decode(code: int) -> float:
    return float(lib().orc_e4m3_decode(code))


def e4m3_encode_rne_sat(u: float) -> int:
    return int(lib().orc_e4m3_encode_rne_sat(u))


def f32_to_bf16_rne(f: float) -> int:
    return int(lib().orc_f32_to_bf16_rne(f))


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def sr_random16(seed: int, i: int, j: int) -> int:
    return int(lib().orc_sr_random16(seed, i, j))


def rht_sign_mask(seed: int) -> int:
    return int(lib().orc_rht_sign_mask(seed))


def rht16_forward(v, mask: int) -> np.ndarray:
    a = np.ascontiguousarray(v, dtype=np.float32).copy()
    assert a.size == 16
    lib().orc_rht16_forward(_p(a), mask)
    return a


def rht16_inverse(v, mask: int) -> np.ndarray:
    a = np.ascontiguousarray(v, dtype=np.float32).copy()
    assert a.size == 16
    lib().orc_rht16_inverse(_p(a), mask)
    return a


def rht_signs(seed: int, d: int) -> np.ndarray:
    """1 where the sign diagonal of the d-point rotation negates (d in 2, 4, 16, 32, 128)."""
    neg = np.zeros(d, dtype=np.uint8)
    if lib().orc_rht_signs(seed, d, _p(neg)) != 0:
        raise ValueError(f"no rotation of size {d}")
    return neg


def rht_forward(v, negate: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(v, dtype=np.float32).copy()
    neg = np.ascontiguousarray(negate, dtype=np.uint8)
    assert a.size == neg.size
    if lib().orc_rht_forward_d(_p(a), a.size, _p(neg)) != 0:
        raise ValueError(f"no rotation of size {a.size}")
    return a


def rht_inverse(v, negate: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(v, dtype=np.float32).copy()
    neg = np.ascontiguousarray(negate, dtype=np.uint8)
    assert a.size == neg.size
    if lib().orc_rht_inverse_d(_p(a), a.size, _p(neg)) != 0:
        raise ValueError(f"no rotation of size {a.size}")
    return a


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ------------------------------------------------------------------ tensors

class QCopy:
    """One quantized copy: codes [outer, inner/2] u8, scales [outer, inner/16] u8.  s_dec and amax are binary32
    scalars, or float32 arrays [outer] for a copy quantized with one tensor-level scale per row (per_row)."""

    def __init__(self, codes, scales, s_dec, amax, outer, inner, per_row=False):
        self.codes, self.scales = codes, scales
        self.s_dec, self.amax = s_dec, amax
        self.outer, self.inner = outer, inner
        self.per_row = per_row


def quantize(x_bf16_bits: np.ndarray, copy: int, block_dim: int = BLOCK_1x16, rounding: int = RNE,
             use_rht: bool = False, rht_seed: int = 0, sr_seed: int = 0, rht_dim: int = 16, amax=None) -> QCopy:
    """x_bf16_bits: uint16 [rows, cols] holding bf16 bit patterns; rht_dim is the rotation size if use_rht;
    amax: None, or the amax to use for the tensor-level scale instead of the tensor's own."""
    x = np.ascontiguousarray(x_bf16_bits, dtype=np.uint16)
    rows, cols = x.shape
    outer, inner = (cols, rows) if copy == COL else (rows, cols)
    codes = np.zeros((outer, inner // 2), dtype=np.uint8)
    scales = np.zeros((outer, inner // 16), dtype=np.uint8)
    ts = np.zeros(2, dtype=np.float32)
    given = None if amax is None else np.array([amax], dtype=np.float32)
    rc = lib().orc_quantize(_p(x), rows, cols, cols, copy, block_dim, rounding, rht_dim if use_rht else 0,
                            rht_seed, sr_seed, None if given is None else _p(given), _p(codes), _p(scales), _p(ts))
    if rc != 0:
        raise ValueError(f"orc_quantize rejected its arguments (rc={rc})")
    return QCopy(codes, scales, np.float32(ts[0]), np.float32(ts[1]), outer, inner)


def quantize_row_scales(x_bf16_bits: np.ndarray, copy: int, rounding: int = RNE, use_rht: bool = False,
                        rht_seed: int = 0, sr_seed: int = 0, rht_dim: int = 16) -> QCopy:
    """1x16 blocks with one FP32 tensor-level scale per row of the copy (per logical row for ROW, per logical
    column for COL) instead of one per tensor (App. B.1, last sentence)."""
    x = np.ascontiguousarray(x_bf16_bits, dtype=np.uint16)
    rows, cols = x.shape
    outer, inner = (cols, rows) if copy == COL else (rows, cols)
    codes = np.zeros((outer, inner // 2), dtype=np.uint8)
    scales = np.zeros((outer, inner // 16), dtype=np.uint8)
    ts = np.zeros(2 * outer, dtype=np.float32)
    rc = lib().orc_quantize_row_scales(_p(x), rows, cols, cols, copy, rounding, rht_dim if use_rht else 0, rht_seed,
                                       sr_seed, _p(codes), _p(scales), _p(ts))
    if rc != 0:
        raise ValueError(f"orc_quantize_row_scales rejected its arguments (rc={rc})")
    return QCopy(codes, scales, ts[:outer].copy(), ts[outer:].copy(), outer, inner, per_row=True)


def _sdec_array(q: QCopy) -> np.ndarray:
    return np.ascontiguousarray(q.s_dec, dtype=np.float32).reshape(-1)


def dequantize(q: QCopy, undo_rht: bool = False, rht_seed: int = 0, rht_dim: int = 16) -> np.ndarray:
    out = np.zeros((q.outer, q.inner), dtype=np.float32)
    if q.per_row:
        sd = _sdec_array(q)
        rc = lib().orc_dequantize_row_scales(_p(q.codes), _p(q.scales), _p(sd), q.outer, q.inner,
                                             rht_dim if undo_rht else 0, rht_seed, _p(out))
        if rc != 0:
            raise ValueError("orc_dequantize_row_scales rejected its arguments")
        return out
    rc = lib().orc_dequantize(_p(q.codes), _p(q.scales), float(q.s_dec), q.outer, q.inner,
                              rht_dim if undo_rht else 0, rht_seed, _p(out))
    if rc != 0:
        raise ValueError("orc_dequantize rejected its arguments")
    return out


def _gemm_head(a: QCopy, b: QCopy):
    assert a.inner == b.inner, "operands must share K"
    return [_p(a.codes), _p(a.scales), float(a.s_dec), _p(b.codes), _p(b.scales), float(b.s_dec)]


def gemm_f64(a: QCopy, b: QCopy, d_prev=None) -> np.ndarray:
    """Eq. 5 on the dequantized operands in binary64.  With d_prev (the FP32 gradient buffer of Sec. 4.1's
    micro-batch accumulation) the result is d_prev + product, still in binary64."""
    out = np.zeros((a.outer, b.outer), dtype=np.float64)
    if a.per_row or b.per_row:
        assert a.inner == b.inner, "operands must share K"
        sa, sb = _sdec_array(a), _sdec_array(b)
        rc = lib().orc_gemm_f64_row_scales(_p(a.codes), _p(a.scales), _p(sa), int(a.per_row), _p(b.codes), _p(b.scales),
                                           _p(sb), int(b.per_row), a.outer, b.outer, a.inner, _p(out))
    else:
        rc = lib().orc_gemm_f64(*_gemm_head(a, b), a.outer, b.outer, a.inner, _p(out))
    assert rc == 0
    if d_prev is not None:
        assert d_prev.shape == out.shape and d_prev.dtype == np.float32
        out = d_prev.astype(np.float64) + out
    return out


def gemm_f64_entries(a: QCopy, b: QCopy, m_idx, n_idx) -> np.ndarray:
    m = np.ascontiguousarray(m_idx, dtype=np.int64)
    n = np.ascontiguousarray(n_idx, dtype=np.int64)
    assert m.shape == n.shape
    out = np.zeros(m.size, dtype=np.float64)
    rc = lib().orc_gemm_f64_entries(*_gemm_head(a, b), a.inner, m.size, _p(m), _p(n), _p(out))
    assert rc == 0
    return out.reshape(m.shape)


def gemm_f32_blockscaled(a: QCopy, b: QCopy) -> np.ndarray:
    out = np.zeros((a.outer, b.outer), dtype=np.float32)
    rc = lib().orc_gemm_f32_blockscaled(*_gemm_head(a, b), a.outer, b.outer, a.inner, _p(out))
    assert rc == 0
    return out


# ------------------------------------------------------------------ MXFP4 (comparison format, Sec. 2 / App. B.4)

def rht_sign_mask32(seed: int) -> int:
    return int(lib().orc_rht_sign_mask32(seed))


def rht32_forward(v, mask: int) -> np.ndarray:
    a = np.ascontiguousarray(v, dtype=np.float32).copy()
    assert a.size == 32
    lib().orc_rht32_forward(_p(a), mask)
    return a


def rht32_inverse(v, mask: int) -> np.ndarray:
    a = np.ascontiguousarray(v, dtype=np.float32).copy()
    assert a.size == 32
    lib().orc_rht32_inverse(_p(a), mask)
    return a


def ue8m0_exponent_round_up(s: float) -> int:
    return int(lib().orc_ue8m0_exponent_round_up(s))


def mx_col_random16(seed: int, i: int, j: int) -> int:
    return int(lib().orc_mx_col_random16(seed, i, j))


def mx_quantize(x_bf16_bits: np.ndarray, copy: int, rounding: int = RNE, use_rht: bool = False, rht_seed: int = 0,
                sr_seed: int = 0) -> QCopy:
    """MXFP4: codes [outer, inner/2], UE8M0 scales [outer, inner/32]; s_dec is 1 (there is no tensor scale)."""
    x = np.ascontiguousarray(x_bf16_bits, dtype=np.uint16)
    rows, cols = x.shape
    outer, inner = (cols, rows) if copy == COL else (rows, cols)
    codes = np.zeros((outer, inner // 2), dtype=np.uint8)
    scales = np.zeros((outer, max(inner // 32, 1)), dtype=np.uint8)
    amax = np.zeros(1, dtype=np.float32)
    rc = lib().orc_mx_quantize(_p(x), rows, cols, cols, copy, rounding, int(use_rht), rht_seed, sr_seed, _p(codes),
                               _p(scales), _p(amax))
    if rc != 0:
        raise ValueError(f"orc_mx_quantize rejected its arguments (rc={rc})")
    return QCopy(codes, scales, np.float32(1.0), np.float32(amax[0]), outer, inner)


def mx_dequantize(q: QCopy, undo_rht: bool = False, rht_seed: int = 0) -> np.ndarray:
    out = np.zeros((q.outer, q.inner), dtype=np.float32)
    rc = lib().orc_mx_dequantize(_p(q.codes), _p(q.scales), q.outer, q.inner, int(undo_rht), rht_seed, _p(out))
    assert rc == 0
    return out


def mx_gemm_f64(a: QCopy, b: QCopy) -> np.ndarray:
    assert a.inner == b.inner
    out = np.zeros((a.outer, b.outer), dtype=np.float64)
    rc = lib().orc_mx_gemm_f64(_p(a.codes), _p(a.scales), _p(b.codes), _p(b.scales), a.outer, b.outer, a.inner, _p(out))
    assert rc == 0
    return out


def mx_gemm_f64_entries(a: QCopy, b: QCopy, m_idx, n_idx) -> np.ndarray:
    m = np.ascontiguousarray(m_idx, dtype=np.int64)
    n = np.ascontiguousarray(n_idx, dtype=np.int64)
    out = np.zeros(m.size, dtype=np.float64)
    rc = lib().orc_mx_gemm_f64_entries(_p(a.codes), _p(a.scales), _p(b.codes), _p(b.scales), a.inner, m.size, _p(m),
                                       _p(n), _p(out))
    assert rc == 0
    return out.reshape(m.shape)
