"""Thin Python binding of the NVFP4 C ABI (include/nvfp4.h).

Argument marshalling only: every step of the path runs in the HIP kernels of
``libnvfp4_hip.so``.  PyTorch supplies device memory and the current stream.
There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libnvfp4_hip.so")

LAYOUT_ROW, LAYOUT_COL = 1, 2
LAYOUT_ROW_RHT = 4   # with LAYOUT_ROW: the row copy is rotated too (16-point, along its columns)
LAYOUT_ROW_SCALES = 8   # one tensor-level scale per row of each copy; tensor scales are float[2 * outer]
BLOCK_1x16, BLOCK_16x16, BLOCK_MX32 = 1, 16, 32
ROUND_RNE, ROUND_SR = 0, 1
OP_FPROP, OP_DGRAD, OP_WGRAD = 0, 1, 2
OUT_F32, OUT_BF16, OUT_F32_ACCUMULATE = 0, 1, 2
COPY_ROW, COPY_COL = 0, 1

EXPORTS = ["nvfp4_quantized_sizes", "nvfp4_quantize", "nvfp4_gemm", "nvfp4_gemm_workspace_bytes", "nvfp4_dequantize",
           "nvfp4_rht_sign_mask", "nvfp4_selftest_conversions", "nvfp4_status_string", "nvfp4_version",
           "nvfp4_linear_workspace_bytes", "nvfp4_linear_forward", "nvfp4_linear_backward",
           "nvfp4_amax", "nvfp4_quantize_with_amax", "nvfp4_quantize_static", "nvfp4_predecode"]
STATIC_SCRATCH_BYTES = 1 << 20


class QTensorStruct(ctypes.Structure):
    """Mirror of ``nvfp4_qtensor``."""
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("row_codes", ctypes.c_void_p), ("row_scales", ctypes.c_void_p),
                ("row_tensor_scale", ctypes.c_void_p),
                ("col_codes", ctypes.c_void_p), ("col_scales", ctypes.c_void_p),
                ("col_tensor_scale", ctypes.c_void_p),
                ("layout_mask", ctypes.c_int32), ("block_dim", ctypes.c_int32),
                ("rounding", ctypes.c_int32), ("col_has_rht", ctypes.c_int32),
                ("rht_seed", ctypes.c_uint64), ("row_has_rht", ctypes.c_int32), ("scale_per_row", ctypes.c_int32),
                ("row_fp16", ctypes.c_void_p), ("col_fp16", ctypes.c_void_p)]


_lib = None


def load_library() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        i64, vp, ci, u64 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64
        L.nvfp4_quantized_sizes.restype = ci
        L.nvfp4_quantized_sizes.argtypes = [i64, i64, vp, vp, vp]
        L.nvfp4_quantize.restype = ci
        L.nvfp4_quantize.argtypes = [vp, i64, i64, i64, ci, ci, ci, ci, u64, u64,
                                     ctypes.POINTER(QTensorStruct), vp, ctypes.c_size_t, vp]
        L.nvfp4_quantize_static.restype = ci
        L.nvfp4_quantize_static.argtypes = [vp, i64, i64, i64, ci, ci, ci, ci, u64, u64, ctypes.POINTER(QTensorStruct), vp]
        L.nvfp4_amax.restype = ci
        L.nvfp4_amax.argtypes = [vp, i64, i64, i64, ci, u64, vp, vp, ctypes.c_size_t, vp]
        L.nvfp4_quantize_with_amax.restype = ci
        L.nvfp4_quantize_with_amax.argtypes = [vp, i64, i64, i64, ci, ci, ci, ci, u64, u64, vp,
                                               ctypes.POINTER(QTensorStruct), vp]
        L.nvfp4_gemm.restype = ci
        L.nvfp4_gemm.argtypes = [ctypes.POINTER(QTensorStruct), ctypes.POINTER(QTensorStruct), ci, vp, ci, i64,
                                 vp, ctypes.c_size_t, vp]
        L.nvfp4_predecode.restype = ci
        L.nvfp4_predecode.argtypes = [ctypes.POINTER(QTensorStruct), ci, vp, ctypes.c_size_t, vp]
        L.nvfp4_gemm_workspace_bytes.restype = ci
        L.nvfp4_gemm_workspace_bytes.argtypes = [i64, i64, i64, vp]
        qp = ctypes.POINTER(QTensorStruct)
        L.nvfp4_linear_workspace_bytes.restype = ci
        L.nvfp4_linear_workspace_bytes.argtypes = [i64, i64, i64, vp]
        L.nvfp4_linear_forward.restype = ci
        L.nvfp4_linear_forward.argtypes = [vp, i64, i64, i64, qp, ci, u64, qp, vp, ci, i64, vp, ctypes.c_size_t, vp]
        L.nvfp4_linear_backward.restype = ci
        L.nvfp4_linear_backward.argtypes = [vp, i64, i64, i64, qp, qp, u64, qp, vp, ci, i64, vp, i64, ci,
                                            vp, ctypes.c_size_t, vp]
        L.nvfp4_dequantize.restype = ci
        L.nvfp4_dequantize.argtypes = [ctypes.POINTER(QTensorStruct), ci, ci, vp, ci, i64, vp]
        L.nvfp4_rht_sign_mask.restype = ctypes.c_uint32
        L.nvfp4_rht_sign_mask.argtypes = [u64]
        L.nvfp4_selftest_conversions.restype = ci
        L.nvfp4_selftest_conversions.argtypes = [vp, vp]
        L.nvfp4_status_string.restype = ctypes.c_char_p
        L.nvfp4_status_string.argtypes = [ci]
        L.nvfp4_version.restype = ci
        L.nvfp4_version.argtypes = []
        _lib = L
    return _lib


class NVFP4Error(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"nvfp4 error {status}: {load_library().nvfp4_status_string(status).decode()}")


def _check(status: int) -> None:
    if status != 0:
        raise NVFP4Error(status)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def quantized_sizes(rows: int, cols: int):
    c, s, w = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(load_library().nvfp4_quantized_sizes(rows, cols, ctypes.addressof(c), ctypes.addressof(s),
                                                ctypes.addressof(w)))
    return c.value, s.value, w.value


def rht_sign_mask(seed: int) -> int:
    return int(load_library().nvfp4_rht_sign_mask(seed))


@dataclass
class QTensor:
    """Device buffers of a quantized tensor plus its C descriptor."""
    desc: QTensorStruct
    rows: int
    cols: int
    row_codes: Optional[torch.Tensor] = None
    row_scales: Optional[torch.Tensor] = None
    row_ts: Optional[torch.Tensor] = None
    col_codes: Optional[torch.Tensor] = None
    col_scales: Optional[torch.Tensor] = None
    col_ts: Optional[torch.Tensor] = None
    row_fp16: Optional[torch.Tensor] = None     # decoded copies (nvfp4_predecode); kept alive here while the descriptor points to them
    col_fp16: Optional[torch.Tensor] = None


def alloc_qtensor(rows: int, cols: int, layout_mask: int, device="cuda", block_dim: int = BLOCK_1x16) -> QTensor:
    quantized_sizes(rows, cols)                       # shape check
    blk = 32 if block_dim == BLOCK_MX32 else 16     # elements per scale byte
    per_row = bool(layout_mask & LAYOUT_ROW_SCALES)   # tensor scales: float[2], or s_dec and amax per row of the copy
    q = QTensor(QTensorStruct(), rows, cols)
    q.desc.rows, q.desc.cols = rows, cols
    if layout_mask & LAYOUT_ROW:
        q.row_codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=device)
        q.row_scales = torch.empty((rows, cols // blk), dtype=torch.uint8, device=device)
        q.row_ts = torch.empty(2 * rows if per_row else 2, dtype=torch.float32, device=device)
        q.desc.row_codes, q.desc.row_scales = q.row_codes.data_ptr(), q.row_scales.data_ptr()
        q.desc.row_tensor_scale = q.row_ts.data_ptr()
    if layout_mask & LAYOUT_COL:
        q.col_codes = torch.empty((cols, rows // 2), dtype=torch.uint8, device=device)
        q.col_scales = torch.empty((cols, rows // blk), dtype=torch.uint8, device=device)
        q.col_ts = torch.empty(2 * cols if per_row else 2, dtype=torch.float32, device=device)
        q.desc.col_codes, q.desc.col_scales = q.col_codes.data_ptr(), q.col_scales.data_ptr()
        q.desc.col_tensor_scale = q.col_ts.data_ptr()
    return q


_workspaces = {}


def _workspace(device, nbytes: int) -> torch.Tensor:
    key = (torch.device(device).index or 0, _stream())
    if key not in _workspaces or _workspaces[key].numel() < nbytes:
        _workspaces[key] = torch.empty(max(nbytes, 1 << 16), dtype=torch.uint8, device=device)
    return _workspaces[key]


def nvfp4_quantize(x: torch.Tensor, layout_mask: int, block_dim: int = BLOCK_1x16, rounding: int = ROUND_RNE,
                   rht_on_col=False, rht_seed: int = 0, sr_seed: int = 0,
                   out: Optional[QTensor] = None, workspace: Optional[torch.Tensor] = None) -> QTensor:
    """x: bf16 CUDA tensor [rows, cols] (last dim contiguous).  rht_on_col: False, True (the format's own rotation
    size) or the size itself (2, 4, 16, 32, 128 for NVFP4)."""
    if not x.is_cuda or x.dtype != torch.bfloat16 or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D bf16 CUDA tensor with unit inner stride")
    rows, cols = x.shape
    if out is None:
        out = alloc_qtensor(rows, cols, layout_mask, x.device, block_dim)
    ws = workspace if workspace is not None else _workspace(x.device, quantized_sizes(rows, cols)[2])
    _check(load_library().nvfp4_quantize(x.data_ptr(), rows, cols, x.stride(0), layout_mask, block_dim, rounding,
                                         int(rht_on_col), rht_seed, sr_seed, ctypes.byref(out.desc),
                                         ws.data_ptr(), ws.numel(), _stream()))
    out.row_fp16 = out.col_fp16 = None          # the library cleared the descriptor's pointers: the codes changed
    return out


def nvfp4_quantize_static(x: torch.Tensor, out: QTensor, layout_mask: int, block_dim: int = BLOCK_1x16,
                          rounding: int = ROUND_RNE, rht_on_col=False, rht_seed: int = 0, sr_seed: int = 0) -> QTensor:
    """nvfp4_quantize without a workspace: `out` must be preallocated (alloc_qtensor); nothing is allocated here or in
    the library."""
    if not x.is_cuda or x.dtype != torch.bfloat16 or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D bf16 CUDA tensor with unit inner stride")
    rows, cols = x.shape
    _check(load_library().nvfp4_quantize_static(x.data_ptr(), rows, cols, x.stride(0), layout_mask, block_dim, rounding,
                                                int(rht_on_col), rht_seed, sr_seed, ctypes.byref(out.desc), _stream()))
    return out


def nvfp4_amax(x: torch.Tensor, rht_on_col=False, rht_seed: int = 0, out: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Pass 1 alone: float32 CUDA tensor [2] = (amax of x, amax of the rotated x or 0)."""
    if not x.is_cuda or x.dtype != torch.bfloat16 or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D bf16 CUDA tensor with unit inner stride")
    rows, cols = x.shape
    if out is None:
        out = torch.empty(2, dtype=torch.float32, device=x.device)
    ws = workspace if workspace is not None else _workspace(x.device, quantized_sizes(rows, cols)[2])
    _check(load_library().nvfp4_amax(x.data_ptr(), rows, cols, x.stride(0), int(rht_on_col), rht_seed, out.data_ptr(),
                                     ws.data_ptr(), ws.numel(), _stream()))
    return out


def nvfp4_quantize_with_amax(x: torch.Tensor, amax: torch.Tensor, layout_mask: int, block_dim: int = BLOCK_1x16,
                             rounding: int = ROUND_RNE, rht_on_col=False, rht_seed: int = 0, sr_seed: int = 0,
                             out: Optional[QTensor] = None) -> QTensor:
    """Pass 2 alone: `amax` is a float32 CUDA tensor [2] as nvfp4_amax returns it."""
    if not x.is_cuda or x.dtype != torch.bfloat16 or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D bf16 CUDA tensor with unit inner stride")
    if not amax.is_cuda or amax.dtype != torch.float32 or amax.numel() != 2 or not amax.is_contiguous():
        raise ValueError("amax must be a contiguous float32 CUDA tensor of 2 elements")
    rows, cols = x.shape
    if out is None:
        out = alloc_qtensor(rows, cols, layout_mask, x.device, block_dim)
    _check(load_library().nvfp4_quantize_with_amax(x.data_ptr(), rows, cols, x.stride(0), layout_mask, block_dim, rounding,
                                                   int(rht_on_col), rht_seed, sr_seed, amax.data_ptr(),
                                                   ctypes.byref(out.desc), _stream()))
    return out


def nvfp4_predecode(q: QTensor, which_copy: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Decode one copy to FP16 once; later nvfp4_gemm calls on `q` read it instead of decoding again.  Returns the
    float16 CUDA tensor [outer, K], which `q` keeps alive."""
    outer, inner = (q.cols, q.rows) if which_copy == COPY_COL else (q.rows, q.cols)
    if out is None:
        dev = (q.row_codes if q.row_codes is not None else q.col_codes).device
        out = torch.empty((outer, inner), dtype=torch.float16, device=dev)
    if not out.is_cuda or out.dtype != torch.float16 or not out.is_contiguous():
        raise ValueError("out must be a contiguous float16 CUDA tensor")
    _check(load_library().nvfp4_predecode(ctypes.byref(q.desc), which_copy, out.data_ptr(), out.numel() * 2, _stream()))
    if which_copy == COPY_COL:
        q.col_fp16 = out
    else:
        q.row_fp16 = out
    return out


def gemm_workspace_bytes(m: int, n: int, k: int) -> int:
    w = ctypes.c_size_t()
    _check(load_library().nvfp4_gemm_workspace_bytes(m, n, k, ctypes.addressof(w)))
    return w.value


def nvfp4_gemm(a: QTensor, b: QTensor, op: int, out_dtype: int = OUT_F32,
               out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """workspace: optional uint8 CUDA tensor of gemm_workspace_bytes(M, N, K) bytes (two-pass route).
    OUT_F32_ACCUMULATE adds into `out` (required, float32)."""
    m = a.cols if op == OP_WGRAD else a.rows
    n = b.rows if op == OP_DGRAD else b.cols
    if out_dtype == OUT_F32_ACCUMULATE and (out is None or out.dtype != torch.float32 or out.shape != (m, n)):
        raise ValueError("OUT_F32_ACCUMULATE needs a float32 `out` of shape (M, N)")
    if out is None:
        dt = torch.float32 if out_dtype == OUT_F32 else torch.bfloat16
        dev = (a.row_codes if a.row_codes is not None else a.col_codes).device
        out = torch.empty((m, n), dtype=dt, device=dev)
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel()) if workspace is not None else (None, 0)
    _check(load_library().nvfp4_gemm(ctypes.byref(a.desc), ctypes.byref(b.desc), op, out.data_ptr(), out_dtype,
                                     out.stride(0), ws_ptr, ws_bytes, _stream()))
    return out


def linear_workspace_bytes(tokens: int, d_in: int, d_out: int) -> int:
    w = ctypes.c_size_t()
    _check(load_library().nvfp4_linear_workspace_bytes(tokens, d_in, d_out, ctypes.addressof(w)))
    return w.value


def _check_bf16_2d(t: torch.Tensor, what: str) -> None:
    if not t.is_cuda or t.dtype != torch.bfloat16 or t.dim() != 2 or t.stride(1) != 1:
        raise ValueError(f"{what} must be a 2-D bf16 CUDA tensor with unit inner stride")


def nvfp4_linear_forward(x: torch.Tensor, qw: QTensor, workspace: torch.Tensor, keep_for_backward: bool = True,
                         rht_seed: int = 0, out_dtype: int = OUT_BF16, qx: Optional[QTensor] = None,
                         y: Optional[torch.Tensor] = None):
    """Returns (y, qx); qx feeds nvfp4_linear_backward."""
    _check_bf16_2d(x, "x")
    tokens, d_in = x.shape
    if qx is None:
        qx = alloc_qtensor(tokens, d_in, LAYOUT_ROW | (LAYOUT_COL if keep_for_backward else 0), x.device)
    if y is None:
        y = torch.empty((tokens, qw.cols), dtype=torch.float32 if out_dtype == OUT_F32 else torch.bfloat16,
                        device=x.device)
    _check(load_library().nvfp4_linear_forward(x.data_ptr(), tokens, d_in, x.stride(0), ctypes.byref(qw.desc),
                                               int(keep_for_backward), rht_seed, ctypes.byref(qx.desc), y.data_ptr(),
                                               out_dtype, y.stride(0), workspace.data_ptr(), workspace.numel(),
                                               _stream()))
    return y, qx


def nvfp4_linear_backward(dy: torch.Tensor, qx: QTensor, qw: QTensor, dw: torch.Tensor, workspace: torch.Tensor,
                          accumulate_dw: bool = True, sr_seed: int = 0, dx_dtype: int = OUT_BF16,
                          qdy: Optional[QTensor] = None, dx: Optional[torch.Tensor] = None):
    """dw: float32 [d_in, d_out], added into when accumulate_dw.  Returns (dx, qdy)."""
    _check_bf16_2d(dy, "dy")
    tokens, d_out = dy.shape
    if dw.dtype != torch.float32 or dw.shape != (qx.cols, d_out) or dw.stride(1) != 1:
        raise ValueError("dw must be float32 [d_in, d_out] with unit inner stride")
    if qdy is None:
        qdy = alloc_qtensor(tokens, d_out, LAYOUT_ROW | LAYOUT_COL, dy.device)
    if dx is None:
        dx = torch.empty((tokens, qx.cols), dtype=torch.float32 if dx_dtype == OUT_F32 else torch.bfloat16,
                         device=dy.device)
    _check(load_library().nvfp4_linear_backward(dy.data_ptr(), tokens, d_out, dy.stride(0), ctypes.byref(qx.desc),
                                                ctypes.byref(qw.desc), sr_seed, ctypes.byref(qdy.desc), dx.data_ptr(),
                                                dx_dtype, dx.stride(0), dw.data_ptr(), dw.stride(0),
                                                int(accumulate_dw), workspace.data_ptr(), workspace.numel(), _stream()))
    return dx, qdy


def nvfp4_dequantize(q: QTensor, which_copy: int, undo_rht: bool = False, out_dtype: int = OUT_F32,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
    outer, inner = (q.cols, q.rows) if which_copy == COPY_COL else (q.rows, q.cols)
    if out is None:
        dt = torch.float32 if out_dtype == OUT_F32 else torch.bfloat16
        dev = (q.row_codes if q.row_codes is not None else q.col_codes).device
        out = torch.empty((outer, inner), dtype=dt, device=dev)
    _check(load_library().nvfp4_dequantize(ctypes.byref(q.desc), which_copy, int(undo_rht), out.data_ptr(),
                                           out_dtype, out.stride(0), _stream()))
    return out


def nvfp4_selftest_conversions() -> list:
    counts = torch.zeros(5, dtype=torch.int64, device="cuda")
    _check(load_library().nvfp4_selftest_conversions(counts.data_ptr(), _stream()))
    torch.cuda.synchronize()
    return [int(v) for v in counts.cpu()]
