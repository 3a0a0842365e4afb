"""CPU-only checks of the C ABI: the library loads, exports every declared symbol,
and rejects bad arguments synchronously (no kernel is ever enqueued here)."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2509_25149_amd import binding as nv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(nv.LIB_PATH):
        from paper_2509_25149_amd import build
        build.build_library()
    return nv.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "nvfp4.h")).read()
    declared = set(re.findall(r"\b(nvfp4_[a-z0-9_]+)\s*\(", header))
    assert declared == set(nv.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.nvfp4_version() >= 100


def test_struct_layout_matches_header(tmp_path):
    # the C compiler's view of the descriptor in include/nvfp4.h against the ctypes mirror, field by field
    fields = [f[0] for f in nv.QTensorStruct._fields_]
    c_names = {"row_tensor_scale": "row_tensor_scale", "col_tensor_scale": "col_tensor_scale"}
    src = tmp_path / "layout.c"
    src.write_text('#include <stddef.h>\n#include <stdio.h>\n#include "nvfp4.h"\nint main(void) {\n'
                   '  printf("%zu\\n", sizeof(nvfp4_qtensor));\n' +
                   "".join(f'  printf("%zu\\n", offsetof(nvfp4_qtensor, {c_names.get(f, f)}));\n' for f in fields) +
                   "  return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert out[0] == ctypes.sizeof(nv.QTensorStruct)
    assert out[1:] == [getattr(nv.QTensorStruct, f).offset for f in fields]
    assert nv.QTensorStruct.rht_seed.offset == 80 and nv.QTensorStruct.row_has_rht.offset == 88
    assert nv.QTensorStruct.scale_per_row.offset == 92 and nv.QTensorStruct.row_fp16.offset == 96
    assert nv.QTensorStruct.col_fp16.offset == 104 and ctypes.sizeof(nv.QTensorStruct) == 112


def test_sizes(lib):
    assert nv.quantized_sizes(256, 512)[:2] == (256 * 512 // 2, 256 * 512 // 16)
    assert 64 <= nv.quantized_sizes(256, 512)[2] <= 8192          # small: a few words per workgroup tile, or per row and column
    assert nv.quantized_sizes(8192, 20480)[2] >= 2 * 40 * 64 * 4
    for bad in ((0, 16), (16, 0), (24, 16), (16, 40), (-16, 16)):
        with pytest.raises(nv.NVFP4Error) as e:
            nv.quantized_sizes(*bad)
        assert e.value.status == -2


def test_status_strings(lib):
    seen = set()
    for s in range(0, -7, -1):
        txt = lib.nvfp4_status_string(s).decode()
        assert txt and txt != "unknown status"
        seen.add(txt)
    assert len(seen) == 7
    assert lib.nvfp4_status_string(-99).decode() == "unknown status"


def _desc(rows=16, cols=16, mask=3, rht=0, seed=0):
    d = nv.QTensorStruct()
    d.rows, d.cols = rows, cols
    for f in ("row_codes", "row_scales", "row_tensor_scale", "col_codes", "col_scales", "col_tensor_scale"):
        setattr(d, f, 0x10000)          # fake, aligned, never dereferenced by the checks below
    d.layout_mask, d.block_dim, d.col_has_rht, d.rht_seed = mask, 1, rht, seed
    return d


def test_quantize_rejects_bad_arguments(lib):
    d = _desc()
    X, WS = 0x20000, 0x30000
    q = lambda *a, **k: lib.nvfp4_quantize(*a)
    ok_tail = (ctypes.byref(d), WS, 256, None)
    assert lib.nvfp4_quantize(None, 16, 16, 16, 1, 1, 0, 0, 0, 0, *ok_tail) == -1
    assert lib.nvfp4_quantize(X, 16, 16, 16, 0, 1, 0, 0, 0, 0, *ok_tail) == -1      # empty layout mask
    assert lib.nvfp4_quantize(X, 16, 16, 16, 4, 1, 0, 0, 0, 0, *ok_tail) == -1      # the row-rotation bit alone
    assert lib.nvfp4_quantize(X, 16, 16, 16, 8, 1, 0, 0, 0, 0, *ok_tail) == -1      # unknown bit
    assert lib.nvfp4_quantize(X, 16, 16, 16, 2 | 4, 1, 0, 16, 0, 0, *ok_tail) == -1  # a rotated row copy needs a row copy,
    assert lib.nvfp4_quantize(X, 16, 16, 16, 1 | 4, 16, 0, 0, 0, 0, *ok_tail) == -1  # 1x16 blocks,
    assert lib.nvfp4_quantize(X, 32, 32, 32, 1 | 4, 32, 0, 0, 0, 0, *ok_tail) == -1  # NVFP4,
    assert lib.nvfp4_quantize(X, 16, 16, 16, 3 | 4, 1, 0, 4, 0, 0, *ok_tail) == -1   # and a col copy plain or rotated by 16
    assert lib.nvfp4_quantize(X, 24, 16, 16, 1 | 4, 1, 0, 0, 0, 0, *ok_tail) == -2   # shapes are checked as ever
    assert lib.nvfp4_quantize_with_amax(X, 16, 16, 16, 1 | 4, 1, 0, 0, 0, 0, WS, ctypes.byref(d), None) == -1
    assert lib.nvfp4_quantize(X, 16, 16, 16, 1, 2, 0, 0, 0, 0, *ok_tail) == -1      # unknown block_dim
    assert lib.nvfp4_quantize(X, 16, 16, 16, 1, 1, 7, 0, 0, 0, *ok_tail) == -1      # unknown rounding
    assert lib.nvfp4_quantize(X, 16, 16, 16, 3, 16, 0, 1, 0, 0, *ok_tail) == -1     # rotation with 16x16 blocks
    assert lib.nvfp4_quantize(X, 16, 16, 16, 1, 1, 0, 1, 0, 0, *ok_tail) == -1      # rotation without a col copy
    for size in (3, 8, 64, 256, -16):                                                # no rotation of these sizes
        assert lib.nvfp4_quantize(X, 256, 16, 16, 2, 1, 0, size, 0, 0, *ok_tail) == -1
    assert lib.nvfp4_quantize(X, 160, 16, 16, 2, 1, 0, 128, 0, 0, *ok_tail) == -2   # rows are not whole rotation groups
    assert lib.nvfp4_quantize(X, 48, 16, 16, 2, 1, 0, 32, 0, 0, *ok_tail) == -2
    assert lib.nvfp4_quantize(X, 24, 16, 16, 1, 1, 0, 0, 0, 0, *ok_tail) == -2
    assert lib.nvfp4_quantize(X, 0, 16, 16, 1, 1, 0, 0, 0, 0, *ok_tail) == -2       # empty tensors are rejected
    assert lib.nvfp4_quantize(X, 16, 0, 16, 1, 1, 0, 0, 0, 0, *ok_tail) == -2
    assert lib.nvfp4_quantize(X, 16, 40, 40, 1, 1, 0, 0, 0, 0, *ok_tail) == -2
    assert lib.nvfp4_quantize(X, 16, 32, 16, 1, 1, 0, 0, 0, 0, *ok_tail) == -2      # ld < cols
    assert lib.nvfp4_quantize(X + 2, 16, 16, 16, 1, 1, 0, 0, 0, 0, *ok_tail) == -1  # misaligned input
    assert lib.nvfp4_quantize(X, 16, 16, 16, 1, 1, 0, 0, 0, 0, ctypes.byref(d), None, 256, None) == -6
    assert lib.nvfp4_quantize(X, 16, 16, 16, 1, 1, 0, 0, 0, 0, ctypes.byref(d), WS, 8, None) == -6
    d2 = _desc()
    d2.col_codes = None
    assert lib.nvfp4_quantize(X, 16, 16, 16, 2, 1, 0, 0, 0, 0, ctypes.byref(d2), WS, 256, None) == -1


def test_gemm_and_dequantize_reject_bad_arguments(lib):
    a, b = _desc(32, 64), _desc(64, 48)
    D = 0x40000
    assert lib.nvfp4_gemm(None, ctypes.byref(b), 0, D, 0, 48, None, 0, None) == -1
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(b), 9, D, 0, 48, None, 0, None) == -1
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(b), 0, D, 5, 48, None, 0, None) == -1
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(b), 0, D, 3, 48, None, 0, None) == -1     # 2 = accumulate is the last mode
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(b), 0, D, 2, 32, None, 0, None) == -2     # accumulate mode is validated like the others
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(b), 0, D, 0, 32, None, 0, None) == -2     # ldd < N
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(b), 1, D, 0, 64, None, 0, None) == -4     # DGRAD: K 64 vs 48
    only_row = _desc(64, 48, mask=1)
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(only_row), 0, D, 0, 48, None, 0, None) == -3
    # WGRAD operands must rotate alike
    p, q = _desc(64, 32, rht=16, seed=5), _desc(64, 48, rht=0)
    assert lib.nvfp4_gemm(ctypes.byref(p), ctypes.byref(q), 2, D, 0, 48, None, 0, None) == -4
    q2 = _desc(64, 48, rht=16, seed=6)
    assert lib.nvfp4_gemm(ctypes.byref(p), ctypes.byref(q2), 2, D, 0, 48, None, 0, None) == -4
    p3, q3 = _desc(128, 32, rht=128, seed=5), _desc(128, 48, rht=32, seed=5)            # same seed, different rotation size
    assert lib.nvfp4_gemm(ctypes.byref(p3), ctypes.byref(q3), 2, D, 0, 48, None, 0, None) == -4
    bad = _desc(128, 32, rht=64, seed=5)                                                # a size that does not exist
    assert lib.nvfp4_dequantize(ctypes.byref(bad), 1, 1, D, 0, 128, None) == -4
    short = _desc(64, 32, rht=128, seed=5)                                              # 64 rows cannot hold a 128-point group
    assert lib.nvfp4_dequantize(ctypes.byref(short), 1, 1, D, 0, 64, None) == -4
    # Fprop / Dgrad read row copies: a rotated row copy needs its partner rotated alike
    xr = _desc(32, 64)
    xr.row_has_rht, xr.rht_seed = 16, 5
    assert lib.nvfp4_gemm(ctypes.byref(xr), ctypes.byref(b), 0, D, 0, 48, None, 0, None) == -4     # B's col copy is plain
    b_other = _desc(64, 48, rht=16, seed=6)
    assert lib.nvfp4_gemm(ctypes.byref(xr), ctypes.byref(b_other), 0, D, 0, 48, None, 0, None) == -4   # other seed
    w_row = _desc(48, 64)
    assert lib.nvfp4_gemm(ctypes.byref(xr), ctypes.byref(w_row), 1, D, 0, 48, None, 0, None) == -4  # Dgrad, W's row copy plain
    assert lib.nvfp4_dequantize(ctypes.byref(a), 3, 0, D, 0, 64, None) == -1
    assert lib.nvfp4_dequantize(ctypes.byref(a), 0, 1, D, 0, 64, None) == -4            # undo_rht on a plain copy
    assert lib.nvfp4_dequantize(ctypes.byref(a), 0, 0, D, 0, 32, None) == -2
    assert lib.nvfp4_dequantize(ctypes.byref(only_row), 1, 0, D, 0, 64, None) == -3


def test_gemm_workspace_query(lib):
    # FP16 copies of both operands (+ FP32 partial tiles when the last round of 256x256 tiles is partial:
    # 640 tiles -> 128 tiles x 2 splits, 1600 tiles -> 64 tiles x 4 splits)
    assert nv.gemm_workspace_bytes(8192, 20480, 5120) == (8192 + 20480) * 5120 * 2
    assert nv.gemm_workspace_bytes(8192, 5120, 20480) == (8192 + 5120) * 20480 * 2 + 256 * 256 * 256 * 4
    assert nv.gemm_workspace_bytes(20480, 5120, 8192) == (20480 + 5120) * 8192 * 2 + 256 * 256 * 256 * 4
    w = ctypes.c_size_t()
    assert lib.nvfp4_gemm_workspace_bytes(8, 16, 16, ctypes.addressof(w)) == -2
    assert lib.nvfp4_gemm_workspace_bytes(16, 16, 16, None) == -1


def test_sign_mask_matches_the_oracle(lib):
    import oracle
    for seed in (0, 1, 2025, 0xDEADBEEFCAFE, 2 ** 64 - 1):
        assert nv.rht_sign_mask(seed) == oracle.rht_sign_mask(seed)


def test_linear_layer_calls_reject_before_enqueueing(lib):
    """The per-layer entry points validate every step first: all of these fail on the host (no GPU here)."""
    w = ctypes.c_size_t()
    assert lib.nvfp4_linear_workspace_bytes(8192, 5120, 20480, ctypes.addressof(w)) == 0
    assert w.value == max(nv.gemm_workspace_bytes(8192, 20480, 5120), nv.gemm_workspace_bytes(8192, 5120, 20480),
                          nv.gemm_workspace_bytes(5120, 20480, 8192))
    assert lib.nvfp4_linear_workspace_bytes(8192, 5120, 20481, ctypes.addressof(w)) == -2
    assert lib.nvfp4_linear_workspace_bytes(16, 16, 16, None) == -1
    qw, qx, qdy = nv.QTensorStruct(), nv.QTensorStruct(), nv.QTensorStruct()
    fake = 0x10000
    for q in (qw, qx, qdy):
        q.row_codes = q.row_scales = q.row_tensor_scale = fake
        q.col_codes = q.col_scales = q.col_tensor_scale = fake
    qw.rows, qw.cols, qw.layout_mask, qw.block_dim = 64, 48, 3, 16
    fwd = lambda *a: lib.nvfp4_linear_forward(*a)
    ok_ws = (fake, 1 << 20, None)
    assert fwd(fake, 32, 64, 64, None, 1, 0, ctypes.byref(qx), fake, 1, 48, *ok_ws) == -1
    assert fwd(fake, 32, 64, 64, ctypes.byref(qw), 1, 0, ctypes.byref(qx), None, 1, 48, *ok_ws) == -1
    assert fwd(fake, 32, 72, 72, ctypes.byref(qw), 1, 0, ctypes.byref(qx), fake, 1, 48, *ok_ws) == -2   # d_in % 16
    assert fwd(fake, 32, 80, 80, ctypes.byref(qw), 1, 0, ctypes.byref(qx), fake, 1, 48, *ok_ws) == -4   # K: 80 vs W's 64
    assert fwd(fake, 32, 64, 64, ctypes.byref(qw), 1, 0, ctypes.byref(qx), fake, 1, 32, *ok_ws) == -2   # ldy < d_out
    assert fwd(fake, 32, 64, 64, ctypes.byref(qw), 1, 0, ctypes.byref(qx), fake, 1, 48, fake, 8, None) == -6
    assert qx.layout_mask == 0                                   # a rejected call leaves the descriptor alone
    bwd = lambda *a: lib.nvfp4_linear_backward(*a)
    qx.rows, qx.cols, qx.layout_mask, qx.block_dim, qx.col_has_rht, qx.rht_seed = 32, 64, 3, 1, 16, 5
    assert bwd(fake, 32, 48, 48, ctypes.byref(qx), ctypes.byref(qw), 0, ctypes.byref(qdy), fake, 7, 64, fake, 48, 1, *ok_ws) == -1
    assert bwd(fake, 32, 48, 48, ctypes.byref(qx), ctypes.byref(qw), 0, ctypes.byref(qdy), fake, 1, 48, fake, 48, 1, *ok_ws) == -2  # lddx < d_in
    assert bwd(fake, 32, 48, 48, ctypes.byref(qx), ctypes.byref(qw), 0, ctypes.byref(qdy), fake, 1, 64, fake, 32, 1, *ok_ws) == -2  # lddw < d_out
    assert bwd(fake, 48, 48, 48, ctypes.byref(qx), ctypes.byref(qw), 0, ctypes.byref(qdy), fake, 1, 64, fake, 48, 1, *ok_ws) == -4  # tokens differ
    qx.col_has_rht = 0
    assert bwd(fake, 32, 48, 48, ctypes.byref(qx), ctypes.byref(qw), 0, ctypes.byref(qdy), fake, 1, 64, fake, 48, 1, *ok_ws) == -3  # no rotated copy kept
    assert qdy.layout_mask == 0


def test_mxfp4_mode_argument_checks(lib):
    """block_dim 32 = MXFP4 (Sec. 2 / App. B.4): whole 32-blocks in both directions, no workspace needed, GEMM needs
    two MXFP4 operands and K a multiple of 128.  All rejected on the host, before anything is enqueued."""
    fake = 0x10000
    q = nv.QTensorStruct()
    q.row_codes = q.row_scales = q.row_tensor_scale = q.col_codes = q.col_scales = q.col_tensor_scale = fake
    qz = lambda rows, cols, ld: lib.nvfp4_quantize(fake, rows, cols, ld, 3, 32, 0, 0, 0, 0, ctypes.byref(q), None, 0, None)
    assert qz(48, 64, 64) == -2 and qz(64, 48, 48) == -2          # 16-multiples are not enough
    assert lib.nvfp4_quantize(fake, 64, 64, 64, 3, 33, 0, 0, 0, 0, ctypes.byref(q), None, 0, None) == -1
    a, b = nv.QTensorStruct(), nv.QTensorStruct()
    for t in (a, b):
        t.row_codes = t.row_scales = t.row_tensor_scale = fake
        t.layout_mask, t.block_dim = 1, 32
    a.rows, a.cols, b.rows, b.cols = 64, 256, 32, 256
    D = fake
    b.block_dim = 1
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(b), 1, D, 0, 32, None, 0, None) == -4      # MXFP4 x NVFP4
    b.block_dim = 32
    a.cols = b.cols = 192
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(b), 1, D, 0, 32, None, 0, None) == -2      # K % 128
    a.cols = b.cols = 256
    a.rows = 48
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(b), 1, D, 0, 32, None, 0, None) == -2      # M % 32
    a.rows = 64
    a.row_scales = fake + 2
    assert lib.nvfp4_gemm(ctypes.byref(a), ctypes.byref(b), 1, D, 0, 32, None, 0, None) == -1      # scale rows are read as dwords
    out = fake
    assert lib.nvfp4_dequantize(ctypes.byref(b), 0, 0, out, 0, 128, None) == -2                    # ld_out < K


def test_separate_passes_reject_bad_arguments(lib):
    """nvfp4_amax / nvfp4_quantize_with_amax validate on the host like nvfp4_quantize (no GPU here)."""
    X, WS, AM = 0x10000, 0x20000, 0x30000
    assert lib.nvfp4_amax(None, 16, 16, 16, 0, 0, AM, WS, 256, None) == -1
    assert lib.nvfp4_amax(X, 16, 16, 16, 0, 0, None, WS, 256, None) == -1
    assert lib.nvfp4_amax(X, 16, 16, 16, 8, 0, AM, WS, 256, None) == -1             # no rotation of size 8
    assert lib.nvfp4_amax(X, 24, 16, 16, 0, 0, AM, WS, 256, None) == -2
    assert lib.nvfp4_amax(X, 48, 16, 16, 32, 0, AM, WS, 256, None) == -2            # 48 rows: no whole groups of 32
    assert lib.nvfp4_amax(X, 16, 16, 16, 0, 0, AM, None, 256, None) == -6
    assert lib.nvfp4_amax(X, 16, 16, 16, 0, 0, AM, WS, 8, None) == -6
    d = _desc()
    tail = (AM, ctypes.byref(d), None)
    assert lib.nvfp4_quantize_with_amax(X, 16, 16, 16, 1, 1, 0, 0, 0, 0, None, ctypes.byref(d), None) == -1   # no amax
    assert lib.nvfp4_quantize_with_amax(X, 32, 32, 32, 1, 32, 0, 0, 0, 0, *tail) == -1                        # MXFP4 has none
    assert lib.nvfp4_quantize_with_amax(X, 16, 16, 16, 0, 1, 0, 0, 0, 0, *tail) == -1
    assert lib.nvfp4_quantize_with_amax(X, 24, 16, 16, 1, 1, 0, 0, 0, 0, *tail) == -2
    assert lib.nvfp4_quantize_with_amax(X, 16, 16, 16, 1, 1, 0, 1, 0, 0, *tail) == -1                         # rotation without a col copy


def test_no_kernel_keeps_arrays_in_scratch_memory():
    """The build records what the compiler reports per kernel.  A patch or fragment array that ends up in scratch
    (private) memory, or register spills reloaded inside a loop, are silent 2-3x slowdowns (both happened here), so:
    no dynamic stack, at most a few spilled values per kernel, none at all in the streaming kernels and in the FP16
    GEMM (whose K steps run behind the stores of the tile before: a reload there would wait for all of them)."""
    import json
    from paper_2509_25149_amd import build
    if not os.path.exists(build.RESOURCES):
        pytest.skip("libnvfp4_hip.resources.json is written by build(); run it first")
    res = json.load(open(build.RESOURCES))
    assert len(res) >= 60
    for name, r in res.items():
        assert r["Dynamic Stack"] == "False", name
        assert r["ScratchSize"] <= 32, (name, r["ScratchSize"])
        if any(k in name for k in ("quantize_mx_kernel", "cast_kernel", "amax_kernel", "cast_wide", "amax_wide", "decode_f16",
                                   "dequantize", "rowscale_", "gemm_f16_kernel")):
            assert r["ScratchSize"] == 0 and r["VGPRs Spill"] == 0, (name, r)
        if "splitk_sum" in name:
            assert r["ScratchSize"] == 0, (name, r)   # (values parked in unused accumulation registers are no memory traffic)
        if "gemm_mx_kernel" in name:
            assert r["ScratchSize"] <= 16 and r["VGPRs Spill"] <= 3, (name, r)     # parked across the loop, not inside it


def test_quantize_static_rejects_before_touching_the_gpu(lib):
    """The entry point that allocates nothing: the size limit and every argument check come before any HIP call."""
    X, OUT = 0x10000, 0x20000
    d = _desc()
    for f in ("row_codes", "row_scales", "row_tensor_scale", "col_codes", "col_scales", "col_tensor_scale"):
        setattr(d, f, OUT)
    tail = (ctypes.byref(d), None)
    assert lib.nvfp4_quantize_static(None, 16, 16, 16, 3, 1, 0, 0, 0, 0, *tail) == -1
    assert lib.nvfp4_quantize_static(X, 24, 16, 16, 3, 1, 0, 0, 0, 0, *tail) == -2
    assert lib.nvfp4_quantize_static(X, 16, 16, 16, 3, 7, 0, 0, 0, 0, *tail) == -1
    assert lib.nvfp4_quantize_static(X, 16, 16, 16, 3, 1, 0, 0, 0, 0, None, None) == -1
    # a workspace need beyond the fixed array (1 MiB): refused, also for MXFP4-sized shapes only when NVFP4
    rows, cols = 128 * 300, 512 * 300
    need = ctypes.c_size_t()
    assert lib.nvfp4_quantized_sizes(rows, cols, None, None, ctypes.addressof(need)) == 0 and need.value > nv.STATIC_SCRATCH_BYTES
    assert lib.nvfp4_quantize_static(X, rows, cols, cols, 3, 1, 0, 0, 0, 0, *tail) == -6
    header = open(os.path.join(ROOT, "include", "nvfp4.h")).read()
    assert "NVFP4_STATIC_SCRATCH_BYTES = 1 << 20" in header and nv.STATIC_SCRATCH_BYTES == 1 << 20


def test_row_scale_mode_argument_checks(lib):
    """NVFP4_LAYOUT_ROW_SCALES (8): 1x16 blocks, rotation 0 / 16, no rotated row copy, no supplied amax."""
    X, OUT, WS = 0x10000, 0x20000, 0x30000
    d = _desc()
    for f in ("row_codes", "row_scales", "row_tensor_scale", "col_codes", "col_scales", "col_tensor_scale"):
        setattr(d, f, OUT)
    tail = (ctypes.byref(d), WS, 1 << 20, None)
    assert lib.nvfp4_quantize(X, 16, 16, 16, 3 | 8, 16, 0, 0, 0, 0, *tail) == -1      # 16x16 blocks
    assert lib.nvfp4_quantize(X, 32, 32, 32, 3 | 8, 32, 0, 0, 0, 0, *tail) == -1      # MXFP4
    assert lib.nvfp4_quantize(X, 16, 16, 16, 3 | 8, 1, 0, 4, 0, 0, *tail) == -1       # 4-point rotation
    assert lib.nvfp4_quantize(X, 16, 16, 16, 1 | 4 | 8, 1, 0, 0, 0, 0, *tail) == -1   # rotated row copy
    assert lib.nvfp4_quantize(X, 16, 16, 16, 8, 1, 0, 0, 0, 0, *tail) == -1           # no copy asked for
    assert lib.nvfp4_quantize(X, 16, 24, 24, 1 | 8, 1, 0, 0, 0, 0, *tail) == -2
    amax = 0x40000
    assert lib.nvfp4_quantize_with_amax(X, 16, 16, 16, 1 | 8, 1, 0, 0, 0, 0, amax, ctypes.byref(d), None) == -1
    # the workspace query covers the per-row mode: amax and encode scale per row and per column
    need = ctypes.c_size_t()
    assert lib.nvfp4_quantized_sizes(8192, 20480, None, None, ctypes.addressof(need)) == 0
    assert need.value >= 2 * (8192 + 20480) * 4
    assert lib.nvfp4_quantize(X, 8192, 20480, 20480, 3 | 8, 1, 0, 0, 0, 0, ctypes.byref(d), WS, need.value - 1, None) == -6


def test_predecode_rejects_bad_arguments(lib):
    OUT, F16 = 0x20000, 0x80000
    d = _desc(rows=32, cols=64, mask=1)
    d.row_codes, d.row_scales, d.row_tensor_scale = OUT, OUT, OUT
    assert lib.nvfp4_predecode(None, 0, F16, 1 << 20, None) == -1
    assert lib.nvfp4_predecode(ctypes.byref(d), 0, None, 1 << 20, None) == -1
    assert lib.nvfp4_predecode(ctypes.byref(d), 2, F16, 1 << 20, None) == -1
    assert lib.nvfp4_predecode(ctypes.byref(d), 0, F16 + 8, 1 << 20, None) == -1          # 16-byte alignment
    assert lib.nvfp4_predecode(ctypes.byref(d), 1, F16, 1 << 20, None) == -3              # no col copy
    assert lib.nvfp4_predecode(ctypes.byref(d), 0, F16, 32 * 64 * 2 - 1, None) == -6      # room for [rows, cols] FP16
    d.block_dim = 32
    assert lib.nvfp4_predecode(ctypes.byref(d), 0, F16, 1 << 20, None) == -1              # MXFP4 is not decoded
    assert d.row_fp16 is None and d.col_fp16 is None                                      # nothing was recorded
