"""nvfp4_quantize_static -- the entry point that allocates nothing (its scratch is a fixed device array inside the
library) -- against nvfp4_quantize with a caller's workspace: same kernels, so every output byte must agree.  Two
calls in a row, the second on a smaller tensor (the array keeps the first call's contents), then a third, larger
again; every rounding / rotation / block mode once.  Collected last on purpose."""
import numpy as np
import pytest
import torch

from paper_2509_25149_amd import binding as nv, synth

pytestmark = pytest.mark.gpu
RC = nv.LAYOUT_ROW | nv.LAYOUT_COL


def to_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def same(a: nv.QTensor, b: nv.QTensor):
    torch.cuda.synchronize()
    for name in ("row_codes", "row_scales", "row_ts", "col_codes", "col_scales", "col_ts"):
        ta, tb = getattr(a, name), getattr(b, name)
        assert (ta is None) == (tb is None), name
        if ta is not None:
            assert torch.equal(ta.view(torch.uint8), tb.view(torch.uint8)), name
    for f in ("rows", "cols", "layout_mask", "block_dim", "rounding", "col_has_rht", "row_has_rht", "rht_seed"):
        assert getattr(a.desc, f) == getattr(b.desc, f), f


MODES = [dict(layout_mask=RC, rounding=nv.ROUND_SR, rht_on_col=True, rht_seed=11, sr_seed=99),     # gradient
         dict(layout_mask=RC, rht_on_col=True, rht_seed=11),                                      # activation
         dict(layout_mask=RC, block_dim=nv.BLOCK_16x16),                                          # weight
         dict(layout_mask=RC, rht_on_col=128, rht_seed=5),                                        # wide rotation
         dict(layout_mask=RC | nv.LAYOUT_ROW_RHT, rht_on_col=16, rht_seed=5, rounding=nv.ROUND_SR, sr_seed=3),
         dict(layout_mask=nv.LAYOUT_ROW),
         dict(layout_mask=RC, block_dim=nv.BLOCK_MX32, rht_on_col=True, rht_seed=4)]              # MXFP4: no scratch at all


@pytest.mark.parametrize("mode", MODES, ids=lambda m: "-".join(f"{k}{v}" for k, v in m.items()))
def test_static_scratch_quantize_equals_quantize(mode):
    kw = dict(mode)
    layout = kw.pop("layout_mask")
    bd = kw.get("block_dim", nv.BLOCK_1x16)
    for i, (rows, cols) in enumerate(((1152, 2080), (256, 544), (2048, 1024))):    # big, smaller, big again
        xb = synth.student_t3(rows, cols, 0.02, 700 + i)
        x = to_dev(xb)
        want = nv.nvfp4_quantize(x, layout, **kw)
        got = nv.alloc_qtensor(rows, cols, layout, block_dim=bd)
        for t in (got.row_codes, got.row_scales, got.col_codes, got.col_scales):
            if t is not None:
                t.fill_(0xEE)
        nv.nvfp4_quantize_static(x, got, layout, **kw)
        same(got, want)


def test_static_scratch_at_a_benchmark_shape_and_its_limit():
    rows, cols = 8192, 20480                                     # the largest tensor of the 12B layer: 30.7 KiB of scratch
    assert nv.quantized_sizes(rows, cols)[2] <= nv.STATIC_SCRATCH_BYTES
    x = to_dev(synth.student_t3(rows, cols, 1e-3, 401))
    want = nv.nvfp4_quantize(x, RC, rounding=nv.ROUND_SR, rht_on_col=True, rht_seed=2025, sr_seed=7)
    got = nv.alloc_qtensor(rows, cols, RC)
    nv.nvfp4_quantize_static(x, got, RC, rounding=nv.ROUND_SR, rht_on_col=True, rht_seed=2025, sr_seed=7)
    same(got, want)
    small = to_dev(synth.normal(128, 512, 1.0, 9))               # and straight after it a one-workgroup tensor
    got2 = nv.alloc_qtensor(128, 512, RC)
    nv.nvfp4_quantize_static(small, got2, RC)
    same(got2, nv.nvfp4_quantize(small, RC))
    # a shape whose workspace need exceeds the fixed array is refused before anything is touched
    import ctypes
    lib = nv.load_library()
    big_rows, big_cols = 128 * 300, 512 * 300
    assert nv.quantized_sizes(big_rows, big_cols)[2] > nv.STATIC_SCRATCH_BYTES
    d = nv.QTensorStruct()
    assert lib.nvfp4_quantize_static(x.data_ptr(), big_rows, big_cols, big_cols, 1, 1, 0, 0, 0, 0, ctypes.byref(d), None) == -6
