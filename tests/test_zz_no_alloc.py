"""The entry point that allocates nothing (fp4_quantize_noalloc) against fp4_quantize, through the C ABI:
bit-identical codes and scales on two calls in a row, the second on a smaller input (the built-in
scratch keeps the first call's contents), then a larger one again; sizes beyond the built-in scratch
are refused before anything is enqueued."""
import ctypes as C

import pytest
import torch

from paper_2501_17116_amd import binding as b
from paper_2501_17116_amd import synth

pytestmark = pytest.mark.gpu


def _both(rows, cols, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(rows, cols, generator=g) * 0.02 * torch.exp(torch.randn(1, cols, generator=g))
    x = synth._finish(x, dtype)
    xd = (x.to(torch.bfloat16) if dtype == "bf16" else x).contiguous().cuda()
    out = {}
    for axis in (b.FP4_AXIS_COL, b.FP4_AXIS_ROW):
        ref_codes, ref_gamma = b.fp4_quantize(xd, axis)
        shape = (cols, rows // 2) if axis == b.FP4_AXIS_COL else (rows, cols // 2)
        codes = torch.full(shape, 0xEE, dtype=torch.uint8, device="cuda")
        gamma = torch.full((cols if axis == b.FP4_AXIS_COL else rows,), -1.0, dtype=torch.float32, device="cuda")
        P = lambda t: C.c_void_p(t.data_ptr())
        st = b.lib().fp4_quantize_noalloc(P(xd), b._dt(xd), rows, cols, cols, axis, P(codes), P(gamma), b._stream())
        assert st == 0, b.status_string(st)
        torch.cuda.synchronize()
        assert torch.equal(codes, ref_codes), (rows, cols, dtype, axis)
        assert torch.equal(gamma.view(torch.int32), ref_gamma.view(torch.int32)), (rows, cols, dtype, axis)
        out[axis] = (codes, gamma)
    return out


def test_noalloc_equals_fp4_quantize_on_consecutive_calls():
    _both(2048, 1032, "bf16", 1)      # several row blocks of partial maxima, ragged column tile
    _both(300, 136, "f32", 2)         # smaller: must not see what the first call left in the scratch
    _both(4096, 4096, "bf16", 3)      # larger again


def test_noalloc_refuses_what_does_not_fit_and_bad_arguments():
    one = C.c_void_p(16)
    L = b.lib()
    # ceil(rows / 128) * cols words > 8 MiB / 4: refused on the host, nothing enqueued
    assert L.fp4_quantize_noalloc(one, 1, 1 << 20, 4096, 4096, b.FP4_AXIS_COL, one, one, None) == -8
    assert "scratch" in b.status_string(-8)
    assert L.fp4_quantize_noalloc(None, 1, 256, 64, 64, b.FP4_AXIS_COL, one, one, None) == -1
    assert L.fp4_quantize_noalloc(one, 1, 255, 64, 64, b.FP4_AXIS_COL, one, one, None) == -2
    assert L.fp4_quantize_noalloc(one, 1, 0, 64, 64, b.FP4_AXIS_COL, one, one, None) == 0
