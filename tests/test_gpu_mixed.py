"""GPU parity of the mixed-format path (Sec. 4.3 ablations W4A8 / W8A4): E4M3 codes and scales
bit-exact against the oracle; the mixed GEMM and the mixed forward pass within a tolerance.

Tolerance of the mixed product.  With an 8-bit operand the matrix core does not add exact products:
the 64 products of one instruction are aligned to the largest of them before they are summed and the
low bits of the smaller ones are dropped (measured: up to 6.4e-5 of the sum of the magnitudes on
operands that use every exponent of both formats).  The bar is therefore
    |got - ref| <= 1e-3 |ref| + 1.5e-4 * sum_k |l_k r_k| / (gamma_l gamma_r)
(plus half a bf16 ulp for bf16 outputs): the first term as for every scaled output, the second the
datapath's own bound with a factor 2 in hand."""
MIX_ACC = 1.5e-4

import numpy as np
import pytest
import torch

from oracle import fp4_oracle as o
from paper_2501_17116_amd import binding as b
from paper_2501_17116_amd import synth

pytestmark = pytest.mark.gpu


def dev(x, dtype):
    return (x.to(torch.bfloat16) if dtype == "bf16" else x.to(torch.float32)).contiguous().cuda()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(7, 64), (33, 520), (64, 4096), (5, 9000), (130, 1024), (3, 10)])
def test_fp8_quantize_rows_bit_exact(shape, dtype):
    R, Cc = shape
    g = torch.Generator().manual_seed(R * 100 + Cc)
    ld = (Cc + 7) // 8 * 8
    x = torch.randn(R, ld, generator=g) * torch.exp(torch.randn(R, 1, generator=g) * 3)
    if R > 2:
        x[2] = 0.0
    x = synth._finish(x, dtype)
    xd = dev(x, dtype)
    if ld != Cc:
        import ctypes as C
        codes = torch.empty((R, Cc), dtype=torch.uint8, device="cuda")
        gamma = torch.empty(R, dtype=torch.float32, device="cuda")
        assert b.lib().fp8_quantize(C.c_void_p(xd.data_ptr()), b._dt(xd), R, Cc, ld, b.FP4_AXIS_ROW,
                                    C.c_void_p(codes.data_ptr()), C.c_void_p(gamma.data_ptr()), None, 0, b._stream()) == 0
    else:
        codes, gamma = b.fp8_quantize(xd, b.FP4_AXIS_ROW)
    rc, rg = o.quantize_rows_fp8(x[:, :Cc].numpy())
    assert np.array_equal(gamma.cpu().numpy().view(np.uint32), rg.view(np.uint32))
    assert np.array_equal(codes.cpu().numpy(), rc)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(256, 64), (300, 136), (1024, 512), (34, 8), (130, 72)])
def test_fp8_quantize_cols_bit_exact(shape, dtype):
    R, Cc = shape
    g = torch.Generator().manual_seed(7 * R + Cc)
    x = torch.randn(R, Cc, generator=g) * 0.02 * torch.exp(torch.randn(1, Cc, generator=g))
    x[:, 1] = 0.0
    x = synth._finish(x, dtype)
    codes, gamma = b.fp8_quantize(dev(x, dtype), b.FP4_AXIS_COL)
    rc, rg = o.quantize_cols_fp8(x.numpy())
    assert codes.shape == (Cc, R)
    assert np.array_equal(gamma.cpu().numpy().view(np.uint32), rg.view(np.uint32))
    assert np.array_equal(codes.cpu().numpy(), rc)


@pytest.mark.parametrize("l_fp8", [True, False])
@pytest.mark.parametrize("shape", [(256, 256, 128), (300, 200, 256), (513, 264, 1152), (40, 8, 128), (700, 1032, 512)])
def test_mixed_gemm_against_the_exact_product(shape, l_fp8):
    """Random codes of both formats, no scales: against the exact integer-scaled product; the device's
    fp32 accumulation may round, so the bar is relative to the sum of the magnitudes."""
    P, Q, K = shape
    g = torch.Generator().manual_seed(P + Q + K)
    c8 = torch.randint(0, 256, (P if l_fp8 else Q, K), generator=g, dtype=torch.uint8)
    c8[(c8 & 0x7F) == 0x7F] = 0x30                       # no NaN patterns
    c4 = torch.randint(0, 16, (Q if l_fp8 else P, K), generator=g, dtype=torch.uint8)
    p4 = torch.from_numpy(o.pack_codes(c4.numpy()))
    v8 = o.e4m3_decode(c8.numpy()).astype(np.float64)
    v4 = o.e2m1_decode(c4.numpy()).astype(np.float64)
    if l_fp8:
        got = b.fp4_gemm_mixed(c8.cuda(), b.FP4_FMT_E4M3, None, p4.cuda(), b.FP4_FMT_E2M1, None)
        ref, mag = v8 @ v4.T, np.abs(v8) @ np.abs(v4).T
    else:
        got = b.fp4_gemm_mixed(p4.cuda(), b.FP4_FMT_E2M1, None, c8.cuda(), b.FP4_FMT_E4M3, None)
        ref, mag = v4 @ v8.T, np.abs(v4) @ np.abs(v8).T
    err = np.abs(got.cpu().numpy().astype(np.float64) - ref)
    assert np.all(err <= MIX_ACC * mag + 1e-30), float((err / (mag + 1e-30)).max())
    assert np.median(err / (mag + 1e-30)) < 2e-5


def _mixed_magnitudes(A, W, act8, alpha):
    """sum_k |a_k w_k| / (gamma_a gamma_w) of the quantized operands the forward pass multiplies."""
    if act8:
        ca, ga = o.quantize_rows_fp8(A)
        va = o.e4m3_decode(ca)
        cw, gw = o.quantize_cols(W)
        vw = o.e2m1_decode(cw)
    else:
        lo, hi = o.occ_thresholds(A, alpha)
        Ac, _ = o.occ_clamp_residual(A, lo, hi)
        ca, ga = o.quantize_rows(Ac)
        va = o.e2m1_decode(ca)
        cw, gw = o.quantize_cols_fp8(W)
        vw = o.e4m3_decode(cw)
    return o.dequant_gemm_values(np.abs(va), ga, np.abs(vw), gw)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", ["w4a8", "w8a4", "w8a4+occ"])
def test_mixed_forward(mode, dtype):
    A, W, _ = synth.small_case(288, 640, 264, dtype, seed=21)
    Ad, Wd = dev(A, dtype), dev(W, dtype)
    act8 = mode == "w4a8"
    alpha = 0.98 if mode.endswith("occ") else 1.0
    Y, ctx = b.fp4_linear_fwd_mixed(Ad, Wd, b.FP4_FMT_E4M3 if act8 else b.FP4_FMT_E2M1,
                                    b.FP4_FMT_E2M1 if act8 else b.FP4_FMT_E4M3, alpha)
    ref = o.linear_fwd_mixed(A.numpy(), W.numpy(), act8, not act8, alpha, "f32").astype(np.float64)
    if act8:
        _, gw = o.quantize_cols(W.numpy())
    else:
        _, gw = o.quantize_cols_fp8(W.numpy())
    assert np.array_equal(ctx.gamma_W.cpu().numpy().view(np.uint32), gw.view(np.uint32))
    mag = _mixed_magnitudes(A.numpy(), W.numpy(), act8, alpha)
    tol = 1e-3 * np.abs(ref) + MIX_ACC * mag
    if dtype == "bf16":
        tol = tol + 2.0 ** -8 * np.abs(ref)
    err = np.abs(Y.float().cpu().numpy().astype(np.float64) - ref)
    assert np.all(err <= tol), (mode, float((err / tol).max()))
    assert np.median(err / (np.abs(ref) + 1e-30)) < (1e-2 if dtype == "bf16" else 1e-4)


def test_mixed_argument_validation():
    import ctypes as C
    one = C.c_void_p(16)
    L = b.lib()
    assert L.fp4_gemm_mixed(one, 1, one, one, 0, one, 8, 8, 64, None, one, 0, 8, None) == -2       # K % 128
    assert L.fp4_gemm_mixed(one, 0, one, one, 0, one, 8, 8, 128, None, one, 0, 8, None) == -3      # both 4-bit
    assert L.fp4_gemm_mixed(one, 1, one, one, 1, one, 8, 8, 128, None, one, 0, 8, None) == -3      # both 8-bit
    ctx = b.fp4_fwd_ctx(16, 16, 16, 16, 16, 0, 16)
    assert L.fp4_linear_fwd_mixed(one, one, 0, 8, 128, 8, 1, 0, C.c_double(0.99), one, C.byref(ctx), one, 1 << 40, None) == -4
