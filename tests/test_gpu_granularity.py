"""GPU parity of tensor-wise scaling (the coarse granularity of the Sec. 4.3 ablation): codes and the
scale bit-exact against the oracle; the forward pass in all four granularity combinations within the
tolerance of the scaled outputs, with the saved scales and residual bit-exact."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import fp4_oracle as o
from paper_2501_17116_amd import binding as b
from paper_2501_17116_amd import synth

pytestmark = pytest.mark.gpu

RTOL = 1e-3
FLOOR = 2e-6


def dev(x, dtype):
    return (x.to(torch.bfloat16) if dtype == "bf16" else x.to(torch.float32)).contiguous().cuda()


def _close(got, ref, out_dtype, what):
    g = got.float().cpu().numpy().astype(np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    tol = RTOL * np.abs(ref) + FLOOR * np.abs(ref).max()
    if out_dtype == "bf16":
        tol = tol + 2.0 ** -8 * np.abs(ref) + 2.0 ** -133
    bad = np.abs(g - ref) > tol
    assert not bad.any(), "%s: %d of %d outside tolerance, worst %g vs %g" % (what, bad.sum(), bad.size, g[bad][0], ref[bad][0])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(1, 8), (7, 64), (33, 520), (64, 4096), (5, 9000), (4100, 72), (300, 16392), (3, 10)])
def test_tensorwise_quantize_bit_exact(shape, dtype):
    R, Cc = shape
    g = torch.Generator().manual_seed(31 * R + Cc)
    ld = (Cc + 7) // 8 * 8
    x = torch.randn(R, ld, generator=g) * torch.exp(torch.randn(R, 1, generator=g) * 2)
    if R > 2:
        x[2] = 0.0
    x[:, Cc:] = 1e6        # beyond the row: must not reach the scale
    x = synth._finish(x, dtype)
    xd = dev(x, dtype)
    codes = torch.empty((R, Cc // 2), dtype=torch.uint8, device="cuda")
    gamma = torch.empty(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(b.workspace_bytes(b.FP4_OP_QUANTIZE, R, Cc, 0, b._dt(xd)), dtype=torch.uint8, device="cuda")
    rc = b.lib().fp4_quantize(C.c_void_p(xd.data_ptr()), b._dt(xd), R, Cc, ld, b.FP4_AXIS_TENSOR, C.c_void_p(codes.data_ptr()),
                              C.c_void_p(gamma.data_ptr()), C.c_void_p(ws.data_ptr()), ws.numel(), b._stream())
    assert rc == 0
    rcodes, rg = o.quantize_tensor(x[:, :Cc].numpy())
    assert gamma.cpu().numpy().view(np.uint32)[0] == np.asarray(rg, dtype=np.float32).reshape(1).view(np.uint32)[0]
    assert np.array_equal(o.unpack_codes(codes.cpu().numpy()), rcodes)


def test_tensorwise_quantize_zero_tensor_and_binding():
    x = torch.zeros(40, 64, device="cuda")
    codes, gamma = b.fp4_quantize(x, b.FP4_AXIS_TENSOR)
    assert gamma.shape == (1,) and float(gamma[0]) == 1.0 and not codes.any()
    y = torch.randn(48, 96, device="cuda").bfloat16()
    codes, gamma = b.fp4_quantize(y, b.FP4_AXIS_TENSOR)
    rc, rg = o.quantize_tensor(y.float().cpu().numpy())
    assert float(gamma[0]) == float(rg) and np.array_equal(o.unpack_codes(codes.cpu().numpy()), rc)


CASES = [(160, 288, 224, "f32", 0.97), (288, 544, 1056, "bf16", 0.99), (96, 128, 96, "bf16", 1.0),
         (1120, 1056, 160, "bf16", 0.98), (64, 4128, 64, "f32", 0.95)]


@pytest.mark.parametrize("act_t,wgt_t", [(True, False), (False, True), (True, True), (False, False)])
@pytest.mark.parametrize("M,K,N,dtype,alpha", CASES)
def test_forward_granularity(M, K, N, dtype, alpha, act_t, wgt_t):
    A, W, _ = synth.small_case(M, K, N, dtype, seed=M + K + N + 1)
    Ad, Wd = dev(A, dtype), dev(W, dtype)
    Y, ctx = b.fp4_linear_fwd_granularity(Ad, Wd, act_t, wgt_t, alpha)
    torch.cuda.synchronize()
    An, Wn = A.numpy(), W.numpy()
    Yref = o.linear_fwd_granularity(An, Wn, act_t, wgt_t, alpha, "f32")
    # saved state: the residual is that of the ordinary forward pass; the weight scales are those used
    _, st = o.fp4_linear_fwd(An, Wn, alpha, "f32")
    nnz = int(ctx.nnz.item())
    assert nnz == st.csr.val.size
    if alpha < 1.0:
        assert np.array_equal(ctx.row_ptr.cpu().numpy(), st.csr.row_ptr)
        assert np.array_equal(ctx.col_idx.cpu().numpy()[:nnz], st.csr.col_idx)
        assert np.array_equal(ctx.val.cpu().numpy()[:nnz].view(np.uint32), st.csr.val.view(np.uint32))
    gw = ctx.gamma_W.cpu().numpy()
    if wgt_t:
        want = np.asarray(o.quantize_tensor(Wn)[1], dtype=np.float32).reshape(1)
        assert np.all(gw.view(np.uint32) == want.view(np.uint32)[0])
    else:
        assert np.array_equal(gw.view(np.uint32), st.gamma_w.view(np.uint32))
    _close(Y, Yref, dtype, "Y")
    if not act_t and not wgt_t:   # vector-wise on both sides: the ordinary entry point, bit for bit
        Y0, _ = b.fp4_linear_fwd(Ad, Wd, alpha)
        assert torch.equal(Y, Y0)


def test_granularity_refuses_per_token_thresholds_with_a_tensor_scale():
    A = torch.randn(64, 128, device="cuda")
    W = torch.randn(128, 64, device="cuda") * 0.02
    ctx = b.FwdCtx(64, 128, 64, 0.99, scope=b.FP4_OCC_TOKEN)
    with pytest.raises(b.Fp4Error):
        b.fp4_linear_fwd_granularity(A, W, True, False, 0.99, ctx=ctx)
    b.fp4_linear_fwd_granularity(A, W, False, True, 0.99, ctx=ctx)   # weights alone: fine
    torch.cuda.synchronize()
