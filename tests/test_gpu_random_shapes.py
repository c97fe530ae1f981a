"""GPU parity on drawn shapes: the whole layer (forward, both gradients) against the oracle on a fixed
list of randomly drawn but reproducible cases -- shapes inside the documented limits (K, M, N multiples of
32 for the three contractions), every operating point of alpha the workspaces provide for, both threshold
scopes, both master dtypes, several outlier structures (outlier channels, an outlier token, heavy tails,
one-sided data, many ties), weights from the cache or not.  Same bars as the hand-picked cases: saved
state bit-exact, outputs within the tolerance of the scaled results."""
import numpy as np
import pytest
import torch

from oracle import fp4_oracle as o
from paper_2501_17116_amd import binding as b
from paper_2501_17116_amd import synth

pytestmark = pytest.mark.gpu

RTOL = 1e-3
FLOOR = 2e-6


def _close(got, ref, out_dtype, what):
    g = got.float().cpu().numpy().astype(np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    tol = RTOL * np.abs(ref) + FLOOR * np.abs(ref).max()
    if out_dtype == "bf16":
        tol = tol + 2.0 ** -8 * np.abs(ref) + 2.0 ** -133
    bad = np.abs(g - ref) > tol
    assert not bad.any(), "%s: %d of %d outside tolerance, worst %g vs %g" % (what, bad.sum(), bad.size, g[bad][0], ref[bad][0])


def _draw(i):
    r = np.random.default_rng(7000 + i)
    M = 32 * int(r.integers(1, 49))
    K = 32 * int(r.integers(1, 73))
    N = 32 * int(r.integers(1, 37))
    if i % 6 == 0:
        M, K = 32 * int(r.integers(66, 80)), 32 * int(r.integers(1, 9))   # tall: long rows in the transposed residual
    alpha = float(r.choice([0.9, 0.95, 0.97, 0.99, 0.995, 0.999]))
    dtype = "bf16" if r.random() < 0.6 else "f32"
    scope = "token" if (i % 3 == 1) else "tensor"
    if scope == "token" and 2 * int(np.floor((1 - alpha) * K)) >= K:
        scope = "tensor"
    kind = ["channels", "token", "heavy", "onesided", "ties"][i % 5]
    cached = bool(r.integers(0, 2))
    return M, K, N, alpha, dtype, scope, kind, cached, r


def _inputs(M, K, N, dtype, kind, r):
    g = torch.Generator().manual_seed(int(r.integers(1, 1 << 30)))
    A = torch.randn(M, K, generator=g)
    if kind == "channels":
        ch = torch.randperm(K, generator=g)[:max(1, K // 100)]
        A[:, ch] *= 30.0
    elif kind == "token":
        A[int(r.integers(0, M))] *= 150.0
    elif kind == "heavy":
        A = A / torch.sqrt((torch.randn(M, K, generator=g) ** 2 + torch.randn(M, K, generator=g) ** 2
                            + torch.randn(M, K, generator=g) ** 2) / 3.0)
    elif kind == "onesided":
        A = A.abs() + 0.25
    else:   # many equal values, thresholds land on ties
        A = torch.round(A * 2.0) / 2.0
    W = torch.randn(K, N, generator=g) * 0.02
    dY = torch.randn(M, N, generator=g) * 0.01
    return synth._finish(A, dtype), synth._finish(W, dtype), synth._finish(dY, dtype)


@pytest.mark.parametrize("i", range(48))
def test_drawn_layer(i):
    M, K, N, alpha, dtype, scope, kind, cached, r = _draw(i)
    A, W, dY = _inputs(M, K, N, dtype, kind, r)
    cast = torch.bfloat16 if dtype == "bf16" else torch.float32
    Ad, Wd, dYd = A.to(cast).cuda(), W.to(cast).cuda(), dY.to(cast).cuda()
    print("case", i, M, K, N, alpha, dtype, scope, kind, "cached" if cached else "plain", flush=True)
    sc = b.FP4_OCC_TOKEN if scope == "token" else b.FP4_OCC_TENSOR
    ctx = b.FwdCtx(M, K, N, alpha, scope=sc)
    wq = b.fp4_prepare_weights(Wd) if cached else None
    if cached:
        Y, _ = b.fp4_linear_fwd_cached(Ad, Wd, wq, alpha, ctx=ctx)
    else:
        Y, _ = b.fp4_linear_fwd(Ad, Wd, alpha, ctx=ctx)
    dA, dW = b.fp4_linear_bwd(dYd, Ad, Wd, ctx, 5.0, 3.0, wq=wq)
    torch.cuda.synchronize()

    An, Wn, dYn = A.numpy(), W.numpy(), dY.numpy()
    Yref, st = o.fp4_linear_fwd(An, Wn, alpha, "f32", scope=scope)
    nnz = int(ctx.nnz.item())
    assert nnz == st.csr.val.size
    assert np.array_equal(ctx.row_ptr.cpu().numpy(), st.csr.row_ptr)
    assert np.array_equal(ctx.col_idx.cpu().numpy()[:nnz], st.csr.col_idx)
    assert np.array_equal(ctx.val.cpu().numpy()[:nnz].view(np.uint32), st.csr.val.view(np.uint32))
    assert np.array_equal(ctx.gamma_W.cpu().numpy().view(np.uint32), st.gamma_w.view(np.uint32))
    thr = ctx.thresholds.cpu().numpy()
    if scope == "token":
        assert np.array_equal(thr.reshape(M, 2)[:, 0], np.asarray(st.lo, dtype=np.float32).reshape(-1))
        assert np.array_equal(thr.reshape(M, 2)[:, 1], np.asarray(st.hi, dtype=np.float32).reshape(-1))
    else:
        assert thr[0] == st.lo and thr[1] == st.hi
    _close(Y, Yref, dtype, "Y")
    _close(dA, o.fp4_linear_bwd_dgrad(dYn, Wn, "f32"), dtype, "dA")
    _close(dW, o.fp4_linear_bwd_wgrad(An, dYn, Wn, alpha, 5.0, 3.0, scope=scope), "f32", "dW")
