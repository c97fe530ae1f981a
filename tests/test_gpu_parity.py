"""GPU parity: every entry point of the C ABI against the CPU oracle on the same seeded inputs.

Bars: 4-bit codes, scales, thresholds, residual triplets and raw accumulators bit-exact;
scaled outputs and gradients within  1e-3 * |ref| + 2e-6 * max|ref|  of the oracle's fp64
value (fp32 outputs), plus half a bf16 ulp (2^-8 |ref|) when the output is bf16.
"""
import numpy as np
import pytest
import torch

from oracle import fp4_oracle as o
from paper_2501_17116_amd import binding as b
from paper_2501_17116_amd import synth

pytestmark = pytest.mark.gpu

RTOL = 1e-3
FLOOR = 2e-6


def dev(x: torch.Tensor, dtype: str) -> torch.Tensor:
    t = x.to(torch.bfloat16) if dtype == "bf16" else x.to(torch.float32)
    return t.contiguous().cuda()


def host_codes(packed: torch.Tensor) -> np.ndarray:
    return o.unpack_codes(packed.cpu().numpy())


def assert_close(got: torch.Tensor, ref: np.ndarray, out_dtype: str, what: str):
    g = got.float().cpu().numpy().astype(np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    tol = RTOL * np.abs(ref) + FLOOR * np.abs(ref).max()
    if out_dtype == "bf16":
        tol = tol + 2.0 ** -8 * np.abs(ref) + 2.0 ** -133
    bad = np.abs(g - ref) > tol
    assert not bad.any(), "%s: %d of %d outside tolerance, worst %g vs %g" % (
        what, bad.sum(), bad.size, g[bad][0], ref[bad][0])
    if out_dtype == "f32":
        rel = np.abs(g - ref) / (np.abs(ref) + 1e-30)
        assert np.median(rel) < 1e-5, what


# ------------------------------------------------------------------------------------------
# quantization
# ------------------------------------------------------------------------------------------
# one shape at least for every variant of the row kernel (1 wave or 1 workgroup per row x units per thread)
ROW_SHAPES = [(7, 64), (16, 10), (33, 520), (64, 4096), (5, 9000), (3, 20000), (1, 2), (130, 1024), (29, 2048),
              (37, 1544), (6, 11008), (4, 14000)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", ROW_SHAPES)
def test_quantize_rows_bit_exact(shape, dtype):
    R, Cc = shape
    ldpad = (Cc + 7) // 8 * 8
    g = torch.Generator().manual_seed(R * 1000 + Cc)
    x = torch.randn(R, ldpad, generator=g) * torch.exp(torch.randn(R, 1, generator=g) * 2)
    x[:, : min(4, Cc)] *= 30
    if R > 2:
        x[2] = 0.0                                    # all-zero row -> gamma 1, codes 0
    x = synth._finish(x, dtype)
    xd = dev(x, dtype)
    if ldpad != Cc:
        # exercise ld > cols through the raw ABI
        import ctypes as C
        codes = torch.empty((R, Cc // 2), dtype=torch.uint8, device="cuda")
        gamma = torch.empty(R, dtype=torch.float32, device="cuda")
        st = b.lib().fp4_quantize(C.c_void_p(xd.data_ptr()), b._dt(xd), R, Cc, ldpad, b.FP4_AXIS_ROW,
                                  C.c_void_p(codes.data_ptr()), C.c_void_p(gamma.data_ptr()), None, 0,
                                  b._stream())
        assert st == 0
    else:
        codes, gamma = b.fp4_quantize(xd, b.FP4_AXIS_ROW)
    torch.cuda.synchronize()
    rc, rg = o.quantize_rows(x[:, :Cc].numpy())
    assert np.array_equal(gamma.cpu().numpy().view(np.uint32), rg.view(np.uint32))
    assert np.array_equal(host_codes(codes), rc)


def test_quantize_ties_and_tiny_values_bit_exact():
    # rows whose absmax is 6 (gamma = 1) so scaled values hit the midpoints exactly
    ties = torch.tensor([6, .25, -.25, .75, -.75, 1.25, -1.25, 1.75, -1.75, 2.5, -2.5, 3.5, -3.5, 5, -5, 0.,
                         -0., 6, -6, 5.9999995, 0.24999999, -0.25000003, 1e-30, -1e-30], dtype=torch.float32)
    x = torch.zeros(4, 32)
    x[0, :ties.numel()] = ties
    x[1, :ties.numel()] = ties * 2 ** -100            # same pattern, gamma = 2^100
    x[2, 0] = 1e-44                                   # subnormal absmax: 6/amax overflows -> gamma 1
    x[3, :ties.numel()] = ties.flip(0)
    codes, gamma = b.fp4_quantize(x.cuda(), b.FP4_AXIS_ROW)
    rc, rg = o.quantize_rows(x.numpy())
    assert np.array_equal(gamma.cpu().numpy().view(np.uint32), rg.view(np.uint32))
    assert np.array_equal(host_codes(codes), rc)


COL_SHAPES = [(256, 64), (300, 136), (1024, 512), (34, 8), (2, 2048), (514, 72)]


def test_device_rounding_equals_the_oracle_bit_for_bit():
    """The packing routine the quantization kernels use (FP4 convert instruction plus the tie correction)
    against the oracle's App. A rounding: thresholds with their neighbours, specials, random bit patterns."""
    rng = np.random.default_rng(5)
    pts = [0.25, 0.5, 0.75, 1, 1.25, 1.5, 1.75, 2, 2.5, 3, 3.5, 4, 5, 6, 7, 0.0]
    edge = []
    for p in pts:
        for sgn in (1, -1):
            v = np.float32(sgn * p)
            edge += [v, np.nextafter(v, np.float32(np.inf)), np.nextafter(v, np.float32(-np.inf))]
    edge += [np.float32(x) for x in (np.inf, -np.inf, np.nan, 1e-45, -1e-45, 1e38, -1e38, -0.0)]
    edge = np.array(edge + [np.float32(0)] * (-len(edge) % 8), np.float32)
    base = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0], np.float32).view(np.uint32)
    near = (base[:, None].astype(np.int64) + np.arange(-2000, 2000)[None, :]).astype(np.uint32).ravel()
    sets = [edge, near.view(np.float32), (near | np.uint32(0x80000000)).view(np.float32),
            rng.integers(0, 2 ** 32, 8_000_000, dtype=np.uint64).astype(np.uint32).view(np.float32),
            rng.uniform(-7, 7, 8_000_000).astype(np.float32)]
    for x in sets:
        # each value also lands in every position of a packed word
        for shift in (0, 3):
            xs = np.roll(x, shift)
            got = b.fp4_device_round_codes(torch.from_numpy(xs).cuda()).cpu().numpy()
            assert np.array_equal(got, o.q_e2m1(xs))


def test_device_rounding_routines_agree_on_every_bit_pattern():
    """All 2^32 fp32 patterns in all eight word positions: packing routine == comparison-chain routine
    (the latter is pinned to the oracle on the host, exhaustively near the thresholds)."""
    assert b.fp4_device_round_sweep() == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", COL_SHAPES)
def test_quantize_cols_bit_exact(shape, dtype):
    R, Cc = shape
    g = torch.Generator().manual_seed(7 * R + Cc)
    x = torch.randn(R, Cc, generator=g) * 0.02 * torch.exp(torch.randn(1, Cc, generator=g))
    x[:, 1] = 0.0
    x = synth._finish(x, dtype)
    codes, gamma = b.fp4_quantize(dev(x, dtype), b.FP4_AXIS_COL)
    rc, rg = o.quantize_cols(x.numpy())
    assert codes.shape == (Cc, R // 2)
    assert np.array_equal(gamma.cpu().numpy().view(np.uint32), rg.view(np.uint32))
    assert np.array_equal(host_codes(codes), rc)


def test_unpack():
    p = torch.randint(0, 256, (37, 24), dtype=torch.uint8)
    assert np.array_equal(b.fp4_unpack(p.cuda()).cpu().numpy(), o.unpack_codes(p.numpy()))


# ------------------------------------------------------------------------------------------
# GEMM
# ------------------------------------------------------------------------------------------
GEMM_SHAPES = [(256, 256, 256), (64, 48, 32), (300, 200, 128), (513, 257, 1056), (1, 8, 64), (700, 1030, 512)]


@pytest.mark.parametrize("shape", GEMM_SHAPES)
def test_gemm_raw_accumulator_bit_exact(shape):
    P, Q, K = shape
    g = torch.Generator().manual_seed(P + Q + K)
    ca = torch.randint(0, 16, (P, K), generator=g, dtype=torch.uint8)
    cb = torch.randint(0, 16, (Q, K), generator=g, dtype=torch.uint8)
    pa = torch.from_numpy(o.pack_codes(ca.numpy())).cuda()
    pb = torch.from_numpy(o.pack_codes(cb.numpy())).cuda()
    acc = b.fp4_gemm(pa, None, pb, None)
    ref = o.gemm_acc(ca.numpy(), cb.numpy())
    assert np.array_equal(acc.cpu().numpy().astype(np.float64), ref)


def test_gemm_extreme_codes_long_k_exact():
    # all +-6 over K = 16384: |acc| = 36 K, the largest accumulator any config produces
    K = 16384
    ca = torch.full((40, K), 7, dtype=torch.uint8)
    cb = torch.full((24, K), 15, dtype=torch.uint8)
    cb[::2] = 7
    acc = b.fp4_gemm(torch.from_numpy(o.pack_codes(ca.numpy())).cuda(), None,
                     torch.from_numpy(o.pack_codes(cb.numpy())).cuda(), None)
    assert np.array_equal(acc.cpu().numpy().astype(np.float64), o.gemm_acc(ca.numpy(), cb.numpy()))


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_gemm_scaled_and_addend(out_dtype):
    P, Q, K = 300, 264, 384
    g = torch.Generator().manual_seed(5)
    A = torch.randn(P, K, generator=g)
    W = torch.randn(K, Q, generator=g) * 0.02
    ca, ga = o.quantize_rows(A.numpy())
    cw, gw = o.quantize_cols(W.numpy())
    add = torch.randn(P, Q, generator=g)
    tdt = torch.bfloat16 if out_dtype == "bf16" else torch.float32
    y = b.fp4_gemm(torch.from_numpy(o.pack_codes(ca)).cuda(), torch.from_numpy(ga).cuda(),
                   torch.from_numpy(o.pack_codes(cw)).cuda(), torch.from_numpy(gw).cuda(), out_dtype=tdt)
    assert_close(y, o.dequant_gemm(ca, ga, cw, gw), out_dtype, "scaled gemm")
    y2 = b.fp4_gemm(torch.from_numpy(o.pack_codes(ca)).cuda(), torch.from_numpy(ga).cuda(),
                    torch.from_numpy(o.pack_codes(cw)).cuda(), torch.from_numpy(gw).cuda(), out_dtype=tdt,
                    addend=add.cuda())
    assert_close(y2, o.dequant_gemm(ca, ga, cw, gw) + add.numpy().astype(np.float64), out_dtype, "gemm+addend")


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_gemm_interior_and_edge_tiles_give_the_same_bits(out_dtype):
    # The kernel finishes tiles that lie wholly inside the output with a branch-free epilogue and tiles on
    # the edge with a masked one.  The same problem computed once with ragged edges and once padded (zero
    # codes, unit scales, zero addend) to whole tiles must agree bit for bit where the two overlap.
    P, Q, K, PP, QP = 288, 296, 384, 512, 512
    g = torch.Generator().manual_seed(11)
    A = torch.randn(P, K, generator=g)
    W = torch.randn(K, Q, generator=g) * 0.02
    ca, ga = o.quantize_rows(A.numpy())
    cw, gw = o.quantize_cols(W.numpy())
    add = torch.randn(P, Q, generator=g)
    tdt = torch.bfloat16 if out_dtype == "bf16" else torch.float32
    pa, pw = o.pack_codes(ca), o.pack_codes(cw)
    small = b.fp4_gemm(torch.from_numpy(pa).cuda(), torch.from_numpy(ga).cuda(), torch.from_numpy(pw).cuda(),
                       torch.from_numpy(gw).cuda(), out_dtype=tdt, addend=add.cuda())
    pa_big = np.zeros((PP, pa.shape[1]), dtype=np.uint8); pa_big[:P] = pa
    pw_big = np.zeros((QP, pw.shape[1]), dtype=np.uint8); pw_big[:Q] = pw
    ga_big = np.ones(PP, dtype=np.float32); ga_big[:P] = ga
    gw_big = np.ones(QP, dtype=np.float32); gw_big[:Q] = gw
    add_big = torch.zeros(PP, QP); add_big[:P, :Q] = add
    big = b.fp4_gemm(torch.from_numpy(pa_big).cuda(), torch.from_numpy(ga_big).cuda(), torch.from_numpy(pw_big).cuda(),
                     torch.from_numpy(gw_big).cuda(), out_dtype=tdt, addend=add_big.cuda())
    torch.cuda.synchronize()
    view = torch.int16 if out_dtype == "bf16" else torch.int32
    assert torch.equal(small.contiguous().view(view), big[:P, :Q].contiguous().view(view))
    assert_close(big[:P, :Q], o.dequant_gemm(ca, ga, cw, gw) + add.numpy().astype(np.float64), out_dtype, "padded gemm+addend")


# ------------------------------------------------------------------------------------------
# OCC
# ------------------------------------------------------------------------------------------
def _check_occ(x: torch.Tensor, dtype: str, alpha: float):
    out = b.occ_clamp_residual(dev(x, dtype), alpha, want_codes=True, want_clamped=True)
    torch.cuda.synchronize()
    xn = x.numpy()
    lo, hi = o.occ_thresholds(xn, alpha)
    thr = out["thresholds"].cpu().numpy()
    assert thr[0] == lo and thr[1] == hi, (thr, lo, hi)
    xc, csr = o.occ_clamp_residual(xn, lo, hi)
    nnz = int(out["nnz"].item())
    assert nnz == csr.val.size <= b.occ_capacity(x.shape[0], x.shape[1], alpha)
    assert np.array_equal(out["row_ptr"].cpu().numpy(), csr.row_ptr)
    assert np.array_equal(out["col_idx"].cpu().numpy()[:nnz], csr.col_idx)
    assert np.array_equal(out["val"].cpu().numpy()[:nnz].view(np.uint32), csr.val.view(np.uint32))
    assert np.array_equal(out["x_clamped"].float().cpu().numpy(), xc)
    rc, rg = o.quantize_rows(xc)
    assert np.array_equal(out["gamma"].cpu().numpy().view(np.uint32), rg.view(np.uint32))
    assert np.array_equal(host_codes(out["codes"]), rc)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape,alpha", [((256, 512), 0.99), ((100, 72), 0.97), ((64, 4096), 0.999),
                                          ((9, 2056), 0.99), ((300, 640), 1.0), ((2, 20000), 0.95),
                                          ((5, 6000), 0.98), ((3, 12000), 0.99), ((130, 11008), 0.99),
                                          ((37, 1544), 0.98), ((29, 2048), 0.99), ((4, 14000), 0.99)])
def test_occ_clamp_residual_bit_exact(shape, alpha, dtype):
    cfg = synth.CONFIGS["c1"]
    x = synth.make_activation(cfg, shape[0], shape[1], salt=shape[0])
    _check_occ(synth._finish(x, dtype), dtype, alpha)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,cols,ld,alpha", [(16, 10, 16, 0.9), (33, 74, 80, 0.97), (9, 2050, 2056, 0.99),
                                                 (40, 520, 1024, 0.98), (3, 20002, 20008, 0.95),
                                                 (5, 9002, 9008, 0.99), (64, 4096, 4104, 0.999)])
def test_occ_raw_abi_ragged_cols_and_padded_rows(rows, cols, ld, alpha, dtype):
    """cols not a multiple of 8 and ld > cols through the C ABI itself: the selection's element-wise
    walk, the ragged last unit of every row under OCC, x_clamped with a leading dimension, and
    guard columns that must stay untouched."""
    import ctypes as C
    cfg = synth.CONFIGS["c1"]
    x = synth._finish(synth.make_activation(cfg, rows, ld, salt=rows + cols), dtype)
    x[:, cols:] = 1e6                                   # padding must not reach thresholds, scales or entries
    xd = dev(x, dtype)
    tdt = xd.dtype
    cap = b.occ_capacity(rows, cols, alpha)
    thr = torch.empty(2, dtype=torch.float32, device="cuda")
    codes = torch.full((rows, cols // 2), 0xEE, dtype=torch.uint8, device="cuda")
    gamma = torch.empty(rows, dtype=torch.float32, device="cuda")
    xc = torch.full((rows, ld), 7.0, dtype=tdt, device="cuda")
    row_ptr = torch.empty(rows + 1, dtype=torch.int64, device="cuda")
    col_idx = torch.empty(max(cap, 1), dtype=torch.int32, device="cuda")
    val = torch.empty(max(cap, 1), dtype=torch.float32, device="cuda")
    nnz = torch.zeros(1, dtype=torch.int64, device="cuda")
    ws = torch.empty(b.workspace_bytes(b.FP4_OP_OCC, rows, cols, 0, b._dt(xd)), dtype=torch.uint8, device="cuda")
    P = lambda t: C.c_void_p(t.data_ptr())
    st = b.lib().occ_clamp_residual(P(xd), b._dt(xd), rows, cols, ld, C.c_double(alpha), P(thr), P(codes), P(gamma),
                                    P(xc), P(row_ptr), P(col_idx), P(val), cap, P(nnz), P(ws), ws.numel(),
                                    b._stream())
    assert st == 0
    torch.cuda.synchronize()
    xn = x[:, :cols].contiguous().numpy()
    lo, hi = o.occ_thresholds(xn, alpha)
    t = thr.cpu().numpy()
    assert t[0] == lo and t[1] == hi, (t, lo, hi)
    xcr, csr = o.occ_clamp_residual(xn, lo, hi)
    n = int(nnz.item())
    assert n == csr.val.size <= cap
    assert np.array_equal(row_ptr.cpu().numpy(), csr.row_ptr)
    assert np.array_equal(col_idx.cpu().numpy()[:n], csr.col_idx)
    assert np.array_equal(val.cpu().numpy()[:n].view(np.uint32), csr.val.view(np.uint32))
    xch = xc.float().cpu().numpy()
    assert np.array_equal(xch[:, :cols], xcr)
    assert np.all(xch[:, cols:] == 7.0)                 # guard columns untouched
    rc, rg = o.quantize_rows(xcr)
    assert np.array_equal(gamma.cpu().numpy().view(np.uint32), rg.view(np.uint32))
    assert np.array_equal(host_codes(codes), rc)


def _check_occ_token(x: torch.Tensor, dtype: str, alpha: float):
    out = b.occ_clamp_residual(dev(x, dtype), alpha, want_codes=True, want_clamped=True, scope=b.FP4_OCC_TOKEN)
    torch.cuda.synchronize()
    xn = x.numpy()
    R, Ccols = xn.shape
    lo, hi = o.occ_thresholds_per_token(xn, alpha)
    thr = out["thresholds"].cpu().numpy().reshape(R, 2)
    assert np.array_equal(thr[:, 0], lo) and np.array_equal(thr[:, 1], hi)
    xc, csr = o.occ_clamp_residual(xn, lo, hi)
    nnz = int(out["nnz"].item())
    assert nnz == csr.val.size <= R * 2 * o.occ_tail_count(Ccols, alpha)
    assert np.array_equal(out["row_ptr"].cpu().numpy(), csr.row_ptr)
    assert np.array_equal(out["col_idx"].cpu().numpy()[:nnz], csr.col_idx)
    assert np.array_equal(out["val"].cpu().numpy()[:nnz].view(np.uint32), csr.val.view(np.uint32))
    assert np.array_equal(out["x_clamped"].float().cpu().numpy(), xc)
    rc, rg = o.quantize_rows(xc)
    assert np.array_equal(out["gamma"].cpu().numpy().view(np.uint32), rg.view(np.uint32))
    assert np.array_equal(host_codes(out["codes"]), rc)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape,alpha", [((256, 512), 0.99), ((100, 72), 0.97), ((64, 4096), 0.999), ((9, 2056), 0.99),
                                          ((300, 640), 1.0), ((5, 6000), 0.98), ((3, 12000), 0.99), ((130, 11008), 0.99),
                                          ((37, 1544), 0.98), ((29, 2048), 0.9), ((4, 14000), 0.97), ((7, 16384), 0.99),
                                          ((6, 16), 0.9), ((33, 4088), 0.99)])
def test_occ_per_token_thresholds_bit_exact(shape, alpha, dtype):
    """The per-token reading: every row's own order statistics (found in registers by radix selection),
    clamp, residual and codes, one row-kernel variant per shape class, ragged row lengths included."""
    cfg = synth.CONFIGS["c1"]
    x = synth.make_activation(cfg, shape[0], shape[1], salt=shape[0] + 1)
    _check_occ_token(synth._finish(x, dtype), dtype, alpha)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_occ_per_token_ties_constant_rows_and_signed_zeros(dtype):
    g = torch.Generator().manual_seed(31)
    x = torch.randint(-3, 4, (40, 256), generator=g).float()          # heavy ties around the thresholds
    x[3] = 1.5                                                        # a constant row: nothing clamped
    x[4] = 0.0
    x[5, ::2] = -0.0
    x[6] = torch.randn(256, generator=g).abs() + 1                    # one-sided rows
    x[7] = -torch.randn(256, generator=g).abs()
    _check_occ_token(synth._finish(x, dtype), dtype, 0.95)
    x = torch.randn(16, 4096, generator=g) * torch.exp(4 * torch.randn(16, 1, generator=g))   # rows of very different scale
    x[:, 7] *= 1e4
    _check_occ_token(synth._finish(x, dtype), dtype, 0.99)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_occ_with_ties_one_sided_and_constant(dtype):
    g = torch.Generator().manual_seed(3)
    x = torch.randint(0, 5, (64, 128), generator=g).float()          # heavy ties, all non-negative
    _check_occ(synth._finish(x, dtype), dtype, 0.97)
    _check_occ(torch.full((16, 64), 1.5), dtype, 0.99)                # constant tensor: nothing clamped
    x = torch.randn(32, 64, generator=g).abs() + 1.0                  # one-sided
    _check_occ(synth._finish(x, dtype), dtype, 0.9)
    x = torch.randn(32, 64, generator=g)
    x[0, 0] = -0.0
    _check_occ(synth._finish(-x.abs(), dtype), dtype, 0.95)


def test_residual_spmm_with_long_rows():
    # rows far longer than the rest take the long-row path; short, empty and ragged ones the tiled path
    g = torch.Generator().manual_seed(17)
    P, Q, N = 1300, 5000, 200
    dense = torch.zeros(P, Q)
    mask = torch.rand(P, Q, generator=g) < 0.01
    mask[3] = True                      # 5000 entries
    mask[1000, ::2] = True              # 2500 entries
    mask[7] = False                     # empty row
    dense[mask] = torch.randn(int(mask.sum()), generator=g)
    rows, cols = np.nonzero(dense.numpy())
    row_ptr = np.zeros(P + 1, np.int64)
    np.cumsum(np.bincount(rows, minlength=P), out=row_ptr[1:])
    vals = dense.numpy()[rows, cols].astype(np.float32)
    D = synth._finish(torch.randn(Q, N, generator=g), "bf16")
    R = b.fp4_residual_spmm(torch.from_numpy(row_ptr).cuda(), torch.from_numpy(cols.astype(np.int32)).cuda(),
                            torch.from_numpy(vals).cuda(), Q, dev(D, "bf16"))
    assert_close(R, dense.numpy().astype(np.float64) @ D.numpy().astype(np.float64), "f32", "spmm long rows")


@pytest.mark.parametrize("dtype,P,n_long", [("f32", 45, 40), ("bf16", 45, 40), ("bf16", 8, 7), ("f32", 14, 12)])
def test_residual_spmm_many_long_rows(dtype, P, n_long):
    # more long rows than the batched dense path accepts: the remainder goes row by row; two
    # slices of D rows, the second ragged; short rows in between
    g = torch.Generator().manual_seed(23)
    Q, N = 2600, 520
    dense = torch.zeros(P, Q)
    mask = torch.rand(P, Q, generator=g) < 0.9
    mask[::9] = torch.rand((P + 8) // 9, Q, generator=g) < 0.02      # rows 0, 9, .. stay short
    dense[mask] = torch.randn(int(mask.sum()), generator=g)
    rows, cols = np.nonzero(dense.numpy())
    row_ptr = np.zeros(P + 1, np.int64)
    np.cumsum(np.bincount(rows, minlength=P), out=row_ptr[1:])
    assert int((np.diff(row_ptr) > 2048).sum()) == n_long
    vals = dense.numpy()[rows, cols].astype(np.float32)
    D = synth._finish(torch.randn(Q, N, generator=g), dtype)
    args = (torch.from_numpy(row_ptr).cuda(), torch.from_numpy(cols.astype(np.int32)).cuda(),
            torch.from_numpy(vals).cuda(), Q, dev(D, dtype))
    R = b.fp4_residual_spmm(*args)
    assert_close(R, dense.numpy().astype(np.float64) @ D.numpy().astype(np.float64), "f32", "spmm many long rows")
    assert torch.equal(R, b.fp4_residual_spmm(*args))      # fixed summation order


def test_residual_spmm():
    g = torch.Generator().manual_seed(11)
    x = torch.randn(70, 96, generator=g)
    lo, hi = o.occ_thresholds(x.numpy(), 0.95)
    _, csr = o.occ_clamp_residual(x.numpy(), lo, hi)
    for dtype in ("f32", "bf16"):
        D = synth._finish(torch.randn(96, 2056, generator=g), dtype)
        R = b.fp4_residual_spmm(torch.from_numpy(csr.row_ptr).cuda(), torch.from_numpy(csr.col_idx).cuda(),
                                torch.from_numpy(csr.val).cuda(), 96, dev(D, dtype))
        assert_close(R, csr.to_dense() @ D.numpy().astype(np.float64), "f32", "spmm")


def test_residual_spmm_random_shapes():
    """Seeded sweep of ragged shapes and densities: rows whose entry counts sit on either side of a multiple of
    four (the kernel walks a row four entries at a time), rows ending on a slab boundary, empty rows and empty
    matrices, a last row that ends exactly at the end of the arrays, several 1024-row blocks."""
    rng = np.random.default_rng(2024)
    cases = [(1, 1, 8), (3, 4, 8), (5, 513, 72), (64, 512, 64), (65, 1030, 136), (1100, 96, 200), (2100, 40, 8),
             (17, 2049, 264), (1, 3000, 16), (1030, 1537, 72)]
    for ci, (P, Q, N) in enumerate(cases):
        for dtype in ("bf16", "f32"):
            dens = [0.0, 0.02, 0.3, 1.0][(ci + (dtype == "f32")) % 4]
            per_row = rng.binomial(min(Q, 2048), dens, size=P) if dens < 1.0 else np.full(P, min(Q, 2048))
            if P > 2:
                per_row[1] = 0
                per_row[2] = min(Q, 4)
            row_ptr = np.zeros(P + 1, np.int64)
            np.cumsum(per_row, out=row_ptr[1:])
            nnz = int(row_ptr[-1])
            cols = np.concatenate([np.sort(rng.choice(Q, size=k, replace=False)) for k in per_row] +
                                  [np.zeros(0, np.int64)]).astype(np.int32)
            vals = rng.standard_normal(nnz).astype(np.float32)
            D = synth._finish(torch.from_numpy(rng.standard_normal((Q, N)).astype(np.float32)), dtype)
            # no slack behind the last entry: a quad read must not run past the arrays
            ci_d = torch.from_numpy(cols).cuda() if nnz else torch.zeros(0, dtype=torch.int32, device="cuda")
            cv_d = torch.from_numpy(vals).cuda() if nnz else torch.zeros(0, dtype=torch.float32, device="cuda")
            R = b.fp4_residual_spmm(torch.from_numpy(row_ptr).cuda(), ci_d, cv_d, Q, dev(D, dtype))
            dense = np.zeros((P, Q))
            rows = np.repeat(np.arange(P), per_row)
            dense[rows, cols] = vals
            ref = dense @ D.numpy().astype(np.float64)
            g = R.cpu().numpy().astype(np.float64)
            # sums of up to 2048 fp32 products: against the sum of the magnitudes
            scale = np.abs(dense) @ np.abs(D.numpy().astype(np.float64))
            assert np.all(np.abs(g - ref) <= 3e-5 * scale + 1e-30), "case %d %s" % (ci, dtype)


# ------------------------------------------------------------------------------------------
# DGE
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_dge_apply(dtype):
    g = torch.Generator().manual_seed(13)
    K, N = 200, 264
    W = torch.randn(K, N, generator=g) * 0.02
    # plant scaled weights on grid points, midpoints and the cap boundary (gamma = 1 column)
    W[:16, 0] = torch.tensor([6, .25, .5, .75, 1, 1.25, 2.5, 3, 3.5, 5, 0, 2.516, 2.484, -5, -0.25, 4.99])
    W = synth._finish(W, dtype)     # after planting: host and device must hold the same master values
    G = torch.randn(K, N, generator=g)
    _, gw = o.quantize_cols(W.numpy())
    ref = G.numpy().astype(np.float64) * o.dge_fprime(o.scaled_weights(W.numpy(), gw), 5.0, 3.0)
    got = b.fp4_dge_apply(G.cuda(), dev(W, dtype), torch.from_numpy(gw).cuda(), 5.0, 3.0)
    g64 = got.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(g64 - ref) <= 1e-5 * np.abs(ref) + 1e-12)
    ste = b.fp4_dge_apply(G.cuda(), dev(W, dtype), torch.from_numpy(gw).cuda(), 0.0, 3.0)
    assert torch.equal(ste.cpu(), G)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("k,cap", [(1.0, 3.0), (3.0, 2.0), (7.0, 5.0), (2.0, 0.4), (0.5, 3.0), (5.0, 1e9)])
def test_dge_apply_other_k_and_cap(k, cap, dtype):
    """Eq. 8 away from the defaults: k = 1 (f' = 1 everywhere, interval midpoints included), k below 1
    (f' -> 0 at a midpoint), a cap below 1/k (active everywhere) and a cap that is never active except
    at exact midpoints."""
    g = torch.Generator().manual_seed(int(10 * k) + 3)
    K, N = 136, 72
    W = torch.randn(K, N, generator=g) * 0.02
    W[:18, 0] = torch.tensor([6, .25, .5, .75, 1, 1.25, 2.5, 3, 3.5, 5, 0, 2.516, 2.484, -5, -0.25, 4.99, 1.75, -1.25])
    W = synth._finish(W, dtype)     # after planting: host and device must hold the same master values
    G = torch.randn(K, N, generator=g)
    _, gw = o.quantize_cols(W.numpy())
    fp = o.dge_fprime(o.scaled_weights(W.numpy(), gw), k, cap)
    assert np.isfinite(fp).all()
    ref = G.numpy().astype(np.float64) * fp
    got = b.fp4_dge_apply(G.cuda(), dev(W, dtype), torch.from_numpy(gw).cuda(), k, cap)
    g64 = got.cpu().numpy().astype(np.float64)
    assert np.isfinite(g64).all()
    assert np.all(np.abs(g64 - ref) <= 1e-5 * np.abs(ref) + 1e-12)


@pytest.mark.parametrize("k,cap", [(1.0, 3.0), (3.0, 2.0), (7.0, 5.0)])
def test_layer_wgrad_other_k_and_cap(k, cap):
    """The DGE factor fused in the weight-gradient epilogue at other (k, cap), planted midpoints included."""
    A, W, dY = synth.small_case(288, 160, 264, "bf16", seed=int(k))
    W[:14, 0] = torch.tensor([6, .25, .75, 1.25, 1.75, 2.5, 3.5, 5, -5, -2.5, 1, 2, 3, 4.]).to(torch.bfloat16).float()
    Ad, Wd, dYd = dev(A, "bf16"), dev(W, "bf16"), dev(dY, "bf16")
    _, ctx = b.fp4_linear_fwd(Ad, Wd, 0.98)
    dW = b.fp4_linear_bwd_wgrad(Ad, dYd, Wd, ctx, k, cap)
    assert_close(dW, o.fp4_linear_bwd_wgrad(A.numpy(), dY.numpy(), W.numpy(), 0.98, k, cap), "f32", "dW")


# ------------------------------------------------------------------------------------------
# the layer: forward, dgrad, wgrad
# ------------------------------------------------------------------------------------------
LAYER_CASES = [
    ("c1", 256, 512, 512, "f32", 0.99),
    ("rag", 160, 288, 224, "f32", 0.97),
    ("rag", 288, 544, 1056, "bf16", 0.99),
    ("off", 96, 128, 96, "bf16", 1.0),
    ("tiny", 32, 32, 32, "f32", 0.9),
    ("long", 2304, 64, 96, "bf16", 0.97),     # an outlier channel: a transposed residual row > 2048 entries
    ("wide", 64, 16416, 32, "bf16", 0.98),    # more input channels than the transpose's LDS tables hold
    # several 1024-row blocks and several LDS slabs in both residual products, all of them ragged
    ("blocks", 1120, 1056, 160, "bf16", 0.98),
    ("blocks", 1056, 608, 96, "f32", 0.95),
    ("sparse", 512, 1024, 288, "bf16", 0.999),   # the sparsest operating point of Sec. 4.3 (0.2 % residual)
    ("sparse", 96, 2048, 96, "f32", 0.999),
    ("dense", 256, 256, 160, "bf16", 0.9),       # the densest residual the workspaces provide for
]


def _layer_inputs(name, M, K, N, dtype):
    if name == "c1":
        cfg = synth.CONFIGS["c1"]
        return synth.make_layer(cfg, cfg.layers[0])
    return synth.small_case(M, K, N, dtype, seed=M + K + N)


@pytest.mark.parametrize("name,M,K,N,dtype,alpha", LAYER_CASES)
def test_layer_forward_backward(name, M, K, N, dtype, alpha):
    A, W, dY = _layer_inputs(name, M, K, N, dtype)
    Ad, Wd, dYd = dev(A, dtype), dev(W, dtype), dev(dY, dtype)
    Y, ctx = b.fp4_linear_fwd(Ad, Wd, alpha)
    torch.cuda.synchronize()
    Yref, st = o.fp4_linear_fwd(A.numpy(), W.numpy(), alpha, "f32")
    # saved state: scales, thresholds, residual -- bit exact
    assert np.array_equal(ctx.gamma_W.cpu().numpy().view(np.uint32), st.gamma_w.view(np.uint32))
    if alpha < 1.0:
        thr = ctx.thresholds.cpu().numpy()
        assert thr[0] == st.lo and thr[1] == st.hi
        nnz = int(ctx.nnz.item())
        assert nnz == st.csr.val.size
        assert np.array_equal(ctx.row_ptr.cpu().numpy(), st.csr.row_ptr)
        assert np.array_equal(ctx.col_idx.cpu().numpy()[:nnz], st.csr.col_idx)
        assert np.array_equal(ctx.val.cpu().numpy()[:nnz].view(np.uint32), st.csr.val.view(np.uint32))
    else:
        assert int(ctx.nnz.item()) == 0
    assert_close(Y, Yref, dtype, "Y")

    dA = b.fp4_linear_bwd_dgrad(dYd, Wd)
    assert_close(dA, o.fp4_linear_bwd_dgrad(dY.numpy(), W.numpy(), "f32"), dtype, "dA")

    if M % 32 == 0:
        dW = b.fp4_linear_bwd_wgrad(Ad, dYd, Wd, ctx, 5.0, 3.0)
        assert dW.dtype == torch.float32
        assert_close(dW, o.fp4_linear_bwd_wgrad(A.numpy(), dY.numpy(), W.numpy(), alpha, 5.0, 3.0), "f32", "dW")
        G = b.fp4_linear_bwd_wgrad(Ad, dYd, Wd, ctx, 0.0, 3.0)
        assert_close(G, o.fp4_linear_bwd_wgrad(A.numpy(), dY.numpy(), W.numpy(), alpha, 0.0, 3.0), "f32", "G (STE)")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_layer_with_outlier_tokens(dtype):
    """Two tokens far larger than the rest: nearly all of their elements are clamped, so their rows of
    the residual exceed the long-row threshold of the sparse product in the forward pass (the other
    layer cases only have long rows in the transposed residual of the weight gradient)."""
    M, K, N, alpha = 96, 4160, 96, 0.97
    A, W, dY = synth.small_case(M, K, N, dtype, seed=4160)
    A[5] *= 200.0
    A[77] *= 300.0
    A = synth._finish(A, dtype)
    Ad, Wd, dYd = dev(A, dtype), dev(W, dtype), dev(dY, dtype)
    Y, ctx = b.fp4_linear_fwd(Ad, Wd, alpha)
    torch.cuda.synchronize()
    Yref, st = o.fp4_linear_fwd(A.numpy(), W.numpy(), alpha, "f32")
    per_row = np.diff(st.csr.row_ptr)
    assert per_row[5] > 2048 and per_row[77] > 2048 and np.median(per_row) < 2048
    nnz = int(ctx.nnz.item())
    assert nnz == st.csr.val.size
    assert np.array_equal(ctx.row_ptr.cpu().numpy(), st.csr.row_ptr)
    assert np.array_equal(ctx.col_idx.cpu().numpy()[:nnz], st.csr.col_idx)
    assert np.array_equal(ctx.val.cpu().numpy()[:nnz].view(np.uint32), st.csr.val.view(np.uint32))
    assert_close(Y, Yref, dtype, "Y")
    dA, dW = b.fp4_linear_bwd(dYd, Ad, Wd, ctx, 5.0, 3.0)
    assert_close(dA, o.fp4_linear_bwd_dgrad(dY.numpy(), W.numpy(), "f32"), dtype, "dA")
    assert_close(dW, o.fp4_linear_bwd_wgrad(A.numpy(), dY.numpy(), W.numpy(), alpha, 5.0, 3.0), "f32", "dW")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_cached_weight_quantizations_equal_the_plain_entry_points(dtype):
    """W's two quantizations prepared once: codes and scales bit-exact against the oracle, and forward /
    activation gradient through the cache bit-identical to the entry points that quantize W themselves."""
    A, W, dY = synth.small_case(288, 544, 1056, dtype, seed=12)
    Ad, Wd, dYd = dev(A, dtype), dev(W, dtype), dev(dY, dtype)
    wq = b.fp4_prepare_weights(Wd)
    torch.cuda.synchronize()
    ct, gw = o.quantize_cols(W.numpy())
    ck, gk = o.quantize_rows(W.numpy())
    assert np.array_equal(wq.gamma_W.cpu().numpy().view(np.uint32), gw.view(np.uint32))
    assert np.array_equal(wq.gamma_Wk.cpu().numpy().view(np.uint32), gk.view(np.uint32))
    assert np.array_equal(host_codes(wq.qWt), ct)
    assert np.array_equal(host_codes(wq.qWk), ck)
    Y0, ctx0 = b.fp4_linear_fwd(Ad, Wd, 0.98)
    Y1, ctx1 = b.fp4_linear_fwd_cached(Ad, Wd, wq, 0.98)
    n = int(ctx0.nnz.item())
    assert n == int(ctx1.nnz.item()) > 0
    assert torch.equal(Y0, Y1) and torch.equal(ctx0.gamma_W, ctx1.gamma_W) and torch.equal(ctx0.val[:n], ctx1.val[:n])
    assert torch.equal(b.fp4_linear_bwd_dgrad(dYd, Wd), b.fp4_linear_bwd_dgrad_cached(dYd, wq))
    dW0 = b.fp4_linear_bwd_wgrad(Ad, dYd, Wd, ctx0)
    dW1 = b.fp4_linear_bwd_wgrad(Ad, dYd, Wd, ctx1)
    assert torch.equal(dW0, dW1)


@pytest.mark.parametrize("name,M,K,N,dtype,alpha", [("c1", 256, 512, 512, "f32", 0.99),
                                                     ("rag", 288, 544, 1056, "bf16", 0.99),
                                                     ("long", 2304, 64, 96, "bf16", 0.9),
                                                     ("blocks", 1120, 1056, 160, "bf16", 0.98),
                                                     ("wide", 64, 11008, 32, "bf16", 0.99),
                                                     ("off", 96, 128, 96, "f32", 1.0)])
def test_layer_with_per_token_thresholds(name, M, K, N, dtype, alpha):
    """Forward and weight gradient under the per-token reading of the clamp (the activation gradient does
    not involve the clamp): saved state bit-exact, outputs within tolerance."""
    A, W, dY = _layer_inputs(name, M, K, N, dtype)
    Ad, Wd, dYd = dev(A, dtype), dev(W, dtype), dev(dY, dtype)
    Y, ctx = b.fp4_linear_fwd(Ad, Wd, alpha, scope=b.FP4_OCC_TOKEN)
    torch.cuda.synchronize()
    Yref, st = o.fp4_linear_fwd(A.numpy(), W.numpy(), alpha, "f32", scope="token")
    if alpha < 1.0:
        thr = ctx.thresholds.cpu().numpy().reshape(M, 2)
        assert np.array_equal(thr[:, 0], st.lo) and np.array_equal(thr[:, 1], st.hi)
        nnz = int(ctx.nnz.item())
        assert nnz == st.csr.val.size
        assert np.array_equal(ctx.row_ptr.cpu().numpy(), st.csr.row_ptr)
        assert np.array_equal(ctx.col_idx.cpu().numpy()[:nnz], st.csr.col_idx)
        assert np.array_equal(ctx.val.cpu().numpy()[:nnz].view(np.uint32), st.csr.val.view(np.uint32))
    assert_close(Y, Yref, dtype, "Y (per-token)")
    dW = b.fp4_linear_bwd_wgrad(Ad, dYd, Wd, ctx, 5.0, 3.0)
    assert_close(dW, o.fp4_linear_bwd_wgrad(A.numpy(), dY.numpy(), W.numpy(), alpha, 5.0, 3.0, scope="token"), "f32",
                 "dW (per-token)")


@pytest.mark.parametrize("M,K,N,dtype,alpha", [(288, 544, 1056, "bf16", 0.98), (1120, 1056, 160, "bf16", 0.98),
                                                (64, 128, 16384, "bf16", 0.97), (256, 512, 512, "f32", 0.99),
                                                (96, 128, 96, "bf16", 1.0), (2304, 64, 96, "bf16", 0.97)])
def test_combined_backward_equals_the_two_entry_points(M, K, N, dtype, alpha):
    """fp4_linear_bwd (dY read once for its row-wise codes and its column maxima) against dgrad + wgrad:
    bit-identical, with and without the weight cache; fp32 masters take the unfused passes."""
    A, W, dY = synth.small_case(M, K, N, dtype, seed=M + N)
    Ad, Wd, dYd = dev(A, dtype), dev(W, dtype), dev(dY, dtype)
    _, ctx = b.fp4_linear_fwd(Ad, Wd, alpha)
    dA0 = b.fp4_linear_bwd_dgrad(dYd, Wd)
    dW0 = b.fp4_linear_bwd_wgrad(Ad, dYd, Wd, ctx, 5.0, 3.0)
    dA1, dW1 = b.fp4_linear_bwd(dYd, Ad, Wd, ctx, 5.0, 3.0)
    assert torch.equal(dA0, dA1) and torch.equal(dW0, dW1)
    wq = b.fp4_prepare_weights(Wd)
    dA2, dW2 = b.fp4_linear_bwd(dYd, Ad, Wd, ctx, 5.0, 3.0, wq=wq)
    assert torch.equal(dA0, dA2) and torch.equal(dW0, dW2)
    assert_close(dW1, o.fp4_linear_bwd_wgrad(A.numpy(), dY.numpy(), W.numpy(), alpha, 5.0, 3.0), "f32", "dW")


def test_forward_is_deterministic_and_keeps_guard_bands():
    A, W, _ = synth.small_case(256, 512, 520, "bf16", seed=1)
    Ad, Wd = dev(A, "bf16"), dev(W, "bf16")
    buf = torch.full((256 + 2, 520), 7.0, dtype=torch.bfloat16, device="cuda")
    Y1, _ = b.fp4_linear_fwd(Ad, Wd, 0.99, Y=buf[1:-1])
    Y1 = Y1.clone()
    Y2, _ = b.fp4_linear_fwd(Ad, Wd, 0.99)
    assert torch.equal(Y1, Y2)
    assert torch.all(buf[0] == 7.0) and torch.all(buf[-1] == 7.0)


def _layer_once(Ad, Wd, dYd, alpha, ctx=None, Y=None, dW=None, ws=None):
    Y, ctx = b.fp4_linear_fwd(Ad, Wd, alpha, ctx=ctx, Y=Y, ws=ws)
    dW = b.fp4_linear_bwd_wgrad(Ad, dYd, Wd, ctx, dW=dW, ws=ws)
    return Y, dW


def test_layer_on_a_user_stream_equals_the_default_stream():
    """On a stream of the caller's the results must be the ones of the default stream, bit for bit."""
    A, W, dY = synth.small_case(384, 512, 264, "bf16", seed=4)
    Ad, Wd, dYd = dev(A, "bf16"), dev(W, "bf16"), dev(dY, "bf16")
    Y0, dW0 = _layer_once(Ad, Wd, dYd, 0.98)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        for _ in range(3):   # back to back, sharing one workspace in stream order
            Y1, dW1 = _layer_once(Ad, Wd, dYd, 0.98)
    s.synchronize()
    assert torch.equal(Y0, Y1) and torch.equal(dW0, dW1)


def test_layer_in_a_captured_graph_equals_eager_on_every_replay():
    A, W, dY = synth.small_case(256, 512, 264, "bf16", seed=6)
    Ad, Wd, dYd = dev(A, "bf16"), dev(W, "bf16"), dev(dY, "bf16")
    M, K = Ad.shape
    N = Wd.shape[1]
    ctx = b.FwdCtx(M, K, N, 0.98, Ad.device)
    ws = b.Workspace()
    Yg = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dWg = torch.empty((K, N), dtype=torch.float32, device="cuda")
    _layer_once(Ad, Wd, dYd, 0.98, ctx=ctx, Y=Yg, dW=dWg, ws=ws)   # sizes the workspace
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        _layer_once(Ad, Wd, dYd, 0.98, ctx=ctx, Y=Yg, dW=dWg, ws=ws)
    gen = torch.Generator(device="cuda").manual_seed(9)
    for rep in range(3):
        Ad.copy_((torch.randn(M, K, generator=gen, device="cuda") * (1 + rep)).bfloat16())
        g.replay()
        torch.cuda.synchronize()
        Ye, dWe = _layer_once(Ad, Wd, dYd, 0.98)   # eager, own buffers
        torch.cuda.synchronize()
        assert torch.equal(Yg, Ye) and torch.equal(dWg, dWe), "replay %d" % rep


_CAPTURE_FIRST = r"""
import sys, torch
sys.path.insert(0, %r)
from paper_2501_17116_amd import binding as b, synth
A, W, dY = synth.small_case(256, 512, 264, "bf16", seed=8)
Ad, Wd, dYd = A.cuda().bfloat16(), W.cuda().bfloat16(), dY.cuda().bfloat16()
M, K = Ad.shape; N = Wd.shape[1]
ctx = b.FwdCtx(M, K, N, 0.98, Ad.device)
ws = b.Workspace()
ws.get(max(b.workspace_bytes(b.FP4_OP_FWD, M, K, N, b._dt(Ad)), b.workspace_bytes(b.FP4_OP_WGRAD, M, K, N, b._dt(Ad))))
Yg = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
dWg = torch.empty((K, N), dtype=torch.float32, device="cuda")
torch.cuda.synchronize()
g = torch.cuda.CUDAGraph()
with torch.cuda.graph(g):          # the library's very first call in this process
    b.fp4_linear_fwd(Ad, Wd, 0.98, ctx=ctx, Y=Yg, ws=ws)
    b.fp4_linear_bwd_wgrad(Ad, dYd, Wd, ctx, dW=dWg, ws=ws)
for rep in range(2):
    g.replay()
    torch.cuda.synchronize()
Ye, ctx2 = b.fp4_linear_fwd(Ad, Wd, 0.98)
dWe = b.fp4_linear_bwd_wgrad(Ad, dYd, Wd, ctx2)
torch.cuda.synchronize()
assert torch.equal(Yg, Ye) and torch.equal(dWg, dWe)
print("capture-first ok")
"""


def test_first_call_of_a_process_inside_a_capture():
    """The library keeps no state, so its very first call in a process may be made under stream capture."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", _CAPTURE_FIRST % root], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "capture-first ok" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]
