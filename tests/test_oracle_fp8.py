"""Pins for the FP8 (E4M3) side of the mixed-format ablations (Sec. 4.3): the format's defining
constants, an independent library cast, brute-force nearest-neighbour rounding, and the mixed
forward pass against a from-the-definitions evaluation."""
import numpy as np
import torch

from oracle import fp4_oracle as o

F32 = np.float32


def test_format_constants_and_decode():
    d = o.e4m3_decode(np.arange(256, dtype=np.uint8))
    assert d[0x38] == 1.0 and d[0x7E] == 448.0 and d[0x08] == 2.0 ** -6 and d[0x01] == 2.0 ** -9 and d[0x00] == 0.0
    assert d[0x30] == 0.5 and d[0x39] == 1.125 and d[0x40] == 2.0 and d[0xB8] == -1.0 and d[0xFE] == -448.0
    mags = d[:0x7F]                                   # 127 finite non-negative values, strictly increasing
    assert np.all(np.diff(mags) > 0)
    # sign / exponent / mantissa decomposition, written out independently
    for c in range(0x7F):
        e, m = c >> 3, c & 7
        v = m / 8 * 2.0 ** -6 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7)
        assert float(d[c]) == v and float(d[c | 0x80]) == -v


def test_rounding_equals_an_independent_cast_and_nearest_neighbour():
    rng = np.random.default_rng(0)
    grid = o.e4m3_decode(np.arange(0x7F, dtype=np.uint8)).astype(np.float64)
    mids = (grid[:-1] + grid[1:]) / 2
    pts = np.concatenate([grid, mids, np.nextafter(mids.astype(F32), F32(np.inf)), np.nextafter(mids.astype(F32), F32(-np.inf)),
                          rng.uniform(-450, 450, 200000), rng.normal(size=200000) * 0.01, rng.normal(size=200000) * 1e-3,
                          [0.0, -0.0, 448.0, -448.0, 463.9]]).astype(F32)
    pts = np.concatenate([pts, -pts])
    codes = o.q_e4m3(pts)
    ref = torch.from_numpy(pts).to(torch.float8_e4m3fn).view(torch.uint8).numpy()   # nearest-even, in range
    assert np.array_equal(codes, ref)
    # nearest neighbour by brute force, ties to the even mantissa
    sub = pts[:4000]
    dist = np.abs(np.abs(sub.astype(np.float64))[:, None] - grid[None, :])
    best = dist.min(axis=1)
    for i in range(sub.size):
        cand = np.nonzero(dist[i] == best[i])[0]
        pick = cand[0] if cand.size == 1 else [c for c in cand if c % 2 == 0][0]
        assert (codes[i] & 0x7F) == pick
    # saturation: beyond the range the magnitude stays 448 (the library cast would give NaN there)
    assert o.q_e4m3(np.array([1e9, -1e9, 470.0], F32)).tolist() == [0x7E, 0xFE, 0x7E]
    # idempotent
    assert np.array_equal(o.q_e4m3(o.e4m3_decode(codes)), codes)


def test_rowwise_scaling_hits_the_format_maximum():
    rng = np.random.default_rng(1)
    x = (rng.normal(size=(50, 96)) * np.exp(rng.normal(size=(50, 1)) * 3)).astype(F32)
    x[3] = 0
    codes, gamma = o.quantize_rows_fp8(x)
    assert gamma[3] == 1.0 and np.all(codes[3] == 0)
    amax = np.abs(x).max(axis=1)
    ok = amax > 0
    assert np.all(np.abs(gamma[ok].astype(np.float64) * amax[ok] - 448.0) <= 448.0 * 2.0 ** -23)
    assert np.all((codes[ok] & 0x7F).max(axis=1) == 0x7E)
    c2, g2 = o.quantize_rows_fp8(x * F32(8))                       # power-of-two invariance
    assert np.array_equal(c2, codes) and np.array_equal(g2[ok] * F32(8), gamma[ok])
    ct, gt = o.quantize_cols_fp8(x)
    cr, gr = o.quantize_rows_fp8(np.ascontiguousarray(x.T))
    assert np.array_equal(ct, cr) and np.array_equal(gt, gr)
    # relative rounding error of a normal-range value: at most 2^-4
    rec = o.e4m3_decode(codes).astype(np.float64) / gamma[:, None]
    big = np.abs(x) > amax[:, None] * 2.0 ** -10
    assert np.all(np.abs(rec - x)[big] <= 2.0 ** -4 * np.abs(x)[big] * (1 + 1e-6))


def _brute_mixed(A, W, act_fp8, wgt_fp8):
    grid8 = [float(v) for v in o.e4m3_decode(np.arange(0x7F, dtype=np.uint8))]
    grid4 = [0, .5, 1, 1.5, 2, 3, 4, 6]

    def near(v, grid, even_ties):
        a = abs(v)
        best = min(range(len(grid)), key=lambda i: (abs(a - grid[i]), (i % 2) if even_ties else -i))
        return grid[best] if v >= 0 else -grid[best]

    def q4(v):   # App. A: ties towards +inf
        cands = sorted(set([-g for g in grid4] + grid4))
        return min(cands, key=lambda g: (abs(v - g), -g))

    def quant(vec, fp8):
        amax = max(abs(t) for t in vec)
        mx = 448.0 if fp8 else 6.0
        gamma = float(F32(F32(mx) / F32(amax))) if amax > 0 else 1.0
        sc = [float(F32(F32(t) * F32(gamma))) for t in vec]
        return ([near(t, grid8, True) for t in sc] if fp8 else [q4(t) for t in sc]), gamma

    M, K = A.shape
    N = W.shape[1]
    qa = [quant(A[i].tolist(), act_fp8) for i in range(M)]
    qw = [quant(W[:, j].tolist(), wgt_fp8) for j in range(N)]
    return np.array([[sum(qa[i][0][c] * qw[j][0][c] for c in range(K)) / (qa[i][1] * qw[j][1]) for j in range(N)]
                     for i in range(M)])


def test_mixed_forward_from_the_definitions():
    rng = np.random.default_rng(2)
    A = rng.normal(size=(5, 16)).astype(F32)
    W = (rng.normal(size=(16, 6)) * 0.02).astype(F32)
    for act8, wgt8 in ((True, False), (False, True)):
        Y = o.linear_fwd_mixed(A, W, act8, wgt8, 1.0)
        assert np.allclose(Y, _brute_mixed(A, W, act8, wgt8), rtol=1e-6, atol=1e-12)
    # an 8-bit operand is closer to the unquantized product than a 4-bit one (why the ablation is run)
    A = rng.normal(size=(64, 256)).astype(F32)
    W = (rng.normal(size=(256, 48)) * 0.02).astype(F32)
    ref = A.astype(np.float64) @ W.astype(np.float64)
    err = lambda y: np.linalg.norm(y - ref) / np.linalg.norm(ref)
    e44 = err(o.fp4_linear_fwd(A, W, 1.0)[0])
    assert err(o.linear_fwd_mixed(A, W, True, False)) < e44 and err(o.linear_fwd_mixed(A, W, False, True)) < e44
    # W8A4 keeps the clamp and its residual
    A[:, 3] *= 40
    lo, hi = o.occ_thresholds(A, 0.98)
    Ac, csr = o.occ_clamp_residual(A, lo, hi)
    Y = o.linear_fwd_mixed(A, W, False, True, 0.98)
    Y0 = o.linear_fwd_mixed(Ac, W, False, True, 1.0)
    # (both sides carry one fp32 rounding, of different magnitudes where the two terms cancel)
    assert np.allclose(Y, Y0 + csr.to_dense() @ W.astype(np.float64), rtol=1e-6, atol=1e-6 * np.abs(Y0).max())
