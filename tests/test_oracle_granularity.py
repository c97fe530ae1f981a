"""Pins of the oracle's granularity ablation (tensor-wise scaling, Sec. 4.3 "Granularity"; App. C.2)
and of the other two 4-bit grids of App. A's format table."""
import math

import numpy as np

from oracle import fp4_oracle as o

F32 = np.float32
GRID15 = [-6, -4, -3, -2, -1.5, -1, -0.5, 0, 0.5, 1, 1.5, 2, 3, 4, 6]


def f32(x):
    return float(F32(x))


def q_near(v, grid=GRID15):
    best = None
    for g in grid:
        d = abs(v - g)
        if best is None or d < best[0] or (d == best[0] and g > best[1]):
            best = (d, g)
    return best[1]


def test_tensorwise_hand_example_and_conventions():
    x = np.array([[3.0, -1.5], [0.75, 0.2]], dtype=F32)
    codes, g = o.quantize_tensor(x)                       # absmax 3 -> gamma 2 -> 6, -3, 1.5, 0.4
    assert g == F32(2.0)
    assert np.array_equal(o.e2m1_decode(codes), np.array([[6.0, -3.0], [1.5, 0.5]], dtype=F32))
    assert np.array_equal(codes, np.array([[7, 13], [3, 1]], dtype=np.uint8))
    z, gz = o.quantize_tensor(np.zeros((3, 4), dtype=F32))
    assert gz == F32(1.0) and not z.any()
    e, ge = o.quantize_tensor(np.zeros((0, 4), dtype=F32))
    assert ge == F32(1.0) and e.shape == (0, 4)


def test_tensorwise_scale_properties():
    rng = np.random.default_rng(3)
    x = (rng.normal(size=(37, 50)) * np.exp(rng.normal(size=(37, 1)) * 2)).astype(F32)
    codes, g = o.quantize_tensor(x)
    amax = np.abs(x).max()
    assert abs(float(g) * float(amax) - 6.0) <= 6.0 * 2.0 ** -23
    r, c = np.unravel_index(np.abs(x).argmax(), x.shape)
    assert codes[r, c] & 7 == 7                           # the largest element lands on +-6
    assert (codes & 7).max() == 7
    # one scale: scaling the tensor by a power of two changes gamma, not the codes
    c2, g2 = o.quantize_tensor(x * F32(0.125))
    assert np.array_equal(c2, codes) and g2 == g * F32(8.0)
    # element by element from the definition, in pure Python
    for (i, j) in [(0, 0), (5, 7), (36, 49), (r, c)]:
        want = q_near(f32(F32(x[i, j]) * g))
        assert float(o.e2m1_decode(codes[i:i + 1, j:j + 1])[0, 0]) == want
    # rows that all have the same absmax: the two granularities coincide
    y = x / np.abs(x).max(axis=1, keepdims=True)
    y = (y * F32(4.0)).astype(F32)
    y[np.arange(37), np.abs(y).argmax(axis=1)] = F32(4.0)
    ct, gt = o.quantize_tensor(y)
    cr, gr = o.quantize_rows(y)
    assert np.array_equal(ct, cr) and np.all(gr == gt)


def test_tensorwise_loses_the_small_rows_vectorwise_keeps():
    # the granularity finding of Sec. 4.3 in miniature: tokens of very different magnitude under one scale
    rng = np.random.default_rng(4)
    x = rng.normal(size=(64, 128)).astype(F32)
    x[:8] *= 100.0
    ct, gt = o.quantize_tensor(x)
    cr, gr = o.quantize_rows(x)
    rec_t = o.e2m1_decode(ct).astype(np.float64) / float(gt)
    rec_r = o.e2m1_decode(cr).astype(np.float64) / gr.astype(np.float64)[:, None]
    small = slice(8, None)
    assert not rec_t[small].any()                         # every small token is flushed to zero
    mse = lambda r: float(np.mean((r[small] - x[small]) ** 2))
    assert mse(rec_r) < 0.05 * mse(rec_t)


def _brute_forward(A, W, act_t, wgt_t, alpha):
    M, K = len(A), len(A[0])
    N = len(W[0])
    flat = sorted(v for r in A for v in r)
    k = int(math.floor((1.0 - alpha) * len(flat)))
    lo, hi = flat[k], flat[len(flat) - 1 - k]
    Ac = [[min(max(v, lo), hi) for v in r] for r in A]
    res = [[f32(F32(A[i][c]) - F32(Ac[i][c])) if A[i][c] != Ac[i][c] else 0.0 for c in range(K)] for i in range(M)]

    def scale(vals):
        amax = max(abs(v) for v in vals)
        return f32(F32(6.0) / F32(amax)) if amax > 0 else 1.0
    ga = [scale([v for r in Ac for v in r])] * M if act_t else [scale(r) for r in Ac]
    gw = [scale([v for r in W for v in r])] * N if wgt_t else [scale([W[c][j] for c in range(K)]) for j in range(N)]
    qa = [[q_near(f32(F32(Ac[i][c]) * F32(ga[i]))) for c in range(K)] for i in range(M)]
    qw = [[q_near(f32(F32(W[c][j]) * F32(gw[j]))) for c in range(K)] for j in range(N)]
    return np.array([[sum(qa[i][c] * qw[j][c] for c in range(K)) / (ga[i] * gw[j])
                      + sum(res[i][c] * W[c][j] for c in range(K)) for j in range(N)] for i in range(M)])


def test_granularity_forward_from_the_definitions():
    rng = np.random.default_rng(6)
    A = rng.normal(size=(6, 8)).astype(F32)
    A[:, 2] *= 12
    A[4] *= 0.05
    W = (rng.normal(size=(8, 5)) * 0.02).astype(F32)
    W[:, 1] *= 30
    for alpha in (1.0, 0.9):
        outs = {}
        for act_t in (False, True):
            for wgt_t in (False, True):
                Y = o.linear_fwd_granularity(A, W, act_t, wgt_t, alpha)
                Yb = _brute_forward(A.tolist(), W.tolist(), act_t, wgt_t, alpha)
                assert np.allclose(Y, Yb, rtol=1e-6, atol=1e-9), (act_t, wgt_t, alpha)
                outs[(act_t, wgt_t)] = Y
        # vector-wise on both sides is the layer's ordinary forward pass
        assert np.array_equal(outs[(False, False)], o.fp4_linear_fwd(A, W, alpha)[0])
        assert not np.array_equal(outs[(True, False)], outs[(False, False)])
        assert not np.array_equal(outs[(False, True)], outs[(False, False)])


def test_printed_grids_of_the_other_formats(golden):
    rows = golden("fp4_formats_table.txt")
    for fmt in ("e1m2", "e3m0"):
        vals = {r[1]: float(r[2]) for r in rows if r[0] == fmt}
        assert len(vals) == 15
        mags = o.FP4_GRIDS[fmt]
        for idx in range(8):
            assert vals["0" + format(idx, "03b")] == float(mags[idx])
            if idx:
                assert vals["1" + format(idx, "03b")] == -float(mags[idx])
    # structure of the three formats: 1 / 2 / 3 exponent bits
    assert np.all(np.diff(o.FP4_GRIDS["e1m2"]) == 0.5)                       # uniform: one binade and subnormals
    assert np.all(o.FP4_GRIDS["e3m0"][2:] / o.FP4_GRIDS["e3m0"][1:-1] == 2)  # powers of two
    assert np.array_equal(o.FP4_GRIDS["e2m1"], o.E2M1_MAGNITUDES)


def test_rowwise_quantization_to_a_grid():
    rng = np.random.default_rng(8)
    x = (rng.normal(size=(9, 40)) * np.exp(rng.normal(size=(9, 1)))).astype(F32)
    x[3] = 0.0
    for fmt in ("e1m2", "e2m1", "e3m0"):
        mags = [float(v) for v in o.FP4_GRIDS[fmt]]
        grid = sorted(set([-m for m in mags] + mags))
        vals, gamma = o.quantize_rows_grid(x, fmt)
        assert gamma[3] == 1.0 and not vals[3].any()
        for i in (0, 1, 8):
            amax = float(np.abs(x[i]).max())
            assert abs(float(gamma[i]) * amax - mags[-1]) <= mags[-1] * 2.0 ** -23
            assert np.abs(vals[i]).max() == mags[-1]
            for j in range(40):
                assert float(vals[i, j]) == q_near(f32(F32(x[i, j]) * gamma[i]), grid), (fmt, i, j)
    # ties go up for either sign, on every grid
    for fmt, tie, up in (("e1m2", 0.25, 0.5), ("e1m2", -0.25, 0.0), ("e3m0", 0.375, 0.5), ("e3m0", -12.0, -8.0)):
        top = float(o.FP4_GRIDS[fmt][-1])
        v, g = o.quantize_rows_grid(np.array([[top, tie]], dtype=F32), fmt)
        assert g[0] == 1.0 and float(v[0, 1]) == up
    # E2M1 through the generic routine is the path's own quantizer
    v, g = o.quantize_rows_grid(x, "e2m1")
    c, g2 = o.quantize_rows(x)
    assert np.array_equal(v, o.e2m1_decode(c)) and np.array_equal(g, g2)
