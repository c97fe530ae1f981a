"""Pins for the differentiable gradient estimator (Sec. 3.1 Eq. 7-8; App. C)."""
import numpy as np

from oracle import fp4_oracle as o

INTERVALS = [(0, .5), (.5, 1), (1, 1.5), (1.5, 2), (2, 3), (3, 4), (4, 6)]


def test_printed_hyperparameters(golden):
    g = dict((r[0], float(r[1])) for r in golden("appendix_b.txt"))
    assert g["dge_k"] == 5 and g["dge_cap"] == 3.0 and g["fp4_max"] == 6.0
    assert len(INTERVALS) * 2 == 14           # "14 distinct quantization intervals"


def test_f_endpoints_midpoints_symmetry():
    k = 5.0
    for l, r in INTERVALS:
        d = r - l
        assert o.dge_f(np.array([float(l)]), k)[0] == l          # grid points are fixed points
        assert o.dge_f(np.array([float(r)]), k)[0] == r
        assert np.isclose(o.dge_f(np.array([l + d / 2]), k)[0], l + d / 2)
        assert np.isclose(o.dge_f(np.array([r - 1e-12]), k)[0], r, atol=1e-2 * d)
        # central symmetry about the midpoint: f(mid + u) + f(mid - u) = 2 mid
        u = np.linspace(0.01, 0.49, 7) * d
        s = o.dge_f(l + d / 2 + u, k) + o.dge_f(l + d / 2 - u, k)
        assert np.allclose(s, 2 * l + d)
    x = np.linspace(-5.9, 5.9, 101)
    assert np.allclose(o.dge_f(-x, k), -o.dge_f(x, k))           # odd in x
    # first positive interval, k = 5: the closed form of Eq. 7 written out
    x = np.array([0.1, 0.2, 0.3, 0.45])
    t = 2 * x / 0.5 - 1
    assert np.allclose(o.dge_f(x, k), 0.25 * (1 + np.sign(t) * np.abs(t) ** 0.2))
    # larger k approaches the hard step
    assert abs(o.dge_f(np.array([0.3]), 50.0)[0] - 0.5) < abs(o.dge_f(np.array([0.3]), 5.0)[0] - 0.5)


def test_fprime_is_the_derivative_of_f():
    for k in (3.0, 5.0, 7.0):
        for sign in (1, -1):
            for l, r in INTERVALS:
                d = r - l
                for frac in (0.05, 0.2, 0.35, 0.65, 0.8, 0.95):
                    x = sign * (l + frac * d)
                    h = 1e-7 * d
                    fd = (o.dge_f(np.array([x + h]), k)[0] - o.dge_f(np.array([x - h]), k)[0]) / (2 * h)
                    fp = o.dge_fprime(np.array([x]), k, cap=None)[0]
                    assert np.isclose(fd, fp, rtol=1e-5), (k, x, fd, fp)


def test_fprime_spot_values_and_cap():
    k, cap = 5.0, 3.0
    grid = np.array([0, .5, 1, 1.5, 2, 3, 4, 6, -0.5, -6])
    assert np.allclose(o.dge_fprime(grid, k, cap), 1 / k)        # |t| = 1 at grid points
    mids = np.array([.25, .75, 1.25, 1.75, 2.5, 3.5, 5.0, -2.5])
    assert np.all(o.dge_fprime(mids, k, cap) == cap)             # t = 0 -> inf -> cap
    assert np.all(np.isinf(o.dge_fprime(mids, k, None)))
    # cap active exactly for |t| < (1/(cap k))^(k/(k-1)) = 0.033876...
    tc = (1.0 / (cap * k)) ** (k / (k - 1))
    assert abs(tc - 0.033876) < 1e-6
    for l, r in INTERVALS:
        d = r - l
        inside = l + d / 2 * (1 + 0.99 * tc)
        outside = l + d / 2 * (1 + 1.01 * tc)
        assert o.dge_fprime(np.array([inside]), k, cap)[0] == cap
        assert o.dge_fprime(np.array([outside]), k, cap)[0] < cap
    # closed form on [2, 3]: x = 2.8 -> t = 0.6
    assert np.isclose(o.dge_fprime(np.array([2.8]), k, cap)[0], 0.2 * 0.6 ** (-0.8))
    # a hair above 6 keeps the [4, 6] formula
    assert np.isclose(o.dge_fprime(np.array([6.000001]), k, cap)[0], 0.2, rtol=1e-5)
    # STE switch
    assert np.all(o.dge_fprime(np.array([0.3, 2.5, -4]), 0.0, cap) == 1.0)


def test_scale_cancellation_long_way_equals_short_way():
    # App. C.2: (dL/dWq (.) 1/sf (.) Q'(W_scaled)) (.) sf == dL/dWq (.) Q'(W_scaled)
    rng = np.random.default_rng(0)
    W = (rng.normal(size=(16, 6)) * 0.02).astype(np.float32)
    G = rng.normal(size=(16, 6))
    _, sf = o.quantize_cols(W)
    Ws = o.scaled_weights(W, sf)
    assert Ws.dtype == np.float32 and np.abs(Ws).max() <= 6.0 * (1 + 2 ** -22)
    qp = o.dge_fprime(Ws, 5.0, 3.0)
    long_way = (G * (1.0 / sf.astype(np.float64))[None, :] * qp) * sf.astype(np.float64)[None, :]
    assert np.allclose(long_way, G * qp, rtol=1e-14)
    # every column's absmax sits on the grid point 6 -> factor 1/k there
    j = np.abs(W).argmax(axis=0)
    assert np.allclose(qp[j, np.arange(6)], 0.2, rtol=1e-4)
