"""Pins for absmax vector-wise quantization (Sec. 2 Eq. 1; Sec. 4.1)."""
import numpy as np

from oracle import fp4_oracle as o

F32 = np.float32


def test_hand_worked_rows():
    # amax 6 -> gamma 1: values already on/near the grid
    c, g = o.quantize_rows(np.array([[6, 3, -1.5, 0.2, -0.3, 2.4, -5.1, 0.0]], F32))
    assert g.tolist() == [1.0]
    assert c.tolist() == [[7, 5, 11, 0, 9, 4, 15, 0]]
    # amax 3 -> gamma 2
    c, g = o.quantize_rows(np.array([[3, 1.5, -0.75, 0.1]], F32))
    assert g.tolist() == [2.0]
    assert c.tolist() == [[7, 5, 11, 0]]     # 6, 3, -1.5, 0.2 -> 0


def test_scale_definition_and_absmax_code():
    rng = np.random.default_rng(0)
    x = (rng.normal(size=(64, 96)) * np.exp(rng.normal(size=(64, 1)) * 3)).astype(F32)
    codes, gamma = o.quantize_rows(x)
    amax = np.abs(x).max(axis=1)
    assert np.array_equal(gamma, (F32(6.0) / amax).astype(F32))
    # gamma * amax within one fp32 ulp of 6 (two roundings)
    prod = gamma.astype(np.float64) * amax.astype(np.float64)
    assert np.all(np.abs(prod - 6.0) <= 6.0 * 2.0 ** -23)
    # the absmax element quantizes to magnitude 6
    j = np.abs(x).argmax(axis=1)
    assert np.all((codes[np.arange(64), j] & 7) == 7)
    # reconstruction error bounded by half the widest interval in scaled units
    rec = o.e2m1_decode(codes) / gamma[:, None]
    assert np.all(np.abs(rec - x) * gamma[:, None] <= 1.0 + 1e-5)


def test_power_of_two_invariance():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(16, 64)).astype(F32)
    c1, g1 = o.quantize_rows(x)
    c2, g2 = o.quantize_rows(x * F32(8.0))
    assert np.array_equal(c1, c2)
    assert np.array_equal(g1, g2 * F32(8.0))


def test_zero_and_vanishing_rows():
    x = np.zeros((3, 8), F32)
    x[1, 2] = 1e-44          # subnormal: 6/amax overflows -> gamma 1
    x[2, 5] = -2.0
    codes, gamma = o.quantize_rows(x)
    assert gamma.tolist() == [1.0, 1.0, 3.0]
    assert not codes[0].any() and not codes[1].any()
    assert codes[2].tolist() == [0, 0, 0, 0, 0, 15, 0, 0]


def test_cols_is_rows_of_transpose_and_transposed_layout():
    rng = np.random.default_rng(2)
    w = rng.normal(size=(12, 5)).astype(F32)
    ct, g = o.quantize_cols(w)
    assert ct.shape == (5, 12) and g.shape == (5,)
    for j in range(5):
        cj, gj = o.quantize_rows(w[:, j][None, :].copy())
        assert np.array_equal(ct[j], cj[0]) and g[j] == gj[0]
    # scales belong to columns: scaling one column changes only that gamma
    w2 = w.copy()
    w2[:, 3] *= 4
    ct2, g2 = o.quantize_cols(w2)
    assert np.array_equal(ct, ct2) and g2[3] == g[3] / 4 and np.array_equal(np.delete(g, 3), np.delete(g2, 3))
