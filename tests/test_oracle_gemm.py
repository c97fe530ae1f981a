"""Pins for the FP4 GEMM accumulator and its scale dequantization (Fig. 2; App. C.2)."""
from fractions import Fraction

import numpy as np

from oracle import fp4_oracle as o

F32 = np.float32
VAL = {c: Fraction(float(o.e2m1_decode(np.array([c], np.uint8))[0])) for c in range(16)}


def test_accumulator_bruteforce_exact_rational():
    rng = np.random.default_rng(0)
    M, K, N = 5, 12, 7                       # non-square: a transposed operand cannot pass
    ca = rng.integers(0, 16, (M, K)).astype(np.uint8)
    cb = rng.integers(0, 16, (N, K)).astype(np.uint8)
    acc = o.gemm_acc(ca, cb)
    assert acc.shape == (M, N)
    for i in range(M):
        for j in range(N):
            s = sum(VAL[int(ca[i, k])] * VAL[int(cb[j, k])] for k in range(K))
            assert Fraction(float(acc[i, j])) == s


def test_accumulator_is_exact_multiple_of_quarter_and_fits_fp32():
    rng = np.random.default_rng(1)
    K = 16384
    ca = rng.integers(0, 16, (4, K)).astype(np.uint8)
    cb = rng.integers(0, 16, (3, K)).astype(np.uint8)
    acc = o.gemm_acc(ca, cb)
    assert np.array_equal(acc * 4, np.round(acc * 4))
    assert np.all(np.abs(acc) <= 36 * K)
    assert np.array_equal(acc.astype(F32).astype(np.float64), acc)     # exact in fp32
    # integer reference: 2*value is an integer, so 4*acc is an integer matmul
    ia = (o.e2m1_decode(ca) * 2).astype(np.int64)
    ib = (o.e2m1_decode(cb) * 2).astype(np.int64)
    assert np.array_equal((ia @ ib.T), (acc * 4).astype(np.int64))


def test_grid_operands_with_unit_scale_reduce_to_plain_matmul():
    rng = np.random.default_rng(2)
    grid = np.array([-6, -4, -3, -2, -1.5, -1, -.5, 0, .5, 1, 1.5, 2, 3, 4, 6], F32)
    A = rng.choice(grid, size=(6, 16)).astype(F32)
    W = rng.choice(grid, size=(16, 9)).astype(F32)
    A[:, 0] = 6                                # every row / column has absmax 6 -> gamma 1
    W[0, :] = -6
    ca, ga = o.quantize_rows(A)
    cw, gw = o.quantize_cols(W)
    assert np.all(ga == 1) and np.all(gw == 1)
    Y = o.dequant_gemm(ca, ga, cw, gw)
    assert np.array_equal(Y, A.astype(np.float64) @ W.astype(np.float64))


def test_scales_are_divided_out_on_the_right_axes():
    # hand example: A = [[3, 1.5]] (gamma 2 -> codes 6, 3), W = [[1], [0.5]] (gamma 6 -> 6, 3)
    A = np.array([[3, 1.5]], F32)
    W = np.array([[1.0], [0.5]], F32)
    ca, ga = o.quantize_rows(A)
    cw, gw = o.quantize_cols(W)
    assert ga.tolist() == [2.0] and gw.tolist() == [6.0]
    assert o.gemm_acc(ca, cw).tolist() == [[45.0]]            # 6*6 + 3*3
    assert o.dequant_gemm(ca, ga, cw, gw).tolist() == [[45.0 / 12.0]]   # = 3*1 + 1.5*0.5
    # per-row and per-column scaling commute with the GEMM
    rng = np.random.default_rng(3)
    A = rng.normal(size=(7, 32)).astype(F32)
    W = rng.normal(size=(32, 5)).astype(F32)
    ca, ga = o.quantize_rows(A)
    cw, gw = o.quantize_cols(W)
    Aq = o.e2m1_decode(ca).astype(np.float64) / ga[:, None]
    Wq = (o.e2m1_decode(cw).astype(np.float64) / gw[:, None]).T
    assert np.allclose(o.dequant_gemm(ca, ga, cw, gw), Aq @ Wq, rtol=1e-13, atol=0)
