"""Whole-layer pins: the oracle's forward / dgrad / wgrad against a from-the-equations
evaluation in pure Python on tiny shapes, plus method-level sanity and App. B."""
import math

import numpy as np

from oracle import fp4_oracle as o

F32 = np.float32
GRID15 = [-6, -4, -3, -2, -1.5, -1, -0.5, 0, 0.5, 1, 1.5, 2, 3, 4, 6]
INTERVALS = [(0, .5), (.5, 1), (1, 1.5), (1.5, 2), (2, 3), (3, 4), (4, 6)]


def f32(x):
    return float(F32(x))


def q_near(v):
    best = None
    for g in GRID15:
        d = abs(v - g)
        if best is None or d < best[0] or (d == best[0] and g > best[1]):
            best = (d, g)
    return best[1]


def quant_vec(vec):
    """Eq. 1 on one vector: returns (grid values, gamma)."""
    amax = max(abs(v) for v in vec)
    gamma = f32(F32(6.0) / F32(amax)) if amax > 0 else 1.0
    return [q_near(f32(F32(v) * F32(gamma))) for v in vec], gamma


def thresholds(flat, alpha):
    s = sorted(flat)
    k = int(math.floor((1.0 - alpha) * len(s)))
    return s[k], s[len(s) - 1 - k]


def fprime(x, k, cap):
    a = abs(x)
    for l, r in INTERVALS:
        if a < r or (l, r) == INTERVALS[-1]:
            t = abs(2 * (a - l) / (r - l) - 1)
            return cap if t == 0 else min(cap, (1 / k) * t ** (1 / k - 1))


def brute_layer(A, W, dY, alpha, k, cap, scope="tensor"):
    M, K = len(A), len(A[0])
    N = len(W[0])
    if scope == "tensor":
        lo, hi = thresholds([v for r in A for v in r], alpha)
        Ac = [[min(max(v, lo), hi) for v in r] for r in A]
    else:   # one pair of order statistics per token
        Ac = []
        for r in A:
            lo, hi = thresholds(list(r), alpha)
            Ac.append([min(max(v, lo), hi) for v in r])
    dA_res = [[f32(F32(A[i][c]) - F32(Ac[i][c])) if A[i][c] != Ac[i][c] else 0.0 for c in range(K)]
              for i in range(M)]
    # forward
    qa = [quant_vec(Ac[i]) for i in range(M)]
    qw = [quant_vec([W[c][j] for c in range(K)]) for j in range(N)]
    Y = [[sum(qa[i][0][c] * qw[j][0][c] for c in range(K)) / (qa[i][1] * qw[j][1])
          + sum(dA_res[i][c] * W[c][j] for c in range(K)) for j in range(N)] for i in range(M)]
    # dgrad: dY per token, W per input channel
    qd = [quant_vec(dY[i]) for i in range(M)]
    qwk = [quant_vec(W[c]) for c in range(K)]
    dA = [[sum(qd[i][0][j] * qwk[c][0][j] for j in range(N)) / (qd[i][1] * qwk[c][1])
           for c in range(K)] for i in range(M)]
    # wgrad: A_c per input channel, dY per output channel, residual, DGE factor
    qat = [quant_vec([Ac[i][c] for i in range(M)]) for c in range(K)]
    qdt = [quant_vec([dY[i][j] for i in range(M)]) for j in range(N)]
    dW = [[(sum(qat[c][0][i] * qdt[j][0][i] for i in range(M)) / (qat[c][1] * qdt[j][1])
            + sum(dA_res[i][c] * dY[i][j] for i in range(M)))
           * (1.0 if k <= 0 else fprime(f32(F32(W[c][j]) * F32(qw[j][1])), k, cap))
           for j in range(N)] for c in range(K)]
    return np.array(Y), np.array(dA), np.array(dW)


def _case(seed, M, K, N):
    rng = np.random.default_rng(seed)
    A = rng.normal(size=(M, K)).astype(F32)
    A[:, 1] *= 15
    W = (rng.normal(size=(K, N)) * 0.02).astype(F32)
    dY = (rng.normal(size=(M, N)) * 0.01).astype(F32)
    return A, W, dY


def test_tiny_layers_from_the_equations():
    for seed, (M, K, N), alpha in ((0, (6, 8, 5), 0.9), (1, (8, 8, 7), 0.95), (2, (3, 10, 4), 1.0)):
        A, W, dY = _case(seed, M, K, N)
        Yb, dAb, dWb = brute_layer(A.tolist(), W.tolist(), dY.tolist(), alpha, 5.0, 3.0)
        Y, st = o.fp4_linear_fwd(A, W, alpha, "f32")
        dA = o.fp4_linear_bwd_dgrad(dY, W, "f32")
        dW = o.fp4_linear_bwd_wgrad(A, dY, W, alpha, 5.0, 3.0)
        assert Y.shape == (M, N) and dA.shape == (M, K) and dW.shape == (K, N)
        assert np.allclose(Y, Yb, rtol=1e-6, atol=1e-9)
        assert np.allclose(dA, dAb, rtol=1e-6, atol=1e-12)
        assert np.allclose(dW, dWb, rtol=1e-6, atol=1e-12)
        if alpha < 1.0:
            assert st.csr.val.size == 2 * o.occ_tail_count(M * K, alpha) > 0


def test_tiny_layers_from_the_equations_per_token_thresholds():
    for seed, (M, K, N), alpha in ((0, (6, 16, 5), 0.9), (1, (8, 24, 7), 0.95), (2, (3, 10, 4), 1.0)):
        A, W, dY = _case(seed, M, K, N)
        Yb, dAb, dWb = brute_layer(A.tolist(), W.tolist(), dY.tolist(), alpha, 5.0, 3.0, scope="token")
        Y, st = o.fp4_linear_fwd(A, W, alpha, "f32", scope="token")
        dW = o.fp4_linear_bwd_wgrad(A, dY, W, alpha, 5.0, 3.0, scope="token")
        assert np.allclose(Y, Yb, rtol=1e-6, atol=1e-9)
        assert np.allclose(dW, dWb, rtol=1e-6, atol=1e-12)
        if alpha < 1.0:
            assert np.all(np.diff(st.csr.row_ptr) == 2 * o.occ_tail_count(K, alpha))
        rows = np.array([0, M - 1])
        Ys, _ = o.fp4_linear_fwd(A, W, alpha, "f32", rows=rows, scope="token")
        assert np.array_equal(Y[rows], Ys)


def test_row_sampling_matches_full_evaluation():
    A, W, dY = _case(3, 32, 64, 24)
    rows = np.array([0, 5, 31])
    Y, _ = o.fp4_linear_fwd(A, W, 0.98, "f32")
    Ys, _ = o.fp4_linear_fwd(A, W, 0.98, "f32", rows=rows)
    assert np.array_equal(Y[rows], Ys)
    assert np.array_equal(o.fp4_linear_bwd_dgrad(dY, W, "bf16")[rows],
                          o.fp4_linear_bwd_dgrad(dY, W, "bf16", rows=rows))
    ks = np.array([1, 2, 63])
    assert np.array_equal(o.fp4_linear_bwd_wgrad(A, dY, W, 0.98)[ks],
                          o.fp4_linear_bwd_wgrad(A, dY, W, 0.98, rows=ks))


def test_ste_switch_and_dge_factor_range():
    A, W, dY = _case(4, 16, 32, 8)
    G = o.fp4_linear_bwd_wgrad(A, dY, W, 0.97, dge_k=0.0)
    dW = o.fp4_linear_bwd_wgrad(A, dY, W, 0.97, dge_k=5.0, dge_cap=3.0)
    ratio = dW[G != 0].astype(np.float64) / G[G != 0]
    assert np.all(ratio >= 0.2 * (1 - 1e-5)) and np.all(ratio <= 3.0 * (1 + 1e-5))


def test_forward_tracks_the_unquantized_product():
    # sanity on the method: with OCC the FP4 layer stays close to A W (outlier channels
    # would otherwise wreck token-wise quantization, Sec. 3.2)
    rng = np.random.default_rng(5)
    A = rng.normal(size=(128, 256)).astype(F32)
    A[:, [3, 99]] *= 30
    W = (rng.normal(size=(256, 64)) * 0.02).astype(F32)
    ref = A.astype(np.float64) @ W.astype(np.float64)
    err = lambda y: np.linalg.norm(y - ref) / np.linalg.norm(ref)
    e_occ = err(o.fp4_linear_fwd(A, W, 0.99)[0])
    e_plain = err(o.fp4_linear_fwd(A, W, 1.0)[0])
    assert e_occ < 0.2 and e_occ < e_plain


def test_appendix_b_printed_numbers(golden):
    g = dict((r[0], float(r[1])) for r in golden("appendix_b.txt"))
    assert round(o.appendix_b_speedup(4096, 2048), 2) == g["ideal_speedup"]
    assert round(o.appendix_b_speedup(4096, 2048, 0.99), 2) == g["adjusted_speedup"]
    dge, occ = o.appendix_b_overheads(4096, 2048, 0.99)
    assert round(dge * 100, 1) == g["dge_overhead_percent"]
    assert round(occ * 100, 1) == g["occ_overhead_percent"]
