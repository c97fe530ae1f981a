"""CPU oracle for the FP4 (E2M1) quantized linear layer, forward and backward.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, obviously-correct restatement of
what the paper defines, written with numpy.  It shares no code with the HIP path and
must never be imported by it; only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may call it.

Precision policy
  * Everything that decides an integer (a 4-bit code, a scale's bit pattern, a
    clamp threshold, a residual entry) is computed in IEEE fp32, one rounding per
    stated operation, exactly as the steps are written below.
  * Everything compared under a tolerance (scaled GEMM outputs, gradients, the DGE
    factor) is computed in fp64 from those fp32-decided quantities.

Paper passages followed (arXiv 2501.17116):
  Sec. 2, Eq. 1            absmax scaling, gamma = MAX_fp4 / max|x|, MAX_fp4 = 6
  App. A, format table     the 16 E2M1 bit patterns and their values
  App. A, kernel listing   round-to-nearest by 14 midpoint thresholds, strict '<'
  Sec. 3.1, Eq. 7-8        DGE surrogate f and its derivative f', cap 3.0, k = 5
  Sec. 3.2                 quantile clamp and sparse residual (OCC)
  Sec. 4.1                 A token-wise, W channel-wise scaling
  App. C.2                 scales dequantized after the GEMM; DGE on scaled weights
  App. B                   FLOP model (3.12x / 2.95x)

Readings taken where the paper is silent are listed in the repository's design
document; each function's docstring names the one it uses.

Every function in this file is pinned by tests/test_oracle_*.py to facts fixed by the
paper or by mathematics (printed table, tie rule, closed forms, brute force).  The
accuracy of the *method* (training loss, downstream scores) is parity unpinned: it
needs the authors' data and training runs.
"""
from __future__ import annotations

import math
from typing import NamedTuple, Optional, Tuple

import numpy as np

F32 = np.float32

# ----------------------------------------------------------------------------------
# E2M1 format (App. A, format table).  Code = s e1 e0 m ; magnitude index 0..7.
# ----------------------------------------------------------------------------------
E2M1_MAGNITUDES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=F32)
FP4_MAX = F32(6.0)

# Midpoints between neighbouring signed grid values, ascending (App. A listing).
_SIGNED_GRID = np.array([-6, -4, -3, -2, -1.5, -1, -0.5, 0, 0.5, 1, 1.5, 2, 3, 4, 6], dtype=F32)
_THRESHOLDS = np.array([-5, -3.5, -2.5, -1.75, -1.25, -0.75, -0.25,
                        0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5], dtype=F32)
# signed-grid position (0..14) -> 4-bit code.  Position 7 is zero and always gets
# code 0000 (the listing returns +0.0 there; pattern 1000 is never produced).
_POS_TO_CODE = np.array([15, 14, 13, 12, 11, 10, 9, 0, 1, 2, 3, 4, 5, 6, 7], dtype=np.uint8)


def e2m1_decode(codes: np.ndarray) -> np.ndarray:
    """4-bit codes -> fp32 values (App. A table).  Both 0000 and 1000 decode to 0."""
    codes = np.asarray(codes, dtype=np.uint8)
    mag = E2M1_MAGNITUDES[codes & 7]
    return np.where((codes & 8) != 0, -mag, mag).astype(F32) + F32(0.0)


def q_e2m1_value(v: np.ndarray) -> np.ndarray:
    """Round fp32 values to the E2M1 grid (App. A listing).

    The listing walks the 14 thresholds upward and returns the grid value of the
    first threshold the input is strictly below; if none, 6.  Hence a midpoint goes to
    its upper neighbour (towards +inf) for either sign, values beyond +-6 saturate and
    NaN (every comparison false) gives +6.
    """
    v = np.asarray(v, dtype=F32)
    pos = np.zeros(v.shape, dtype=np.int64)
    for t in _THRESHOLDS:
        pos += ~(v < t)          # thresholds passed before the first 'v < t' holds
    return _SIGNED_GRID[pos]


def q_e2m1(v: np.ndarray) -> np.ndarray:
    """Same rounding, returned as 4-bit codes (uint8, one code per element)."""
    v = np.asarray(v, dtype=F32)
    pos = np.zeros(v.shape, dtype=np.int64)
    for t in _THRESHOLDS:
        pos += ~(v < t)
    return _POS_TO_CODE[pos]


def pack_codes(codes: np.ndarray) -> np.ndarray:
    """[R, C] codes -> [R, C/2] bytes; element 2t in bits 3:0, element 2t+1 in bits 7:4."""
    codes = np.asarray(codes, dtype=np.uint8)
    assert codes.shape[-1] % 2 == 0
    return (codes[..., 0::2] | (codes[..., 1::2] << 4)).astype(np.uint8)


def unpack_codes(packed: np.ndarray) -> np.ndarray:
    packed = np.asarray(packed, dtype=np.uint8)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = packed & 15
    out[..., 1::2] = packed >> 4
    return out


# ----------------------------------------------------------------------------------
# absmax vector-wise quantization (Sec. 2 Eq. 1; Sec. 4.1)
# ----------------------------------------------------------------------------------
def absmax_scale(amax: np.ndarray) -> np.ndarray:
    """gamma = fl32(6 / amax) (Eq. 1).  Reading: gamma = 1 when amax is 0 or when the
    quotient is not finite (all-zero or vanishing vector; the paper is silent)."""
    amax = np.asarray(amax, dtype=F32)
    with np.errstate(divide="ignore", over="ignore", invalid="ignore"):
        g = (FP4_MAX / amax).astype(F32)
    ok = np.isfinite(g) & (amax > 0)
    return np.where(ok, g, F32(1.0)).astype(F32)


def quantize_rows(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """One scale per row: codes[r, c] = Q(fl32(x[r, c] * gamma[r])).  Returns
    (codes [R, C] one per byte, gamma [R] fp32).  Token-wise for activations."""
    x = np.asarray(x, dtype=F32)
    amax = np.max(np.abs(x), axis=1) if x.shape[1] else np.zeros(x.shape[0], F32)
    gamma = absmax_scale(amax)
    scaled = (x * gamma[:, None]).astype(F32)
    return q_e2m1(scaled), gamma


def quantize_cols(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """One scale per column (channel-wise for W[c_i, c_o]).  Codes come back
    TRANSPOSED, [C, R], so the contracted axis is contiguous."""
    x = np.asarray(x, dtype=F32)
    codes_t, gamma = quantize_rows(np.ascontiguousarray(x.T))
    return codes_t, gamma


# ----------------------------------------------------------------------------------
# OCC: quantile clamp + sparse residual (Sec. 3.2)
# ----------------------------------------------------------------------------------
def occ_tail_count(n: int, alpha: float) -> int:
    """Elements allowed in each tail: k = floor((1 - alpha) * n), in fp64."""
    return int(math.floor((1.0 - float(alpha)) * float(n)))


def occ_thresholds(x: np.ndarray, alpha: float) -> Tuple[np.float32, np.float32]:
    """Per-tensor two-sided thresholds as order statistics without interpolation:
    with v sorted ascending, lo = v[k], hi = v[n-1-k] (Sec. 3.2; density 2(1-alpha) in
    App. B fixes the two-sided reading).  alpha = 1 gives (min, max): clamp = identity."""
    flat = np.asarray(x, dtype=F32).ravel()
    n = flat.size
    k = occ_tail_count(n, alpha)
    if not (0 <= 2 * k < n):
        raise ValueError("need 0 <= 2*floor((1-alpha)*n) < n")
    v = np.sort(flat, kind="stable")
    return F32(v[k]), F32(v[n - 1 - k])


def occ_thresholds_per_token(x: np.ndarray, alpha: float) -> Tuple[np.ndarray, np.ndarray]:
    """Second reading of the clamp's scope (Sec. 3.2 never names the axis the quantile is taken
    over): one (lo, hi) pair per token, the order statistics of that row alone, with
    k = floor((1 - alpha) * cols) elements allowed in each tail of every row.  Same two-sided,
    no-interpolation definition as occ_thresholds; the residual density stays 2(1-alpha) and
    every row gets at most 2k entries.  Returns (lo [R], hi [R]) fp32."""
    x = np.asarray(x, dtype=F32)
    cols = x.shape[1]
    k = occ_tail_count(cols, alpha)
    if not (0 <= 2 * k < cols):
        raise ValueError("need 0 <= 2*floor((1-alpha)*cols) < cols")
    v = np.sort(x, axis=1, kind="stable")
    return v[:, k].astype(F32), v[:, cols - 1 - k].astype(F32)


class Csr(NamedTuple):
    row_ptr: np.ndarray  # int64 [R+1]
    col_idx: np.ndarray  # int32 [nnz], ascending inside each row
    val: np.ndarray      # fp32  [nnz]
    shape: Tuple[int, int]

    def to_dense(self, dtype=np.float64) -> np.ndarray:
        d = np.zeros(self.shape, dtype=dtype)
        rows = np.repeat(np.arange(self.shape[0]), np.diff(self.row_ptr))
        d[rows, self.col_idx] = self.val
        return d


def occ_clamp_residual(x: np.ndarray, lo: np.float32, hi: np.float32) -> Tuple[np.ndarray, Csr]:
    """Y_c = clamp(Y, lo, hi); Delta = Y - Y_c kept where the clamp changed the value
    (Sec. 3.2).  val = fl32(x - threshold).  lo, hi: scalars (per-tensor thresholds) or one
    value per row (per-token thresholds)."""
    x = np.asarray(x, dtype=F32)
    lo = np.asarray(lo, dtype=F32)
    hi = np.asarray(hi, dtype=F32)
    if lo.ndim == 1:
        lo, hi = lo[:, None], hi[:, None]
    below = x < lo
    above = x > hi
    xc = np.where(below, lo, np.where(above, hi, x)).astype(F32)
    res = np.where(below, (x - lo).astype(F32), np.where(above, (x - hi).astype(F32), F32(0))).astype(F32)
    mask = below | above
    rows, cols = np.nonzero(mask)            # row-major order: ascending cols in a row
    row_ptr = np.zeros(x.shape[0] + 1, dtype=np.int64)
    np.cumsum(mask.sum(axis=1), out=row_ptr[1:])
    return xc, Csr(row_ptr, cols.astype(np.int32), res[rows, cols].astype(F32), x.shape)


# ----------------------------------------------------------------------------------
# FP4 GEMM (Fig. 2; App. C.2): raw accumulator and scaled result
# ----------------------------------------------------------------------------------
def gemm_acc(codes_l: np.ndarray, codes_rt: np.ndarray) -> np.ndarray:
    """acc[i, j] = sum_k v(codes_l[i, k]) * v(codes_rt[j, k]) in fp64.

    Every product is a multiple of 1/4 bounded by 36, so for any contraction length
    used here the sum is exact in fp64 (and in fp32) whatever the order."""
    a = e2m1_decode(codes_l).astype(np.float64)
    b = e2m1_decode(codes_rt).astype(np.float64)
    return a @ b.T


def dequant_gemm(codes_l, gamma_l, codes_rt, gamma_r) -> np.ndarray:
    """(Q(L) Q(R)) with both scale vectors divided out afterwards (Fig. 2 caption;
    App. C.2, Eq. 16 and the paragraph after it), fp64."""
    acc = gemm_acc(codes_l, codes_rt)
    inv_l = 1.0 / gamma_l.astype(np.float64)
    inv_r = 1.0 / gamma_r.astype(np.float64)
    return acc * inv_l[:, None] * inv_r[None, :]


def round_to_dtype(y: np.ndarray, dtype: str) -> np.ndarray:
    """Single final rounding (nearest, ties to even) of fp64 results to the output
    dtype; returned as fp32 holding exactly the rounded values."""
    y = np.asarray(y, dtype=np.float64)
    if dtype == "f32":
        return y.astype(F32)
    if dtype == "bf16":
        # bf16 = 8 significant bits, exponent range of fp32 (spacing never below 2^-133).
        m, e = np.frexp(np.abs(y))                    # |y| = m * 2^e, m in [0.5, 1)
        e = np.maximum(e, -125)                       # subnormal range: fixed spacing
        q = np.rint(np.ldexp(np.abs(y), 8 - e))       # np.rint rounds half to even
        out = np.copysign(np.ldexp(q, e - 8), y)
        return np.where(np.isfinite(y), out, y).astype(F32)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------------
# DGE (Sec. 3.1 Eq. 7, 8; App. C.2)
# ----------------------------------------------------------------------------------
_INTERVAL_LO = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0])
_INTERVAL_W = np.array([0.5, 0.5, 0.5, 0.5, 1.0, 1.0, 2.0])


def _interval(a: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """E2M1 interval [l, l+delta] containing magnitude a (7 per sign, 14 in all).
    Magnitudes at or above 4 (including a rounding hair above 6) use [4, 6]."""
    idx = np.searchsorted(_INTERVAL_LO[1:], a, side="right")
    return _INTERVAL_LO[idx], _INTERVAL_W[idx]


def dge_f(x: np.ndarray, k: float) -> np.ndarray:
    """Differentiable surrogate of Q on the whole E2M1 range (Eq. 7 applied to each
    interval, mirrored for negative x).  fp64."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    l, d = _interval(a)
    t = 2.0 * (a - l) / d - 1.0
    fa = l + d / 2.0 * (1.0 + np.sign(t) * np.abs(t) ** (1.0 / k))
    return np.sign(x) * fa


def dge_fprime(x: np.ndarray, k: float, cap: Optional[float] = 3.0) -> np.ndarray:
    """f'(x) = (1/k) |2(a-l)/delta - 1|^(1/k - 1), capped (Eq. 8 and the cap stated
    with it).  k <= 0 selects the straight-through estimator f' = 1.  fp64."""
    x = np.asarray(x, dtype=np.float64)
    if k <= 0:
        return np.ones_like(x)
    a = np.abs(x)
    l, d = _interval(a)
    t = np.abs(2.0 * (a - l) / d - 1.0)
    with np.errstate(divide="ignore"):
        fp = (1.0 / k) * t ** (1.0 / k - 1.0)
    if cap is not None:
        fp = np.minimum(fp, cap)
    return fp


def scaled_weights(W: np.ndarray, gamma_w: np.ndarray) -> np.ndarray:
    """W_scaled = fl32(W * sf), sf broadcast over output channels (App. C.2, Eq. 14)."""
    return (np.asarray(W, dtype=F32) * np.asarray(gamma_w, dtype=F32)[None, :]).astype(F32)


# ----------------------------------------------------------------------------------
# Mixed formats (Sec. 4.3 ablations: W4A8 = 4-bit weights with 8-bit activations, W8A4 the
# reverse).  The paper names FP8 without fixing the variant or a rounding rule; reading: the
# OCP E4M3 format (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities, largest
# magnitude 448, subnormal quantum 2^-9), round to nearest with ties to even, sign kept,
# magnitudes above 448 saturate; absmax scaling as Eq. 1 with MAX = 448, vector-wise like FP4.
# ----------------------------------------------------------------------------------
FP8_MAX = F32(448.0)


def q_e4m3(v: np.ndarray) -> np.ndarray:
    """fp32 values -> E4M3 codes (uint8).  Finite inputs."""
    v = np.asarray(v, dtype=F32)
    a = np.abs(v.astype(np.float64))
    _, e = np.frexp(np.maximum(a, 2.0 ** -6))            # a = m * 2^e, m in [0.5, 1)  =>  binade exponent e - 1
    quantum = np.ldexp(1.0, (e - 1) - 3)                  # three mantissa bits; 2^-9 below the smallest normal
    q = np.minimum(np.rint(a / quantum) * quantum, 448.0)   # np.rint: ties to even
    m, e2 = np.frexp(np.where(q >= 2.0 ** -6, q, 1.0))
    normal = (((e2 - 1) + 7).astype(np.int64) << 3) | np.rint((m * 2.0 - 1.0) * 8.0).astype(np.int64)
    sub = np.rint(q * 512.0).astype(np.int64)            # 0..7 in units of 2^-9
    mag = np.where(q >= 2.0 ** -6, normal, sub)
    return (mag | (np.signbit(v).astype(np.int64) << 7)).astype(np.uint8)


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """E4M3 codes -> fp32 values (exact).  The NaN patterns (0x7f, 0xff) are never produced."""
    codes = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    ef, mf = (codes >> 3) & 15, codes & 7
    mag = np.where(ef == 0, mf * 2.0 ** -9, (1.0 + mf / 8.0) * np.exp2(ef.astype(np.float64) - 7.0))
    return np.where(codes & 128, -mag, mag).astype(F32)


def quantize_rows_fp8(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """One scale per row, gamma = fl32(448 / absmax) (1 for a vanishing row), codes = E4M3 of
    fl32(x * gamma)."""
    x = np.asarray(x, dtype=F32)
    amax = np.max(np.abs(x), axis=1) if x.shape[1] else np.zeros(x.shape[0], F32)
    with np.errstate(divide="ignore", over="ignore", invalid="ignore"):
        g = (FP8_MAX / amax).astype(F32)
    gamma = np.where(np.isfinite(g) & (amax > 0), g, F32(1.0)).astype(F32)
    return q_e4m3((x * gamma[:, None]).astype(F32)), gamma


def quantize_cols_fp8(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """One scale per column, codes transposed [C, R] (as quantize_cols)."""
    return quantize_rows_fp8(np.ascontiguousarray(np.asarray(x, dtype=F32).T))


def dequant_gemm_values(vals_l: np.ndarray, gamma_l: np.ndarray, vals_rt: np.ndarray, gamma_r: np.ndarray) -> np.ndarray:
    """(L Rt^T) / (gamma_l gamma_r) for decoded operand values of any format, fp64 (Fig. 2)."""
    acc = vals_l.astype(np.float64) @ vals_rt.astype(np.float64).T
    return acc * (1.0 / gamma_l.astype(np.float64))[:, None] * (1.0 / gamma_r.astype(np.float64))[None, :]


def linear_fwd_mixed(A: np.ndarray, W: np.ndarray, act_fp8: bool, wgt_fp8: bool, alpha: float = 1.0,
                     out_dtype: str = "f32") -> np.ndarray:
    """Forward pass with one operand in FP8 (Sec. 4.3): W4A8 (act_fp8: activations E4M3 per token, no
    clamp -- the ablation isolates the weight side) or W8A4 (wgt_fp8: weights E4M3 per output channel,
    activations FP4 with the clamp and residual of Sec. 3.2)."""
    A = np.asarray(A, dtype=F32)
    W = np.asarray(W, dtype=F32)
    res = None
    if act_fp8:
        if alpha != 1.0:
            raise ValueError("the clamp belongs to 4-bit activations")
        ca, ga = quantize_rows_fp8(A)
        va = e4m3_decode(ca)
    else:
        lo, hi = occ_thresholds(A, alpha)
        Ac, csr = occ_clamp_residual(A, lo, hi)
        ca, ga = quantize_rows(Ac)
        va = e2m1_decode(ca)
        res = csr
    if wgt_fp8:
        cw, gw = quantize_cols_fp8(W)
        vw = e4m3_decode(cw)
    else:
        cw, gw = quantize_cols(W)
        vw = e2m1_decode(cw)
    Y = dequant_gemm_values(va, ga, vw, gw)
    if res is not None and res.val.size:
        Y = Y + res.to_dense() @ W.astype(np.float64)
    return round_to_dtype(Y, out_dtype)


# ----------------------------------------------------------------------------------
# Granularity ablation (Sec. 4.3 "Granularity"; App. C.2: sf a scalar for tensor-wise
# quantization): one scale for the whole tensor instead of one per token / channel.
# ----------------------------------------------------------------------------------
def quantize_tensor(x: np.ndarray) -> Tuple[np.ndarray, np.float32]:
    """Tensor-wise absmax quantization: gamma = fl32(6 / max|x|) for the whole tensor (same
    conventions as absmax_scale), codes[r, c] = Q(fl32(x[r, c] * gamma)).  Returns (codes [R, C],
    gamma as an fp32 scalar)."""
    x = np.asarray(x, dtype=F32)
    amax = np.max(np.abs(x)) if x.size else F32(0.0)
    gamma = absmax_scale(np.asarray(amax, dtype=F32)).reshape(())
    return q_e2m1((x * gamma).astype(F32)), F32(gamma)


def linear_fwd_granularity(A: np.ndarray, W: np.ndarray, act_tensorwise: bool, wgt_tensorwise: bool,
                           alpha: float = 1.0, out_dtype: str = "f32") -> np.ndarray:
    """The forward pass of the granularity ablation: as fp4_linear_fwd, with the scale of the
    activations and / or of the weights taken over the whole (clamped) tensor.  The clamp and the
    residual are those of the per-tensor reading, unchanged."""
    A = np.asarray(A, dtype=F32)
    W = np.asarray(W, dtype=F32)
    lo, hi = occ_thresholds(A, alpha)
    Ac, csr = occ_clamp_residual(A, lo, hi)
    if act_tensorwise:
        ca, g = quantize_tensor(Ac)
        ga = np.full(A.shape[0], g, dtype=F32)
    else:
        ca, ga = quantize_rows(Ac)
    if wgt_tensorwise:
        cw, g = quantize_tensor(W)
        cwt, gw = np.ascontiguousarray(cw.T), np.full(W.shape[1], g, dtype=F32)
    else:
        cwt, gw = quantize_cols(W)
    Y = dequant_gemm(ca, ga, cwt, gw)
    if csr.val.size:
        Y = Y + csr.to_dense() @ W.astype(np.float64)
    return round_to_dtype(Y, out_dtype)


# ----------------------------------------------------------------------------------
# The other two 4-bit formats of App. A's format table (E1M2, E3M0): grids only, for the
# format comparison of Sec. 4.3 on the CPU; no kernel uses them.
# ----------------------------------------------------------------------------------
FP4_GRIDS = {
    "e1m2": np.array([0.0, 0.5, 1.0, 1.5, 2.0, 2.5, 3.0, 3.5], dtype=F32),
    "e2m1": E2M1_MAGNITUDES,
    "e3m0": np.array([0.0, 0.25, 0.5, 1.0, 2.0, 4.0, 8.0, 16.0], dtype=F32),
}


def quantize_rows_grid(x: np.ndarray, fmt: str) -> Tuple[np.ndarray, np.ndarray]:
    """Row-wise absmax quantization to one of the 4-bit grids: gamma = fl32(MAX_fmt / absmax) (Eq. 1
    with the format's largest magnitude), then the nearest grid value with a midpoint going to its
    upper neighbour, as the App. A listing does for E2M1.  Returns (grid VALUES [R, C], gamma [R])."""
    x = np.asarray(x, dtype=F32)
    mags = FP4_GRIDS[fmt]
    grid = np.concatenate([-mags[:0:-1], mags]).astype(F32)            # 15 signed values, ascending
    mids = ((grid[:-1].astype(np.float64) + grid[1:]) / 2).astype(F32)   # exact in fp32
    amax = np.max(np.abs(x), axis=1) if x.shape[1] else np.zeros(x.shape[0], F32)
    with np.errstate(divide="ignore", over="ignore", invalid="ignore"):
        g = (mags[-1] / amax).astype(F32)
    gamma = np.where(np.isfinite(g) & (amax > 0), g, F32(1.0)).astype(F32)
    scaled = (x * gamma[:, None]).astype(F32)
    pos = np.zeros(scaled.shape, dtype=np.int64)
    for t in mids:
        pos += ~(scaled < t)
    return grid[pos] + F32(0.0), gamma


# ----------------------------------------------------------------------------------
# The linear layer: forward, dgrad, wgrad
# ----------------------------------------------------------------------------------
class FwdState(NamedTuple):
    lo: np.float32        # scalars (per-tensor thresholds) or vectors over tokens (per-token)
    hi: np.float32
    csr: Csr
    gamma_a: np.ndarray
    gamma_w: np.ndarray
    codes_a: np.ndarray   # [M, K]
    codes_wt: np.ndarray  # [N, K]


def _thresholds(A: np.ndarray, alpha: float, scope: str):
    if scope == "tensor":
        return occ_thresholds(A, alpha)
    if scope == "token":
        return occ_thresholds_per_token(A, alpha)
    raise ValueError(scope)


def fp4_linear_fwd(A: np.ndarray, W: np.ndarray, alpha: float, out_dtype: str = "f32",
                   rows: Optional[np.ndarray] = None, scope: str = "tensor") -> Tuple[np.ndarray, FwdState]:
    """Y = dequant(Q(A_c) Q(W)) + Delta_A W   (Fig. 2; Sec. 3.2; App. C.2).

    A_c is A clamped at the per-tensor thresholds and quantized token-wise, W is
    quantized per output channel, the residual uses the unquantized W in fp64.
    `rows` restricts the output to a subset of tokens (thresholds and column scales
    still come from the full tensors) so large shapes can be checked by sampling.
    scope = "token" takes the per-token reading of the thresholds (then lo, hi in the
    returned state are vectors over all tokens)."""
    A = np.asarray(A, dtype=F32)
    W = np.asarray(W, dtype=F32)
    lo, hi = _thresholds(A, alpha, scope)
    codes_wt, gamma_w = quantize_cols(W)
    A_sel = A if rows is None else A[rows]
    if scope == "token" and rows is not None:
        Ac, csr = occ_clamp_residual(A_sel, lo[rows], hi[rows])
    else:
        Ac, csr = occ_clamp_residual(A_sel, lo, hi)
    codes_a, gamma_a = quantize_rows(Ac)
    Y = dequant_gemm(codes_a, gamma_a, codes_wt, gamma_w)
    if csr.val.size:
        Y = Y + csr.to_dense() @ W.astype(np.float64)
    return round_to_dtype(Y, out_dtype), FwdState(lo, hi, csr, gamma_a, gamma_w, codes_a, codes_wt)


def fp4_linear_bwd_dgrad(dY: np.ndarray, W: np.ndarray, out_dtype: str = "f32",
                         rows: Optional[np.ndarray] = None) -> np.ndarray:
    """dA = dY W^T as an FP4 GEMM contracting over output channels: dY scaled per
    token, W per input channel (scales on the non-contracted axes, Sec. 4.1)."""
    dY = np.asarray(dY, dtype=F32)
    W = np.asarray(W, dtype=F32)
    d_sel = dY if rows is None else dY[rows]
    codes_d, gamma_d = quantize_rows(d_sel)
    codes_w, gamma_wk = quantize_rows(W)           # [K, N], one scale per input channel
    return round_to_dtype(dequant_gemm(codes_d, gamma_d, codes_w, gamma_wk), out_dtype)


def fp4_linear_bwd_wgrad(A: np.ndarray, dY: np.ndarray, W: np.ndarray, alpha: float,
                         dge_k: float = 5.0, dge_cap: float = 3.0,
                         rows: Optional[np.ndarray] = None, scope: str = "tensor") -> np.ndarray:
    """dW = (A^T dY) (.) f'(W_scaled)   (Sec. 3.1 Eq. 3-6; App. C.2 Eq. 22).

    A^T dY is an FP4 GEMM contracting over tokens: clamped A scaled per input channel,
    dY per output channel, plus Delta_A^T dY in fp64.  f' is evaluated on
    W * gamma_W with the forward's per-output-channel scales.  `rows` selects input
    channels (rows of dW).  Result fp32."""
    A = np.asarray(A, dtype=F32)
    dY = np.asarray(dY, dtype=F32)
    W = np.asarray(W, dtype=F32)
    lo, hi = _thresholds(A, alpha, scope)
    Ac, csr = occ_clamp_residual(A, lo, hi)
    if rows is not None:
        Ac_sel = Ac[:, rows]
    else:
        Ac_sel = Ac
    codes_at, gamma_ak = quantize_cols(Ac_sel)      # [K', M]
    codes_dt, gamma_dn = quantize_cols(dY)          # [N, M]
    G = dequant_gemm(codes_at, gamma_ak, codes_dt, gamma_dn)
    if csr.val.size:
        dT = csr.to_dense().T                       # [K, M]
        if rows is not None:
            dT = dT[rows]
        G = G + dT @ dY.astype(np.float64)
    _, gamma_w = quantize_cols(W)
    Ws = scaled_weights(W, gamma_w)
    if rows is not None:
        Ws = Ws[rows]
    return round_to_dtype(G * dge_fprime(Ws, dge_k, dge_cap), "f32")


# ----------------------------------------------------------------------------------
# Fidelity metrics (Table 1 columns) and the App. B FLOP model
# ----------------------------------------------------------------------------------
def fidelity(x: np.ndarray, xq: np.ndarray) -> Tuple[float, float, float]:
    """(cosine similarity, MSE, SNR in dB) between a tensor and its reconstruction."""
    x = np.asarray(x, dtype=np.float64).ravel()
    xq = np.asarray(xq, dtype=np.float64).ravel()
    cos = float(x @ xq / (np.linalg.norm(x) * np.linalg.norm(xq)))
    mse = float(np.mean((x - xq) ** 2))
    snr = float(10.0 * np.log10(np.sum(x ** 2) / np.sum((x - xq) ** 2)))
    return cos, mse, snr


def dequantized_activation(x: np.ndarray, alpha: Optional[float], compensate: bool,
                           scope: str = "tensor") -> np.ndarray:
    """Reconstruction of an activation tensor after token-wise FP4 quantization, with
    optional clamp and optional residual added back (the three rows of Table 1)."""
    x = np.asarray(x, dtype=F32)
    if alpha is None:
        xc, res = x, None
    else:
        lo, hi = _thresholds(x, alpha, scope)
        xc, csr = occ_clamp_residual(x, lo, hi)
        res = csr.to_dense() if compensate else None
    codes, gamma = quantize_rows(xc)
    rec = e2m1_decode(codes).astype(np.float64) / gamma.astype(np.float64)[:, None]
    return rec if res is None else rec + res


def appendix_b_speedup(h: int, s: int, alpha: Optional[float] = None) -> float:
    """Theoretical per-layer speed-up of App. B.  alpha=None: ideal (no overhead).
    With alpha: DGE (+32 in the denominator) and OCC overhead.  The printed OCC term
    24(1-alpha)h does not reproduce the printed 2.95x / 5.6 %; 48(1-alpha)h (the
    residual costed against the table's own 24bsh^2 total) does, and is used here."""
    num = 24.0 * h + 5.0 * s + 36.0
    den = 6.0 * h + 5.0 * s + 36.0
    if alpha is not None:
        den += 48.0 * (1.0 - alpha) * h + 32.0
    return num / den


def appendix_b_overheads(h: int, s: int, alpha: float) -> Tuple[float, float]:
    base = 6.0 * h + 5.0 * s + 36.0
    return 32.0 / base, 48.0 * (1.0 - alpha) * h / base
