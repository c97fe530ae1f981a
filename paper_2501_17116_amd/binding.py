"""ctypes binding of libfp4mi.so: argument marshalling only.

Every function here has the name and the meaning of the C entry point it calls
(include/fp4_linear.h); torch supplies device memory and the current HIP stream,
nothing else.  There is no fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfp4mi.so")

FP4_F32, FP4_BF16 = 0, 1
FP4_AXIS_ROW, FP4_AXIS_COL, FP4_AXIS_TENSOR = 0, 1, 2
FP4_OCC_TENSOR, FP4_OCC_TOKEN = 0, 1
FP4_OP_QUANTIZE, FP4_OP_OCC, FP4_OP_FWD, FP4_OP_DGRAD, FP4_OP_WGRAD, FP4_OP_SPMM, FP4_OP_PREPARE, FP4_OP_FWD_MIXED, FP4_OP_BWD = range(9)
FP4_FMT_E2M1, FP4_FMT_E4M3 = 0, 1

_lib = None


class Fp4Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, status_string(status), status))


class fp4_fwd_ctx(C.Structure):
    _fields_ = [("gamma_W", C.c_void_p), ("thresholds", C.c_void_p), ("row_ptr", C.c_void_p),
                ("col_idx", C.c_void_p), ("val", C.c_void_p), ("capacity", C.c_int64),
                ("nnz", C.c_void_p), ("scope", C.c_int32)]


class fp4_weight_cache(C.Structure):
    _fields_ = [("qWt", C.c_void_p), ("gamma_W", C.c_void_p), ("qWk", C.c_void_p), ("gamma_Wk", C.c_void_p)]


def lib() -> C.CDLL:
    """The native library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("native library %s not built: run `python -c 'import __graft_entry__ as g; "
                               "g.build()'` (needs hipcc)" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        vp, i64, f32, f64, sz, i32 = C.c_void_p, C.c_int64, C.c_float, C.c_double, C.c_size_t, C.c_int
        L.fp4_status_string.restype = C.c_char_p
        L.fp4_status_string.argtypes = [i32]
        L.fp4_workspace_bytes.restype = sz
        L.fp4_workspace_bytes.argtypes = [i32, i64, i64, i64, i32]
        L.fp4_occ_capacity.restype = i64
        L.fp4_occ_capacity.argtypes = [i64, i64, f64]
        L.fp4_quantize.argtypes = [vp, i32, i64, i64, i64, i32, vp, vp, vp, sz, vp]
        L.fp4_quantize_noalloc.argtypes = [vp, i32, i64, i64, i64, i32, vp, vp, vp]
        L.fp4_quantize_noalloc.restype = i32
        L.occ_clamp_residual.argtypes = [vp, i32, i64, i64, i64, f64, vp, vp, vp, vp, vp, vp, vp, i64, vp,
                                         vp, sz, vp]
        L.occ_clamp_residual_token.argtypes = L.occ_clamp_residual.argtypes
        L.occ_clamp_residual_token.restype = i32
        L.fp4_occ_capacity_token.restype = i64
        L.fp4_occ_capacity_token.argtypes = [i64, i64, f64]
        L.fp4_linear_fwd.argtypes = [vp, vp, i32, i64, i64, i64, f64, vp, C.POINTER(fp4_fwd_ctx), vp, sz, vp]
        L.fp4_linear_bwd_dgrad.argtypes = [vp, vp, i32, i64, i64, i64, vp, vp, sz, vp]
        L.fp4_linear_bwd_wgrad.argtypes = [vp, vp, vp, i32, i64, i64, i64, C.POINTER(fp4_fwd_ctx), f32, f32,
                                           vp, vp, sz, vp]
        L.fp4_prepare_weights.argtypes = [vp, i32, i64, i64, C.POINTER(fp4_weight_cache), vp, sz, vp]
        L.fp4_linear_fwd_cached.argtypes = [vp, vp, C.POINTER(fp4_weight_cache), i32, i64, i64, i64, f64, vp,
                                            C.POINTER(fp4_fwd_ctx), vp, sz, vp]
        L.fp4_linear_bwd_dgrad_cached.argtypes = [vp, C.POINTER(fp4_weight_cache), i32, i64, i64, i64, vp, vp, sz, vp]
        for name in ("fp4_prepare_weights", "fp4_linear_fwd_cached", "fp4_linear_bwd_dgrad_cached"):
            getattr(L, name).restype = i32
        L.fp4_linear_bwd.argtypes = [vp, vp, vp, C.POINTER(fp4_weight_cache), i32, i64, i64, i64, C.POINTER(fp4_fwd_ctx),
                                     f32, f32, vp, vp, vp, sz, vp]
        L.fp4_linear_bwd.restype = i32
        L.fp8_quantize.argtypes = [vp, i32, i64, i64, i64, i32, vp, vp, vp, sz, vp]
        L.fp4_gemm_mixed.argtypes = [vp, i32, vp, vp, i32, vp, i64, i64, i64, vp, vp, i32, i64, vp]
        L.fp4_linear_fwd_mixed.argtypes = [vp, vp, i32, i64, i64, i64, i32, i32, f64, vp, C.POINTER(fp4_fwd_ctx), vp, sz, vp]
        L.fp4_linear_fwd_granularity.argtypes = [vp, vp, i32, i64, i64, i64, i32, i32, f64, vp, C.POINTER(fp4_fwd_ctx), vp, sz,
                                                 vp]
        L.fp4_linear_fwd_granularity.restype = i32
        L.fp8_host_round_codes.argtypes = [vp, i64, vp]
        for name in ("fp8_quantize", "fp4_gemm_mixed", "fp4_linear_fwd_mixed", "fp8_host_round_codes"):
            getattr(L, name).restype = i32
        L.fp4_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp, i32, i64, vp]
        L.fp4_unpack.argtypes = [vp, i64, i64, vp, vp]
        L.fp4_dge_apply.argtypes = [vp, vp, i32, vp, i64, i64, f32, f32, vp, vp]
        L.fp4_residual_spmm.argtypes = [vp, vp, vp, i64, i64, vp, i32, i64, vp, vp, sz, vp]
        L.fp4_host_round_codes.argtypes = [vp, i64, vp]
        L.fp4_device_round_codes.argtypes = [vp, i64, vp, vp]
        L.fp4_device_round_sweep.argtypes = [vp, vp]
        L.fp4_probe_mfma.argtypes = [vp, i64, i32, i32, vp, vp]
        L.fp4_probe_mfma.restype = i32
        L.fp4_probe_copy.argtypes = [vp, vp, i64, vp]
        L.fp4_probe_copy.restype = i32
        L.fp4_trace_begin.argtypes = [i32]
        L.fp4_trace_begin.restype = i32
        L.fp4_trace_end.argtypes = [vp, vp, i32]
        L.fp4_trace_end.restype = i32
        for name in ("fp4_quantize", "occ_clamp_residual", "fp4_linear_fwd", "fp4_linear_bwd_dgrad",
                     "fp4_linear_bwd_wgrad", "fp4_gemm", "fp4_unpack", "fp4_dge_apply", "fp4_residual_spmm",
                     "fp4_host_round_codes", "fp4_device_round_codes", "fp4_device_round_sweep"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().fp4_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise Fp4Error(status, where)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FP4_F32
    if t.dtype == torch.bfloat16:
        return FP4_BF16
    raise TypeError("dtype must be float32 or bfloat16, got %s" % t.dtype)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_check(*ts):
    for t in ts:
        if t is not None:
            if not t.is_cuda:
                raise ValueError("tensors must live on the GPU")
            if not t.is_contiguous():
                raise ValueError("tensors must be contiguous")


def workspace_bytes(op: int, M: int, K: int, N: int, dt: int) -> int:
    return int(lib().fp4_workspace_bytes(op, M, K, N, dt))


def occ_capacity(rows: int, cols: int, alpha: float) -> int:
    return int(lib().fp4_occ_capacity(rows, cols, float(alpha)))


class Workspace:
    """A growable device byte buffer handed to the entry points as their workspace.

    One Workspace serves calls that stream order serializes (the ABI's workspace rule): use one
    per stream.  Growing keeps the outgrown buffers alive until release(), because kernels
    enqueued earlier may still be running in them and torch's allocator knows nothing of
    streams other than the one a tensor was allocated on."""

    def __init__(self, device="cuda"):
        self.device = device
        self.buf = torch.empty(0, dtype=torch.uint8, device=device)
        self._outgrown = []

    def get(self, nbytes: int) -> torch.Tensor:
        if self.buf.numel() < nbytes:
            if self.buf.numel():
                self._outgrown.append(self.buf)
            self.buf = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        return self.buf

    def release(self) -> None:
        """Drop outgrown buffers; call after the streams that used them have been synchronized."""
        self._outgrown.clear()


_default_ws = {}   # (device index, stream handle) -> Workspace: never shared between streams


def _ws(nbytes: int, ws: Optional[Workspace]) -> torch.Tensor:
    if ws is None:
        key = (torch.cuda.current_device(), torch.cuda.current_stream().cuda_stream)
        ws = _default_ws.get(key)
        if ws is None:
            ws = _default_ws[key] = Workspace()
    return ws.get(nbytes)


class FwdCtx:
    """Device buffers the forward pass fills for the weight-gradient pass."""

    def __init__(self, M: int, K: int, N: int, alpha: float, device="cuda", scope: int = FP4_OCC_TENSOR):
        cap = occ_capacity(M, K, alpha) if alpha < 1.0 else 0
        self.alpha = float(alpha)
        self.scope = scope
        self.gamma_W = torch.empty(N, dtype=torch.float32, device=device)
        self.thresholds = torch.empty(2 * M if scope == FP4_OCC_TOKEN else 2, dtype=torch.float32, device=device)
        self.row_ptr = torch.empty(M + 1, dtype=torch.int64, device=device)
        self.col_idx = torch.empty(max(cap, 1), dtype=torch.int32, device=device)
        self.val = torch.empty(max(cap, 1), dtype=torch.float32, device=device)
        self.nnz = torch.zeros(1, dtype=torch.int64, device=device)
        self.capacity = cap
        self.c = fp4_fwd_ctx(self.gamma_W.data_ptr(), self.thresholds.data_ptr(), self.row_ptr.data_ptr(),
                             self.col_idx.data_ptr(), self.val.data_ptr(), cap, self.nnz.data_ptr(), scope)


def fp4_quantize(x: torch.Tensor, axis: int, ws: Optional[Workspace] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    _dev_check(x)
    rows, cols = x.shape
    if axis == FP4_AXIS_ROW:
        codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
        gamma = torch.empty(rows, dtype=torch.float32, device=x.device)
    elif axis == FP4_AXIS_TENSOR:   # one scale for the whole tensor, codes laid out as for ROW
        codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
        gamma = torch.empty(1, dtype=torch.float32, device=x.device)
    else:
        codes = torch.empty((cols, rows // 2), dtype=torch.uint8, device=x.device)
        gamma = torch.empty(cols, dtype=torch.float32, device=x.device)
    nb = workspace_bytes(FP4_OP_QUANTIZE, rows, cols, 0, _dt(x))
    w = _ws(nb, ws)
    _check(lib().fp4_quantize(_ptr(x), _dt(x), rows, cols, cols, axis, _ptr(codes), _ptr(gamma), _ptr(w),
                              w.numel(), _stream()), "fp4_quantize")
    return codes, gamma


def fp4_quantize_noalloc(x: torch.Tensor, axis: int, codes: torch.Tensor, gamma: torch.Tensor) -> None:
    """fp4_quantize without a workspace, into outputs the caller brings (nothing is allocated)."""
    _dev_check(x, codes, gamma)
    rows, cols = x.shape
    _check(lib().fp4_quantize_noalloc(_ptr(x), _dt(x), rows, cols, cols, axis, _ptr(codes), _ptr(gamma),
                                      _stream()), "fp4_quantize_noalloc")


def occ_clamp_residual(x: torch.Tensor, alpha: float, want_codes: bool = True, want_clamped: bool = False,
                       capacity: Optional[int] = None, ws: Optional[Workspace] = None,
                       scope: int = FP4_OCC_TENSOR) -> dict:
    _dev_check(x)
    rows, cols = x.shape
    token = scope == FP4_OCC_TOKEN
    if capacity is not None:
        cap = capacity
    elif token:
        cap = int(lib().fp4_occ_capacity_token(rows, cols, float(alpha)))
    else:
        cap = occ_capacity(rows, cols, alpha)
    dev = x.device
    out = {
        "thresholds": torch.empty(2 * rows if token else 2, dtype=torch.float32, device=dev),
        "codes": torch.empty((rows, cols // 2), dtype=torch.uint8, device=dev) if want_codes else None,
        "gamma": torch.empty(rows, dtype=torch.float32, device=dev) if want_codes else None,
        "x_clamped": torch.empty_like(x) if want_clamped else None,
        "row_ptr": torch.empty(rows + 1, dtype=torch.int64, device=dev),
        "col_idx": torch.empty(max(cap, 1), dtype=torch.int32, device=dev),
        "val": torch.empty(max(cap, 1), dtype=torch.float32, device=dev),
        "nnz": torch.zeros(1, dtype=torch.int64, device=dev),
    }
    nb = workspace_bytes(FP4_OP_OCC, rows, cols, 0, _dt(x))
    w = _ws(nb, ws)
    fn = lib().occ_clamp_residual_token if token else lib().occ_clamp_residual
    _check(fn(_ptr(x), _dt(x), rows, cols, cols, float(alpha), _ptr(out["thresholds"]),
                                    _ptr(out["codes"]), _ptr(out["gamma"]), _ptr(out["x_clamped"]),
                                    _ptr(out["row_ptr"]), _ptr(out["col_idx"]), _ptr(out["val"]), cap,
                                    _ptr(out["nnz"]), _ptr(w), w.numel(), _stream()), "occ_clamp_residual")
    return out


def fp4_linear_fwd(A: torch.Tensor, W: torch.Tensor, alpha: float, ctx: Optional[FwdCtx] = None,
                   Y: Optional[torch.Tensor] = None, ws: Optional[Workspace] = None, scope: int = FP4_OCC_TENSOR):
    """scope only matters when no ctx is passed (a ctx carries its own)."""
    _dev_check(A, W, Y)
    M, K = A.shape
    K2, N = W.shape
    if K2 != K or A.dtype != W.dtype:
        raise ValueError("A [M,K] and W [K,N] must agree in K and dtype")
    if ctx is None:
        ctx = FwdCtx(M, K, N, alpha, A.device, scope)
    if Y is None:
        Y = torch.empty((M, N), dtype=A.dtype, device=A.device)
    nb = workspace_bytes(FP4_OP_FWD, M, K, N, _dt(A))
    w = _ws(nb, ws)
    _check(lib().fp4_linear_fwd(_ptr(A), _ptr(W), _dt(A), M, K, N, float(alpha), _ptr(Y), C.byref(ctx.c),
                                _ptr(w), w.numel(), _stream()), "fp4_linear_fwd")
    return Y, ctx


class WeightCache:
    """Device buffers for W's two quantizations (forward's per-output-channel, dgrad's per-input-channel)."""

    def __init__(self, K: int, N: int, device="cuda"):
        self.K, self.N = K, N
        self.qWt = torch.empty((N, K // 2), dtype=torch.uint8, device=device)
        self.gamma_W = torch.empty(N, dtype=torch.float32, device=device)
        self.qWk = torch.empty((K, N // 2), dtype=torch.uint8, device=device)
        self.gamma_Wk = torch.empty(K, dtype=torch.float32, device=device)
        self.c = fp4_weight_cache(self.qWt.data_ptr(), self.gamma_W.data_ptr(), self.qWk.data_ptr(),
                                  self.gamma_Wk.data_ptr())


def fp4_prepare_weights(W: torch.Tensor, wq: Optional[WeightCache] = None, ws: Optional[Workspace] = None) -> WeightCache:
    _dev_check(W)
    K, N = W.shape
    if wq is None:
        wq = WeightCache(K, N, W.device)
    w = _ws(workspace_bytes(FP4_OP_PREPARE, 0, K, N, _dt(W)), ws)
    _check(lib().fp4_prepare_weights(_ptr(W), _dt(W), K, N, C.byref(wq.c), _ptr(w), w.numel(), _stream()),
           "fp4_prepare_weights")
    return wq


def fp4_linear_fwd_cached(A: torch.Tensor, W: torch.Tensor, wq: WeightCache, alpha: float,
                          ctx: Optional[FwdCtx] = None, Y: Optional[torch.Tensor] = None,
                          ws: Optional[Workspace] = None):
    _dev_check(A, W, Y)
    M, K = A.shape
    K2, N = W.shape
    if K2 != K or A.dtype != W.dtype or (wq.K, wq.N) != (K, N):
        raise ValueError("A [M,K], W [K,N] and the weight cache must agree")
    if ctx is None:
        ctx = FwdCtx(M, K, N, alpha, A.device)
    if Y is None:
        Y = torch.empty((M, N), dtype=A.dtype, device=A.device)
    w = _ws(workspace_bytes(FP4_OP_FWD, M, K, N, _dt(A)), ws)
    _check(lib().fp4_linear_fwd_cached(_ptr(A), _ptr(W), C.byref(wq.c), _dt(A), M, K, N, float(alpha), _ptr(Y),
                                       C.byref(ctx.c), _ptr(w), w.numel(), _stream()), "fp4_linear_fwd_cached")
    return Y, ctx


def fp4_linear_bwd_dgrad_cached(dY: torch.Tensor, wq: WeightCache, dA: Optional[torch.Tensor] = None,
                                ws: Optional[Workspace] = None) -> torch.Tensor:
    _dev_check(dY, dA)
    M, N = dY.shape
    K = wq.K
    if wq.N != N:
        raise ValueError("dY [M,N] and the weight cache must agree in N")
    if dA is None:
        dA = torch.empty((M, K), dtype=dY.dtype, device=dY.device)
    w = _ws(workspace_bytes(FP4_OP_DGRAD, M, K, N, _dt(dY)), ws)
    _check(lib().fp4_linear_bwd_dgrad_cached(_ptr(dY), C.byref(wq.c), _dt(dY), M, K, N, _ptr(dA), _ptr(w),
                                             w.numel(), _stream()), "fp4_linear_bwd_dgrad_cached")
    return dA


def fp4_linear_bwd_dgrad(dY: torch.Tensor, W: torch.Tensor, dA: Optional[torch.Tensor] = None,
                         ws: Optional[Workspace] = None) -> torch.Tensor:
    _dev_check(dY, W, dA)
    M, N = dY.shape
    K, N2 = W.shape
    if N2 != N or dY.dtype != W.dtype:
        raise ValueError("dY [M,N] and W [K,N] must agree in N and dtype")
    if dA is None:
        dA = torch.empty((M, K), dtype=dY.dtype, device=dY.device)
    nb = workspace_bytes(FP4_OP_DGRAD, M, K, N, _dt(dY))
    w = _ws(nb, ws)
    _check(lib().fp4_linear_bwd_dgrad(_ptr(dY), _ptr(W), _dt(dY), M, K, N, _ptr(dA), _ptr(w), w.numel(),
                                      _stream()), "fp4_linear_bwd_dgrad")
    return dA


def fp4_linear_bwd_wgrad(A: torch.Tensor, dY: torch.Tensor, W: torch.Tensor, ctx: FwdCtx, dge_k: float = 5.0,
                         dge_cap: float = 3.0, dW: Optional[torch.Tensor] = None,
                         ws: Optional[Workspace] = None) -> torch.Tensor:
    _dev_check(A, dY, W, dW)
    M, K = A.shape
    _, N = W.shape
    if dY.shape != (M, N) or W.shape != (K, N) or not (A.dtype == dY.dtype == W.dtype):
        raise ValueError("shape / dtype mismatch")
    if dW is None:
        dW = torch.empty((K, N), dtype=torch.float32, device=A.device)
    nb = workspace_bytes(FP4_OP_WGRAD, M, K, N, _dt(A))
    w = _ws(nb, ws)
    _check(lib().fp4_linear_bwd_wgrad(_ptr(A), _ptr(dY), _ptr(W), _dt(A), M, K, N, C.byref(ctx.c),
                                      float(dge_k), float(dge_cap), _ptr(dW), _ptr(w), w.numel(), _stream()),
           "fp4_linear_bwd_wgrad")
    return dW


def fp4_linear_bwd(dY: torch.Tensor, A: torch.Tensor, W: torch.Tensor, ctx: FwdCtx, dge_k: float = 5.0, dge_cap: float = 3.0,
                   wq: Optional["WeightCache"] = None, dA: Optional[torch.Tensor] = None, dW: Optional[torch.Tensor] = None,
                   ws: Optional[Workspace] = None):
    """Both gradients in one call (dY read once for both of its quantizations).  Returns (dA, dW)."""
    _dev_check(dY, A, W, dA, dW)
    M, K = A.shape
    _, N = W.shape
    if dY.shape != (M, N) or W.shape != (K, N) or not (A.dtype == dY.dtype == W.dtype):
        raise ValueError("shape / dtype mismatch")
    if dA is None:
        dA = torch.empty((M, K), dtype=dY.dtype, device=dY.device)
    if dW is None:
        dW = torch.empty((K, N), dtype=torch.float32, device=dY.device)
    w = _ws(workspace_bytes(FP4_OP_BWD, M, K, N, _dt(A)), ws)
    _check(lib().fp4_linear_bwd(_ptr(dY), _ptr(A), _ptr(W), C.byref(wq.c) if wq is not None else None, _dt(A), M, K, N,
                                C.byref(ctx.c), float(dge_k), float(dge_cap), _ptr(dA), _ptr(dW), _ptr(w), w.numel(),
                                _stream()), "fp4_linear_bwd")
    return dA, dW


def fp4_gemm(codes_l: torch.Tensor, gamma_l: Optional[torch.Tensor], codes_rt: torch.Tensor,
             gamma_r: Optional[torch.Tensor], out_dtype=torch.float32, addend: Optional[torch.Tensor] = None,
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev_check(codes_l, gamma_l, codes_rt, gamma_r, addend)
    P, kb = codes_l.shape
    Q, kb2 = codes_rt.shape
    if kb != kb2:
        raise ValueError("operands disagree in K")
    ldo = Q
    if out is None:
        ldo = (Q + 7) // 8 * 8          # the ABI wants a leading dimension that is a multiple of 8
        full = torch.empty((P, ldo), dtype=out_dtype, device=codes_l.device)
        out = full[:, :Q]
        if addend is not None and ldo != Q:
            pad = torch.zeros((P, ldo), dtype=torch.float32, device=codes_l.device)
            pad[:, :Q] = addend
            addend = pad
    _check(lib().fp4_gemm(_ptr(codes_l), _ptr(gamma_l), _ptr(codes_rt), _ptr(gamma_r), P, Q, 2 * kb,
                          _ptr(addend), _ptr(out), _dt(out), ldo, _stream()), "fp4_gemm")
    return out


def fp8_quantize(x: torch.Tensor, axis: int, ws: Optional[Workspace] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """E4M3 codes (one per byte; COL: transposed) and scales gamma = 448 / absmax."""
    _dev_check(x)
    rows, cols = x.shape
    shape, n = ((rows, cols), rows) if axis == FP4_AXIS_ROW else ((cols, rows), cols)
    codes = torch.empty(shape, dtype=torch.uint8, device=x.device)
    gamma = torch.empty(n, dtype=torch.float32, device=x.device)
    w = _ws(workspace_bytes(FP4_OP_QUANTIZE, rows, cols, 0, _dt(x)), ws)
    _check(lib().fp8_quantize(_ptr(x), _dt(x), rows, cols, cols, axis, _ptr(codes), _ptr(gamma), _ptr(w), w.numel(),
                              _stream()), "fp8_quantize")
    return codes, gamma


def fp4_gemm_mixed(codes_l: torch.Tensor, fmt_l: int, gamma_l: Optional[torch.Tensor], codes_rt: torch.Tensor, fmt_r: int,
                   gamma_r: Optional[torch.Tensor], out_dtype=torch.float32, addend: Optional[torch.Tensor] = None):
    _dev_check(codes_l, gamma_l, codes_rt, gamma_r, addend)
    P, Q = codes_l.shape[0], codes_rt.shape[0]
    Kc = codes_l.shape[1] * (1 if fmt_l == FP4_FMT_E4M3 else 2)
    if Kc != codes_rt.shape[1] * (1 if fmt_r == FP4_FMT_E4M3 else 2):
        raise ValueError("operands disagree in K")
    if Q % 8:
        raise ValueError("Q must be a multiple of 8 here")
    out = torch.empty((P, Q), dtype=out_dtype, device=codes_l.device)
    _check(lib().fp4_gemm_mixed(_ptr(codes_l), fmt_l, _ptr(gamma_l), _ptr(codes_rt), fmt_r, _ptr(gamma_r), P, Q, Kc,
                                _ptr(addend), _ptr(out), _dt(out), Q, _stream()), "fp4_gemm_mixed")
    return out


def fp4_linear_fwd_mixed(A: torch.Tensor, W: torch.Tensor, act_fmt: int, wgt_fmt: int, alpha: float = 1.0,
                         ctx: Optional[FwdCtx] = None, Y: Optional[torch.Tensor] = None, ws: Optional[Workspace] = None):
    _dev_check(A, W, Y)
    M, K = A.shape
    K2, N = W.shape
    if K2 != K or A.dtype != W.dtype:
        raise ValueError("A [M,K] and W [K,N] must agree in K and dtype")
    if ctx is None:
        ctx = FwdCtx(M, K, N, alpha, A.device)
    if Y is None:
        Y = torch.empty((M, N), dtype=A.dtype, device=A.device)
    w = _ws(workspace_bytes(FP4_OP_FWD_MIXED, M, K, N, _dt(A)), ws)
    _check(lib().fp4_linear_fwd_mixed(_ptr(A), _ptr(W), _dt(A), M, K, N, act_fmt, wgt_fmt, float(alpha), _ptr(Y),
                                      C.byref(ctx.c), _ptr(w), w.numel(), _stream()), "fp4_linear_fwd_mixed")
    return Y, ctx


def fp4_linear_fwd_granularity(A: torch.Tensor, W: torch.Tensor, act_tensorwise: bool, wgt_tensorwise: bool,
                               alpha: float = 1.0, ctx: Optional[FwdCtx] = None, Y: Optional[torch.Tensor] = None,
                               ws: Optional[Workspace] = None):
    """Forward pass with tensor-wise scaling of the activations and / or the weights."""
    _dev_check(A, W, Y)
    M, K = A.shape
    K2, N = W.shape
    if K2 != K or A.dtype != W.dtype:
        raise ValueError("A [M,K] and W [K,N] must agree in K and dtype")
    if ctx is None:
        ctx = FwdCtx(M, K, N, alpha, A.device)
    if Y is None:
        Y = torch.empty((M, N), dtype=A.dtype, device=A.device)
    w = _ws(workspace_bytes(FP4_OP_FWD, M, K, N, _dt(A)), ws)
    _check(lib().fp4_linear_fwd_granularity(_ptr(A), _ptr(W), _dt(A), M, K, N, int(bool(act_tensorwise)),
                                            int(bool(wgt_tensorwise)), float(alpha), _ptr(Y), C.byref(ctx.c), _ptr(w),
                                            w.numel(), _stream()), "fp4_linear_fwd_granularity")
    return Y, ctx


def fp8_host_round_codes(x_host):
    """numpy fp32 array (host) -> uint8 E4M3 codes, through the library's own rounding routine."""
    import numpy as np
    x = np.ascontiguousarray(x_host, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    _check(lib().fp8_host_round_codes(x.ctypes.data_as(C.c_void_p), x.size, out.ctypes.data_as(C.c_void_p)),
           "fp8_host_round_codes")
    return out


def fp4_unpack(codes: torch.Tensor) -> torch.Tensor:
    _dev_check(codes)
    rows, half = codes.shape
    out = torch.empty((rows, 2 * half), dtype=torch.uint8, device=codes.device)
    _check(lib().fp4_unpack(_ptr(codes), rows, 2 * half, _ptr(out), _stream()), "fp4_unpack")
    return out


def fp4_dge_apply(G: torch.Tensor, W: torch.Tensor, gamma_W: torch.Tensor, dge_k: float = 5.0,
                  dge_cap: float = 3.0, dW: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev_check(G, W, gamma_W, dW)
    K, N = W.shape
    if dW is None:
        dW = torch.empty_like(G)
    _check(lib().fp4_dge_apply(_ptr(G), _ptr(W), _dt(W), _ptr(gamma_W), K, N, float(dge_k), float(dge_cap),
                               _ptr(dW), _stream()), "fp4_dge_apply")
    return dW


def fp4_residual_spmm(row_ptr: torch.Tensor, col_idx: torch.Tensor, val: torch.Tensor, Q: int,
                      D: torch.Tensor, R: Optional[torch.Tensor] = None, ws: Optional[Workspace] = None) -> torch.Tensor:
    _dev_check(row_ptr, col_idx, val, D, R)
    P = row_ptr.numel() - 1
    N = D.shape[1]
    if R is None:
        R = torch.empty((P, N), dtype=torch.float32, device=D.device)
    w = _ws(workspace_bytes(FP4_OP_SPMM, P, Q, N, _dt(D)), ws)
    _check(lib().fp4_residual_spmm(_ptr(row_ptr), _ptr(col_idx), _ptr(val), P, Q, _ptr(D), _dt(D), N,
                                   _ptr(R), _ptr(w), w.numel(), _stream()), "fp4_residual_spmm")
    return R


def fp4_host_round_codes(x_host):
    """numpy fp32 array (host) -> uint8 codes, through the library's own rounding routine."""
    import numpy as np
    x = np.ascontiguousarray(x_host, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    _check(lib().fp4_host_round_codes(x.ctypes.data_as(C.c_void_p), x.size, out.ctypes.data_as(C.c_void_p)),
           "fp4_host_round_codes")
    return out


def fp4_device_round_codes(x):
    """fp32 CUDA tensor (numel a multiple of 8) -> uint8 codes, through the quantization kernels' packing routine."""
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    out = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    _check(lib().fp4_device_round_codes(x.data_ptr(), x.numel(), out.data_ptr(), _stream()), "fp4_device_round_codes")
    return out


def fp4_device_round_sweep(device="cuda:0") -> int:
    """Number of fp32 bit patterns (times eight word positions) where the device's packing routine and its
    comparison-chain routine disagree; 0 is the only acceptable result."""
    import torch
    cnt = torch.zeros(1, dtype=torch.int64, device=device)
    _check(lib().fp4_device_round_sweep(cnt.data_ptr(), _stream()), "fp4_device_round_sweep")
    return int(cnt.item())


FP4_TRACE_GEMM, FP4_TRACE_SPMM = 0, 1


def fp4_trace_begin(max_launches: int) -> None:
    _check(lib().fp4_trace_begin(int(max_launches)), "fp4_trace_begin")


def fp4_trace_end(max_launches: int):
    """[(kind, ms)] of the GEMM / tiled sparse-product launches recorded since fp4_trace_begin, in order."""
    buf = (C.c_float * max_launches)()
    kinds = (C.c_int * max_launches)()
    n = lib().fp4_trace_end(C.cast(buf, C.c_void_p), C.cast(kinds, C.c_void_p), max_launches)
    if n < 0:
        raise Fp4Error(n, "fp4_trace_end")
    return [(int(kinds[i]), float(buf[i])) for i in range(min(n, max_launches))]


def fp4_probe_mfma(operand_bytes: torch.Tensor, workgroups: int, iters: int, sink: torch.Tensor) -> None:
    _dev_check(operand_bytes, sink)
    _check(lib().fp4_probe_mfma(_ptr(operand_bytes), operand_bytes.numel() * operand_bytes.element_size(),
                                int(workgroups), int(iters), _ptr(sink), _stream()), "fp4_probe_mfma")


def fp4_probe_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    _dev_check(src, dst)
    _check(lib().fp4_probe_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream()),
           "fp4_probe_copy")
