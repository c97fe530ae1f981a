"""Seeded synthetic inputs for the FP4 linear layer (shared by tests, bench and smoke).

This module only draws random tensors with the shapes and value structure of the
paper's workloads (Sec. 4.1: LLaMA-2 linear layers; App. D: weights roughly normal
with a small range, activations with outliers concentrated in a few channels or
heavy-tailed).  It holds none of the method's arithmetic: no quantization, no
clamping, no scaling by method-defined factors.  Both the CPU oracle's callers and
the GPU path's callers take their inputs from here so they see the same numbers.

All tensors are generated on the CPU in fp32 from a torch.Generator seeded with
    20250117 + 1000 * config + tensor_id      (A=0, W=1, dY=2, outlier channels=3)
and, for "bf16 master" configs, rounded to bf16 (round-to-nearest-even) and widened
back to fp32, so the fp32 array and the bf16 tensor hold identical values.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Tuple

import torch

BASE_SEED = 20250117
TID_A, TID_W, TID_DY, TID_PERM = 0, 1, 2, 3


@dataclasses.dataclass(frozen=True)
class LayerShape:
    name: str
    M: int  # tokens
    K: int  # input channels  c_i
    N: int  # output channels c_o


@dataclasses.dataclass(frozen=True)
class Config:
    idx: int
    name: str
    dtype: str          # "f32" | "bf16"
    layers: Tuple[LayerShape, ...]
    act: str            # "gauss_outlier" | "student_t3"
    outlier_frac: float
    outlier_scale: float
    alpha: float
    dge_k: float = 5.0
    dge_cap: float = 3.0


def _layers(M, spec):
    return tuple(LayerShape(n, M, k, o) for (n, k, o) in spec)


CONFIGS: Dict[str, Config] = {
    # single fp32 layer; the case the oracle finishes in seconds
    "c1": Config(1, "single-layer-fp32", "f32", _layers(256, [("lin", 512, 512)]),
                 "gauss_outlier", 0.005, 20.0, 0.99),
    "c2": Config(2, "llama2-1.3b-block", "bf16",
                 _layers(8192, [("qkv", 2048, 6144), ("o", 2048, 2048), ("gate", 2048, 5504),
                                ("up", 2048, 5504), ("down", 5504, 2048)]),
                 "gauss_outlier", 0.001, 50.0, 0.99),
    "c3": Config(3, "llama2-7b-block", "bf16",
                 _layers(16384, [("qkv", 4096, 12288), ("o", 4096, 4096), ("gate_up", 4096, 11008),
                                 ("down", 11008, 4096)]),
                 "gauss_outlier", 0.001, 50.0, 0.99),
    "c4": Config(4, "llama2-13b-block-student-t", "bf16",
                 _layers(16384, [("qkv", 5120, 15360), ("ffn", 5120, 13824), ("down", 13824, 5120)]),
                 "student_t3", 0.0, 1.0, 0.99),
    "c5": Config(5, "llama2-7b-layer-step", "bf16",
                 _layers(16384, [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096),
                                 ("o", 4096, 4096), ("gate", 4096, 11008), ("up", 4096, 11008),
                                 ("down", 11008, 4096)]),
                 "gauss_outlier", 0.001, 50.0, 0.99),
}


def _gen(config_idx: int, tensor_id: int, salt: int = 0) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(BASE_SEED + 1000 * config_idx + tensor_id + 100 * salt)
    return g


def _finish(x: torch.Tensor, dtype: str) -> torch.Tensor:
    """Round to the master dtype and return fp32 holding exactly those values."""
    if dtype == "bf16":
        return x.to(torch.bfloat16).to(torch.float32)
    return x.to(torch.float32)


def outlier_channels(config_idx: int, K: int, frac: float, salt: int = 0) -> torch.Tensor:
    n_out = max(1, int(round(frac * K)))
    perm = torch.randperm(K, generator=_gen(config_idx, TID_PERM, salt))
    return perm[:n_out].sort().values


def make_activation(cfg: Config, M: int, K: int, salt: int = 0) -> torch.Tensor:
    g = _gen(cfg.idx, TID_A, salt)
    if cfg.act == "gauss_outlier":
        x = torch.randn(M, K, generator=g, dtype=torch.float32)
        ch = outlier_channels(cfg.idx, K, cfg.outlier_frac, salt)
        x[:, ch] *= cfg.outlier_scale
    elif cfg.act == "student_t3":
        z = torch.randn(M, K, generator=g, dtype=torch.float32)
        chi = torch.zeros(M, K, dtype=torch.float32)
        for _ in range(3):
            chi += torch.randn(M, K, generator=g, dtype=torch.float32) ** 2
        x = z / torch.sqrt(chi / 3.0)
    else:
        raise ValueError(cfg.act)
    return _finish(x, cfg.dtype)


def make_weight(cfg: Config, K: int, N: int, salt: int = 0) -> torch.Tensor:
    w = torch.randn(K, N, generator=_gen(cfg.idx, TID_W, salt), dtype=torch.float32) * 0.02
    return _finish(w, cfg.dtype)


def make_grad_out(cfg: Config, M: int, N: int, salt: int = 0) -> torch.Tensor:
    d = torch.randn(M, N, generator=_gen(cfg.idx, TID_DY, salt), dtype=torch.float32) * 1e-2
    return _finish(d, cfg.dtype)


def make_layer(cfg: Config, layer: LayerShape, salt: int = 0, M: int | None = None):
    """(A[M,K], W[K,N], dY[M,N]) as fp32 CPU tensors holding master-dtype values."""
    M = layer.M if M is None else M
    return (make_activation(cfg, M, layer.K, salt), make_weight(cfg, layer.K, layer.N, salt),
            make_grad_out(cfg, M, layer.N, salt))


def small_case(M: int, K: int, N: int, dtype: str = "f32", seed: int = 0, act: str = "gauss_outlier",
               outlier_frac: float = 0.01, outlier_scale: float = 20.0):
    """Free-shape case for parity tests (ragged tiles, tiny sizes)."""
    cfg = Config(900 + seed, "small", dtype, (LayerShape("lin", M, K, N),), act, outlier_frac,
                 outlier_scale, 0.99)
    return make_layer(cfg, cfg.layers[0])


def gemm_flops(layers: List[LayerShape]) -> float:
    return float(sum(2.0 * l.M * l.K * l.N for l in layers))
