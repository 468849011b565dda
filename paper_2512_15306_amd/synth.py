"""Seeded synthetic inputs with the shapes and value distributions of the benchmark configs.

This module holds no arithmetic of the method (no absmax, scaling, FP8 casting or
GEMM): it only draws random BF16 tensors.  Both the GPU tests/benchmark and the
CPU oracle tests take their inputs from here, so that the two sides see the same
bytes.

The paper measures on its own training runs; these tensors stand in for the
activations, weights and output gradients of the linear layers of Qwen-2.5-style
transformer blocks (the 7B shapes reproduce the paper's count of FP8 operations
per token, Section 4 "Impact of FP8").
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import torch

BASE_SEED = 20251215


@dataclass(frozen=True)
class Linear:
    name: str
    K: int   # input features (contraction length of the forward GEMM)
    N: int   # output features


@dataclass(frozen=True)
class Config:
    index: int
    name: str
    M: int                       # tokens
    linears: Tuple[Linear, ...]
    x_dist: str                  # "normal" or "student_t3"
    x_outlier_frac: float        # fraction of K-channels multiplied by x_outlier_gain
    x_outlier_gain: float
    w_std: float
    dy_std: float


CONFIGS: Dict[int, Config] = {
    1: Config(1, "single-linear", 256, (Linear("linear", 512, 1024),),
              "normal", 0.0, 1.0, 0.02, 1e-3),
    2: Config(2, "3B-class block", 4096,
              (Linear("qkv", 3072, 5120), Linear("o", 3072, 3072),
               Linear("gate_up", 3072, 16384), Linear("down", 8192, 3072)),
              "normal", 0.0, 1.0, 0.02, 1e-4),
    3: Config(3, "7B-class block", 8192,
              (Linear("qkv", 3584, 4608), Linear("o", 3584, 3584),
               Linear("gate_up", 3584, 37888), Linear("down", 18944, 3584)),
              "normal", 0.005, 50.0, 0.02, 1e-4),
    4: Config(4, "14B-class block", 8192,
              (Linear("qkv", 5120, 7168), Linear("o", 5120, 5120),
               Linear("gate_up", 5120, 27648), Linear("down", 13824, 5120)),
              "normal", 0.005, 50.0, 0.02, 1e-4),
    5: Config(5, "32B-class block", 16384,
              (Linear("qkv", 5120, 7168), Linear("o", 5120, 5120),
               Linear("gate_up", 5120, 55296), Linear("down", 27648, 5120)),
              "student_t3", 0.01, 100.0, 0.02, 1e-5),
}


def tensor_seed(config: int, linear: int, which: int) -> int:
    """which: 0 = X, 1 = W, 2 = dY, 3 = outlier-channel permutation, 4 = GU (SwiGLU input), 5 = dh,
    6 = branch output added to the residual stream, 7 = RMSNorm weight."""
    return BASE_SEED + 1000 * config + 10 * linear + which


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _randn(shape, device, seed: int) -> torch.Tensor:
    return torch.randn(shape, generator=_gen(device, seed), device=device, dtype=torch.float32)


def make_x(cfg: Config, li: int, device="cpu", M: Optional[int] = None) -> torch.Tensor:
    """Activations X[M, K] in BF16."""
    lin = cfg.linears[li]
    M = cfg.M if M is None else M
    g = _gen(device, tensor_seed(cfg.index, li, 0))
    x = torch.randn((M, lin.K), generator=g, device=device, dtype=torch.float32)
    if cfg.x_dist == "student_t3":
        chi2 = torch.zeros_like(x)
        for _ in range(3):
            chi2 += torch.randn((M, lin.K), generator=g, device=device, dtype=torch.float32) ** 2
        x = x / torch.sqrt(chi2 / 3.0)
        del chi2
    elif cfg.x_dist != "normal":
        raise ValueError(cfg.x_dist)
    n_out = int(round(cfg.x_outlier_frac * lin.K))
    if n_out > 0:
        gp = _gen("cpu", tensor_seed(cfg.index, li, 3))
        cols = torch.randperm(lin.K, generator=gp)[:n_out].to(device)
        x[:, cols] *= cfg.x_outlier_gain
    return x.to(torch.bfloat16)


def make_w(cfg: Config, li: int, device="cpu") -> torch.Tensor:
    """Weights W[N, K] in BF16 (PyTorch's [out, in] layout)."""
    lin = cfg.linears[li]
    w = _randn((lin.N, lin.K), device, tensor_seed(cfg.index, li, 1)) * cfg.w_std
    return w.to(torch.bfloat16)


def make_dy(cfg: Config, li: int, device="cpu", M: Optional[int] = None) -> torch.Tensor:
    """Output gradients dY[M, N] in BF16."""
    lin = cfg.linears[li]
    M = cfg.M if M is None else M
    dy = _randn((M, lin.N), device, tensor_seed(cfg.index, li, 2)) * cfg.dy_std
    return dy.to(torch.bfloat16)


def swiglu_dims(cfg: Config) -> Tuple[int, int]:
    """(M, I) of the block's SwiGLU: I is the width of the down projection's input."""
    gate_up = next(l for l in cfg.linears if l.name == "gate_up")
    return cfg.M, gate_up.N // 2


def make_gu(cfg: Config, device="cpu", M: Optional[int] = None) -> torch.Tensor:
    """Output GU[M, 2I] of the gate+up projection in BF16: N(0, std) with the standard deviation a
    product of unit-variance activations with the config's weights has, std = w_std * sqrt(K)."""
    li = next(i for i, l in enumerate(cfg.linears) if l.name == "gate_up")
    lin = cfg.linears[li]
    M = cfg.M if M is None else M
    gu = _randn((M, lin.N), device, tensor_seed(cfg.index, li, 4)) * (cfg.w_std * lin.K ** 0.5)
    return gu.to(torch.bfloat16)


def make_dh(cfg: Config, device="cpu", M: Optional[int] = None) -> torch.Tensor:
    """Gradient dh[M, I] arriving at the SwiGLU output in BF16 (N(0, dy_std))."""
    li = next(i for i, l in enumerate(cfg.linears) if l.name == "gate_up")
    M = cfg.M if M is None else M
    dh = _randn((M, cfg.linears[li].N // 2), device, tensor_seed(cfg.index, li, 5)) * cfg.dy_std
    return dh.to(torch.bfloat16)


def make_norm_inputs(cfg: Config, device="cpu", M: Optional[int] = None):
    """(res, x, w) of the RMSNorm in front of the block's first linear: the residual stream res[M, C]
    with the config's activation distribution (outlier channels included), the branch output x[M, C]
    added to it (N(0, 0.5)) and the norm's weight w[C] (1 + N(0, 0.1)); C is the hidden size."""
    M = cfg.M if M is None else M
    C = cfg.linears[0].K
    res = make_x(cfg, 0, device=device, M=M)
    x = (_randn((M, C), device, tensor_seed(cfg.index, 0, 6)) * 0.5).to(torch.bfloat16)
    w = (1.0 + _randn((C,), device, tensor_seed(cfg.index, 0, 7)) * 0.1).to(torch.bfloat16)
    return res, x, w


def linear_flops(cfg: Config) -> int:
    """Forward + dgrad + wgrad: three GEMMs of 2*M*K*N each, summed over the block's linears."""
    return sum(6 * cfg.M * l.K * l.N for l in cfg.linears)


def quantize_elements(cfg: Config) -> int:
    """Elements of X, W and dY over all linears (each is absmax-ed and quantized once)."""
    return sum(cfg.M * l.K + l.N * l.K + cfg.M * l.N for l in cfg.linears)


def bf16_bits(t: torch.Tensor):
    """BF16 tensor -> numpy uint16 bit patterns on the host (for the oracle)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view("uint16")


def small_cases() -> List[Tuple[int, int, int]]:
    """(M, K, N) shapes the oracle finishes in seconds; they span several tiles and ragged tails."""
    return [(256, 512, 1024), (384, 640, 896), (272, 400, 528), (100, 72, 136), (33, 17, 5),
            (1, 1, 1), (16, 128, 16), (512, 256, 256)]
