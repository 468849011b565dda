"""Shared plumbing of the GPU parity tests: run the library through its binding, run the oracle on the
same bytes, compare.  No arithmetic of the method lives here."""
import numpy as np
import torch

import oracle
from paper_2512_15306_amd import llmq, synth

DEV = "cuda:0"
FMAX = {0: 448.0, 1: 57344.0}
GEMM_TOL = 2.0 ** -7          # |y_gpu - y_oracle| <= GEMM_TOL * sum_t |a_t b_t| / (sA sB), per element


def f32_bits(t: torch.Tensor) -> int:
    return int(t.detach().cpu().view(torch.int32).item()) & 0xFFFFFFFF


def np_f32_bits(v) -> int:
    return int(np.float32(v).view(np.uint32))


def gpu_amax(x: torch.Tensor, fmt: int, want_scale=True):
    a = torch.full((1,), -1.0, device=x.device, dtype=torch.float32)
    s = torch.full((1,), -1.0, device=x.device, dtype=torch.float32) if want_scale else None
    ws = torch.full((llmq.llmq_amax_workspace_bytes(),), 0xFF, device=x.device, dtype=torch.uint8)   # garbage on entry
    llmq.llmq_amax(x, fmt, a, s, ws)
    return a, s


def gpu_quantize(x: torch.Tensor, d_scale: torch.Tensor, fmt: int, transpose=True):
    rows, cols = x.shape
    q = torch.full((rows, cols), 0xAA, device=x.device, dtype=torch.uint8)
    qt = torch.full((cols, rows), 0xAA, device=x.device, dtype=torch.uint8) if transpose else None
    llmq.llmq_quantize_fp8(x, d_scale, fmt, q, qt)
    return q, qt


def oracle_quantized(x: torch.Tensor, fmt: int):
    """(amax, scale, q, qt) of a BF16 tensor by the oracle."""
    xb = synth.bf16_bits(x)
    a = oracle.amax_bf16(xb)
    s = oracle.scale(a, fmt)
    q, qt = oracle.quantize(xb.reshape(x.shape), s, fmt)
    return a, s, q, qt


def bf16_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def assert_gemm_close(c_gpu: torch.Tensor, y: np.ndarray, S: np.ndarray, what=""):
    got = bf16_to_f64(c_gpu)
    err = np.abs(got - y)
    bound = GEMM_TOL * S
    bad = np.argwhere(err > bound)
    assert bad.size == 0, "%s: %d elements out of tolerance, first %s got %r want %r bound %r" % (
        what, len(bad), bad[0], got[tuple(bad[0])], y[tuple(bad[0])], bound[tuple(bad[0])])
    # the comparison must not be vacuous
    assert np.isfinite(got).all() and (S > 0).any()
