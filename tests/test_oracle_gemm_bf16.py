"""Pins for the oracle's BF16 contraction (the baseline GEMM the FP8 path is compared with; CPU only)."""
import numpy as np
import torch

import oracle
from paper_2512_15306_amd import synth


def _bits(t):
    return synth.bf16_bits(t)


def test_integer_operands_against_brute_force():
    rng = np.random.default_rng(3)
    R, C, T = 7, 5, 33
    a = rng.integers(-9, 10, (R, T))
    b = rng.integers(-9, 10, (C, T))
    want = np.zeros((R, C), np.int64)
    mag = np.zeros((R, C), np.int64)
    for r in range(R):
        for c in range(C):
            for t in range(T):
                want[r, c] += a[r, t] * b[c, t]
                mag[r, c] += abs(a[r, t] * b[c, t])
    y, S = oracle.gemm_bf16_tn(_bits(torch.from_numpy(a).to(torch.bfloat16)), _bits(torch.from_numpy(b).to(torch.bfloat16)))
    assert np.array_equal(y, want.astype(np.float64)) and np.array_equal(S, mag.astype(np.float64))
    # operand order: the transposed product is the transposed result, and a different matrix otherwise
    yt, _ = oracle.gemm_bf16_tn(_bits(torch.from_numpy(b).to(torch.bfloat16)), _bits(torch.from_numpy(a).to(torch.bfloat16)))
    assert np.array_equal(yt, want.T.astype(np.float64))


def test_against_library_matmul_and_sampling():
    g = torch.Generator().manual_seed(5)
    A = (torch.randn(23, 70, generator=g)).to(torch.bfloat16)
    B = (torch.randn(31, 70, generator=g) * 0.02).to(torch.bfloat16)
    y, S = oracle.gemm_bf16_tn(_bits(A), _bits(B))
    np.testing.assert_allclose(y, (A.double() @ B.double().T).numpy(), rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(S, (A.double().abs() @ B.double().abs().T).numpy(), rtol=1e-12)
    rr, cc = np.array([0, 22, 5, 5]), np.array([30, 0, 7, 8])
    ys, Ss = oracle.gemm_bf16_tn_sampled(_bits(A), _bits(B), rr, cc)
    assert np.array_equal(ys, y[rr, cc]) and np.array_equal(Ss, S[rr, cc])
