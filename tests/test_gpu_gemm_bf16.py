"""GPU parity: the BF16 baseline GEMM against the oracle (binary64 sum of exact products)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import llmq, synth
from gpu_common import DEV, bf16_to_f64

pytestmark = pytest.mark.gpu

# tuned tiles (several tile shapes, odd number of K steps, multiple rounds) and generic shapes
SHAPES = [(256, 256, 128), (512, 768, 320), (384, 640, 192), (128, 128, 64), (768, 512, 1024), (100, 72, 40), (33, 17, 5), (1, 1, 1),
          (256, 256, 100)]


def _rand(shape, seed, std=1.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * std).to(torch.bfloat16)


def _check(c, y, S, T, what, prev=None):
    got = bf16_to_f64(c)
    want = y if prev is None else y + prev
    # binary32 accumulation in any order over T products, then one rounding to BF16 (two with accumulate)
    bound = np.abs(want) * 2.0 ** -8 * (1 if prev is None else 2) + T * 2.0 ** -24 * S + 1e-30
    bad = np.argwhere(np.abs(got - want) > bound)
    assert bad.size == 0, "%s: %d out of tolerance, first %s got %r want %r" % (what, len(bad), bad[0], got[tuple(bad[0])], want[tuple(bad[0])])
    assert np.isfinite(got).all() and (S > 0).any()


@pytest.mark.parametrize("shape", SHAPES)
def test_bf16_gemm_against_oracle(shape):
    R, C, T = shape
    print("bf16 gemm R=%d C=%d T=%d" % shape, flush=True)
    A, B = _rand((R, T), 100 + R + T), _rand((C, T), 200 + C + T, 0.05)
    y, S = oracle.gemm_bf16_tn(synth.bf16_bits(A), synth.bf16_bits(B))
    c = torch.full((R, C), -7.0, dtype=torch.bfloat16, device=DEV)
    llmq.llmq_bf16_gemm_tn(A.to(DEV), B.to(DEV), c)
    _check(c, y, S, T, "plain")
    prev = _rand((R, C), 300 + R, 0.5).to(DEV)
    c2 = prev.clone()
    llmq.llmq_bf16_gemm_tn(A.to(DEV), B.to(DEV), c2, accumulate=True)
    _check(c2, y, S, T, "accumulate", prev=bf16_to_f64(prev))
    c3 = torch.empty_like(c)
    llmq.llmq_bf16_gemm_tn(A.to(DEV), B.to(DEV), c3)
    assert torch.equal(c3, c)


def test_integer_operands_are_exact():
    g = torch.Generator(device="cpu").manual_seed(11)
    A = torch.randint(-4, 5, (256, 192), generator=g).to(torch.bfloat16)
    B = torch.randint(-4, 5, (384, 192), generator=g).to(torch.bfloat16)
    c = torch.empty((256, 384), dtype=torch.bfloat16, device=DEV)
    llmq.llmq_bf16_gemm_tn(A.to(DEV), B.to(DEV), c)
    y, _ = oracle.gemm_bf16_tn(synth.bf16_bits(A), synth.bf16_bits(B))
    want = torch.from_numpy(y).to(torch.bfloat16)        # sums up to 3072: rounding to BF16 is part of the contract
    assert torch.equal(c.cpu(), want)


@pytest.mark.parametrize("tile", ["4x4", "4x3", "3x3", "2x2", "4x2", "3x2"])
def test_every_tile_shape(tile, monkeypatch):
    monkeypatch.setenv("LLMQ_GEMM_TILE", tile)
    R, C, T = 768, 768, 448
    A, B = _rand((R, T), 7), _rand((C, T), 8, 0.05)
    y, S = oracle.gemm_bf16_tn(synth.bf16_bits(A), synth.bf16_bits(B))
    c = torch.empty((R, C), dtype=torch.bfloat16, device=DEV)
    llmq.llmq_bf16_gemm_tn(A.to(DEV), B.to(DEV), c)
    _check(c, y, S, T, tile)


def test_config_linear_at_full_size_sampled():
    """Forward GEMM of config 3's attention-out linear (8192 x 3584 x 3584) in BF16: 4096 sampled outputs
    plus a full tile-boundary row and column."""
    cfg = synth.CONFIGS[3]
    X, W = synth.make_x(cfg, 1, device=DEV), synth.make_w(cfg, 1, device=DEV)
    M, K = X.shape
    N = W.shape[0]
    c = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    llmq.llmq_bf16_gemm_tn(X, W, c)
    rng = np.random.default_rng(17)
    rr = np.concatenate([rng.integers(0, M, 4096), np.full(N, 255), np.arange(M)])
    cc = np.concatenate([rng.integers(0, N, 4096), np.arange(N), np.full(M, 256)])
    y, S = oracle.gemm_bf16_tn_sampled(synth.bf16_bits(X), synth.bf16_bits(W), rr, cc)
    got = bf16_to_f64(c)[rr, cc]
    assert (np.abs(got - y) <= np.abs(y) * 2.0 ** -8 + K * 2.0 ** -24 * S).all()
