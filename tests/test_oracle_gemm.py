"""Pins for the oracle's contraction (forward / dgrad / wgrad all reduce to it), CPU only.

Section 3 ("Overview"): the transformer-block matmuls run in FP8 and return BF16; FP8 GEMM is
TN-only, so both operands are stored with the contraction index contiguous.  Checks: exact
integer matmul by brute force on lossless inputs, the library matmul on decoded values, the
adjoint identity linking the three GEMMs, and consistency of the sampled variant.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import synth


def _int_tensor(rng, shape, top=7):
    """Small integers, mostly in {-2..2}, with one +-top entry that fixes the absmax."""
    v = rng.integers(-2, 3, size=shape).astype(np.float32)
    i = tuple(rng.integers(0, s) for s in shape)
    v[i] = top * (1 if rng.random() < 0.5 else -1)
    return v


def _q(vals, fmt):
    x = torch.from_numpy(vals).to(torch.bfloat16)
    xb = synth.bf16_bits(x)
    s = oracle.scale(oracle.amax_bf16(xb), fmt)
    q, qt = oracle.quantize(xb, s, fmt)
    return q, qt, s


@pytest.mark.parametrize("M,K,N", [(5, 7, 3), (4, 32, 6), (9, 16, 11), (1, 1, 1)])
def test_three_gemms_equal_integer_matmul_by_brute_force(M, K, N):
    rng = np.random.default_rng(100 + M + K + N)
    X = _int_tensor(rng, (M, K))
    W = _int_tensor(rng, (N, K))
    dY = _int_tensor(rng, (M, N))
    Xq, Xqt, sx = _q(X, oracle.E4M3)
    Wq, Wqt, sw = _q(W, oracle.E4M3)
    dYq, dYqt, sdy = _q(dY, oracle.E5M2)
    assert (float(sx), float(sw), float(sdy)) == (64.0, 64.0, 8192.0)
    Xi, Wi, dYi = X.astype(np.int64), W.astype(np.int64), dY.astype(np.int64)
    # brute force in Python integers, written index by index
    Y = [[sum(int(Xi[m, k]) * int(Wi[n, k]) for k in range(K)) for n in range(N)] for m in range(M)]
    dX = [[sum(int(dYi[m, n]) * int(Wi[n, k]) for n in range(N)) for k in range(K)] for m in range(M)]
    dW = [[sum(int(dYi[m, n]) * int(Xi[m, k]) for m in range(M)) for k in range(K)] for n in range(N)]
    y, S = oracle.gemm_tn(Xq, oracle.E4M3, Wq, oracle.E4M3, sx, sw)
    assert y.shape == (M, N) and np.array_equal(y, np.array(Y, dtype=np.float64))
    Sb = [[sum(abs(int(Xi[m, k]) * int(Wi[n, k])) for k in range(K)) for n in range(N)] for m in range(M)]
    assert np.array_equal(S, np.array(Sb, dtype=np.float64))
    dx, _ = oracle.gemm_tn(dYq, oracle.E5M2, Wqt, oracle.E4M3, sdy, sw)
    assert dx.shape == (M, K) and np.array_equal(dx, np.array(dX, dtype=np.float64))
    dw, _ = oracle.gemm_tn(dYqt, oracle.E5M2, Xqt, oracle.E4M3, sdy, sx)
    assert dw.shape == (N, K) and np.array_equal(dw, np.array(dW, dtype=np.float64))


def test_against_library_matmul_on_decoded_values():
    cfg = synth.CONFIGS[1]
    M, K, N = 48, 96, 40
    x = synth.make_x(cfg, 0, M=M)[:, :K].contiguous()
    w = synth.make_w(cfg, 0)[:N, :K].contiguous()
    xb, wb = synth.bf16_bits(x), synth.bf16_bits(w)
    sx = oracle.scale(oracle.amax_bf16(xb), oracle.E4M3)
    sw = oracle.scale(oracle.amax_bf16(wb), oracle.E4M3)
    xq, _ = oracle.quantize(xb, sx, oracle.E4M3)
    wq, _ = oracle.quantize(wb, sw, oracle.E4M3)
    tab = oracle.decode_table(oracle.E4M3)
    want = (tab[xq] @ tab[wq].T) / (float(sx) * float(sw))
    wantS = (np.abs(tab[xq]) @ np.abs(tab[wq]).T) / (float(sx) * float(sw))
    y, S = oracle.gemm_tn(xq, oracle.E4M3, wq, oracle.E4M3, sx, sw)
    assert np.allclose(y, want, rtol=0, atol=1e-12 * wantS.max())
    assert np.allclose(S, wantS, rtol=1e-13, atol=0)
    # and it approximates the unquantised product to FP8 accuracy: the whole point of the scaling
    exact = x.double().numpy() @ w.double().numpy().T
    assert np.abs(y - exact).max() <= 2 * 2.0 ** -4 * wantS.max()
    # mixed formats, rectangular, sampled == full
    dy = synth.make_dy(cfg, 0, M=M)[:, :N].contiguous()
    dyb = synth.bf16_bits(dy)
    sdy = oracle.scale(oracle.amax_bf16(dyb), oracle.E5M2)
    dyq, dyqt = oracle.quantize(dyb, sdy, oracle.E5M2)
    _, wqt = oracle.quantize(wb, sw, oracle.E4M3)
    t5 = oracle.decode_table(oracle.E5M2)
    want = (t5[dyq] @ tab[wqt].T) / (float(sdy) * float(sw))
    dx, Sdx = oracle.gemm_tn(dyq, oracle.E5M2, wqt, oracle.E4M3, sdy, sw)
    assert dx.shape == (M, K) and np.allclose(dx, want, rtol=0, atol=1e-12 * Sdx.max())
    rng = np.random.default_rng(5)
    rr, cc = rng.integers(0, M, 64), rng.integers(0, K, 64)
    ys, Ss = oracle.gemm_tn_sampled(dyq, oracle.E5M2, wqt, oracle.E4M3, sdy, sw, rr, cc)
    assert np.array_equal(ys, dx[rr, cc]) and np.array_equal(Ss, Sdx[rr, cc])
    with pytest.raises(IndexError):
        oracle.gemm_tn_sampled(dyq, oracle.E5M2, wqt, oracle.E4M3, sdy, sw, [M], [0])


def test_adjoint_identity_ties_forward_dgrad_wgrad():
    """<dY, X W^T> = <dY W, X> = <dY^T X, W> on the dequantised operands."""
    cfg = synth.CONFIGS[1]
    M, K, N = 40, 56, 24
    x = synth.make_x(cfg, 0, M=M)[:, :K].contiguous()
    w = synth.make_w(cfg, 0)[:N, :K].contiguous()
    dy = synth.make_dy(cfg, 0, M=M)[:, :N].contiguous()
    xb, wb, dyb = (synth.bf16_bits(t) for t in (x, w, dy))
    # use E4M3 for all three so that every operand has one decoded value on both sides
    sx, sw, sd = (oracle.scale(oracle.amax_bf16(b), oracle.E4M3) for b in (xb, wb, dyb))
    xq, xqt = oracle.quantize(xb, sx, oracle.E4M3)
    wq, wqt = oracle.quantize(wb, sw, oracle.E4M3)
    dq, dqt = oracle.quantize(dyb, sd, oracle.E4M3)
    tab = oracle.decode_table(oracle.E4M3)
    X, W, D = tab[xq] / float(sx), tab[wq] / float(sw), tab[dq] / float(sd)
    y, _ = oracle.gemm_tn(xq, 0, wq, 0, sx, sw)
    dx, _ = oracle.gemm_tn(dq, 0, wqt, 0, sd, sw)
    dw, _ = oracle.gemm_tn(dqt, 0, xqt, 0, sd, sx)
    a, b, c = np.sum(D * y), np.sum(dx * X), np.sum(dw * W)
    scale_ = np.sum(np.abs(D) * (np.abs(X) @ np.abs(W).T))
    assert abs(a - b) <= 1e-12 * scale_ and abs(a - c) <= 1e-12 * scale_ and abs(a) > 1e-6 * scale_


def test_planted_mistakes_would_be_caught():
    """The integer brute-force pin has teeth: a transposed or swapped operand changes the result."""
    rng = np.random.default_rng(1)
    X = _int_tensor(rng, (6, 8))
    W = _int_tensor(rng, (6, 8))
    Xq, Xqt, sx = _q(X, oracle.E4M3)
    Wq, Wqt, sw = _q(W, oracle.E4M3)
    good, _ = oracle.gemm_tn(Xq, 0, Wq, 0, sx, sw)
    swapped, _ = oracle.gemm_tn(Wq, 0, Xq, 0, sx, sw)
    assert np.array_equal(good, X.astype(np.float64) @ W.astype(np.float64).T)
    assert np.array_equal(swapped, good.T) and not np.array_equal(swapped, good)
    wrong_fmt, _ = oracle.gemm_tn(Xq, 1, Wq, 0, sx, sw)
    assert not np.array_equal(wrong_fmt, good)
