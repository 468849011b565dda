"""Pins for the oracle's RMSNorm + residual addition (CPU only).

Section 3 (kernel-fusion paragraph) of the paper joins the residual addition with the RMS-norm and has the
kernel return the absmax of the normalised output.  What has to be right: the addition and its rounding,
the definition of the norm (mean of squares over the row, eps inside the root, weight per column), and the
binary32 normalisation that decides the stored bits once the row statistic is given.
"""
import numpy as np
import torch

import oracle
from paper_2512_15306_amd import synth


def _bits(t):
    return synth.bf16_bits(t)


def _f32(bits16):
    return (bits16.astype(np.uint32) << 16).view(np.float32)


def _rand(shape, seed, std=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * std).to(torch.bfloat16)


def _half_ulp_bf16(v):
    a = np.maximum(np.abs(v), 2.0 ** -126)
    return 0.5 * 2.0 ** (np.floor(np.log2(a)) - 7)


def test_residual_add_is_the_library_bf16_addition():
    r, x = _rand((37, 53), 1, 2.0), _rand((37, 53), 2, 0.3)
    assert np.array_equal(oracle.residual_add(_bits(r), _bits(x)), _bits(r + x))
    # exact cases and a tie: 1 + 2^-8 lies half way between 1 and the next BF16 number and goes to even
    one, tie, tiny = 0x3F80, 0x3B80, 0x0001
    assert list(oracle.residual_add(np.array([one, one, one], np.uint16), np.array([one, tie, tiny], np.uint16))) == [0x4000, 0x3F80, 0x3F80]
    assert list(oracle.residual_add(np.array([0x3F81], np.uint16), np.array([tie], np.uint16))) == [0x3F82]
    # not commutative mistakes: x - r would fail here
    assert list(oracle.residual_add(_bits(torch.tensor([3.0]).bfloat16()), _bits(torch.tensor([-1.0]).bfloat16()))) == [0x4000]


def test_definition_against_library_rms_norm_in_binary64():
    res, w = _rand((29, 96), 3, 1.7), _rand((96,), 4, 1.0)
    for eps in (0.0, 1e-6, 1e-2):
        want = torch.nn.functional.rms_norm(res.double(), (96,), w.double(), eps).numpy()
        got = oracle.rmsnorm_exact(_bits(res), _bits(w), eps)
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=0)
        rstd = oracle.rms_rstd(_bits(res), eps)
        np.testing.assert_allclose(rstd, 1.0 / np.sqrt((res.double().numpy() ** 2).mean(axis=1) + eps), rtol=1e-14)


def test_closed_forms_and_invariants():
    C = 24
    w = _rand((C,), 5)
    wb = _bits(w)
    # a constant row c has mean square c^2: y = sign(c) w for eps = 0
    for cval in (1.0, -2.0, 0.5):
        row = torch.full((1, C), cval).bfloat16()
        y = oracle.rmsnorm_exact(_bits(row), wb, 0.0)
        np.testing.assert_allclose(y[0], np.sign(cval) * w.double().numpy(), rtol=1e-15)
        assert abs(oracle.rms_rstd(_bits(row), 0.0)[0] - 1.0 / abs(cval)) < 1e-15
    # eps sits inside the root: an all-zero row has rstd = eps^-1/2 and y = 0
    z = np.zeros((1, C), np.uint16)
    assert abs(oracle.rms_rstd(z, 0.25)[0] - 2.0) < 1e-15
    assert (oracle.rmsnorm_exact(z, wb, 0.25) == 0).all()
    # scale invariance for eps = 0 (powers of two are exact in BF16), and mean((y/w)^2) = 1
    res = _rand((6, C), 6)
    y1 = oracle.rmsnorm_exact(_bits(res), wb, 0.0)
    y2 = oracle.rmsnorm_exact(_bits((res.float() * 8.0).bfloat16()), wb, 0.0)
    np.testing.assert_allclose(y1, y2, rtol=1e-14)
    ones = _bits(torch.ones(C).bfloat16())
    yn = oracle.rmsnorm_exact(_bits(res), ones, 0.0)
    np.testing.assert_allclose((yn ** 2).mean(axis=1), 1.0, rtol=1e-14)
    # rows are independent and the weight runs along columns (a per-row weight would fail on this shape)
    res2 = _rand((C + 3, C), 7)
    full = oracle.rmsnorm_exact(_bits(res2), wb, 1e-6)
    for m in (0, 5, C + 2):
        np.testing.assert_array_equal(full[m], oracle.rmsnorm_exact(_bits(res2[m:m + 1]), wb, 1e-6)[0])
    assert not np.allclose(full[:, 0] / res2[:, 0].double().numpy() * 1.0, full[:, 1] / res2[:, 1].double().numpy())


def test_apply_is_the_rounded_definition_given_the_statistic():
    res, w = _rand((64, 160), 8, 3.0), _rand((160,), 9)
    eps = 1e-6
    rstd64 = oracle.rms_rstd(_bits(res), eps)
    rstd = rstd64.astype(np.float32)
    bits = oracle.rmsnorm_apply(_bits(res), _bits(w), rstd)
    got = _f32(bits).astype(np.float64)
    want = oracle.rmsnorm_exact(_bits(res), _bits(w), eps)
    bound = _half_ulp_bf16(want) * (1 + 2.0 ** -9) + np.abs(want) * 2.0 ** -21
    assert (np.abs(got - want) <= bound).all()
    # exactly representable case: rstd = 0.5, w = 3 -> y = 1.5 res
    r2 = torch.tensor([[2.0, -2.0, 2.0, -2.0]]).bfloat16()
    y = oracle.rmsnorm_apply(_bits(r2), _bits(torch.full((4,), 3.0).bfloat16()), np.array([0.5], np.float32))
    assert list(_f32(y)[0]) == [3.0, -3.0, 3.0, -3.0]
    # the statistic is per row: swapping two rows' statistics changes the result
    sw = rstd.copy()
    sw[[0, 1]] = sw[[1, 0]]
    assert not np.array_equal(oracle.rmsnorm_apply(_bits(res), _bits(w), sw), bits)
    # an independent BF16 pipeline (library ops in binary32) agrees up to rounding ties
    lib = _bits(((res.float() * torch.from_numpy(rstd)[:, None]) * w.float()).to(torch.bfloat16))
    assert np.array_equal(lib, bits)
