"""Pins for the oracle's SwiGLU (CPU only).

The paper (Section 3, kernel-fusion paragraph; Section 3 "Activation checkpointing") gives the
non-linearity extra outputs -- absmax of the result, and FP8 bytes when the absmax is known -- but no
new arithmetic: what has to be right is SwiGLU itself, its derivative and the tensor layout.  The
checks: closed forms and identities of the logistic function, a library SiLU in binary64 and in
BF16, finite differences and library autograd for the backward pass, hand-computed cases that fix
the layout, and the binary32 evaluation against the binary64 definition over every BF16 gate value.
"""
import math

import numpy as np
import torch

import oracle
from paper_2512_15306_amd import synth

ALL_BF16 = np.arange(65536, dtype=np.uint32).astype(np.uint16)
FINITE = ALL_BF16[(ALL_BF16 & 0x7F80) != 0x7F80]


def _f32(bits16):
    return (bits16.astype(np.uint32) << 16).view(np.float32)


def _bits(t):
    return synth.bf16_bits(t)


def _bf16(vals):
    return _bits(torch.tensor(vals, dtype=torch.float32).to(torch.bfloat16))


def _half_ulp_bf16(v):
    """Half the BF16 spacing at |v| (v binary64), with the subnormal floor."""
    a = np.maximum(np.abs(v), 2.0 ** -126)
    return 0.5 * 2.0 ** (np.floor(np.log2(a)) - 7)


def _rand_case(seed, M, I, gstd=2.0, ustd=1.5, dstd=1e-3):
    g = torch.Generator().manual_seed(seed)
    gu = torch.cat([torch.randn(M, I, generator=g) * gstd, torch.randn(M, I, generator=g) * ustd], dim=1).to(torch.bfloat16)
    dh = (torch.randn(M, I, generator=g) * dstd).to(torch.bfloat16)
    return gu, dh


def test_logistic_closed_forms_and_identities():
    assert oracle.sigmoid_exact(0.0) == 0.5
    assert abs(oracle.sigmoid_exact(math.log(3.0)) - 0.75) < 1e-15
    assert abs(oracle.sigmoid_exact(-math.log(3.0)) - 0.25) < 1e-15
    for x in np.linspace(-30, 30, 241):
        assert abs(oracle.sigmoid_exact(x) + oracle.sigmoid_exact(-x) - 1.0) < 1e-15
        want = torch.sigmoid(torch.tensor(x, dtype=torch.float64)).item()
        assert abs(oracle.sigmoid_exact(x) - want) <= 1e-15 * max(want, 1e-300) + 1e-300
    assert oracle.sigmoid_exact(800.0) == 1.0 and oracle.sigmoid_exact(-800.0) == 0.0


def test_binary32_logistic_tracks_the_definition_for_every_bf16_gate():
    worst = 0.0
    for b in FINITE:
        g = float(_f32(np.array([b], np.uint16))[0])
        got = float(oracle.sigmoid_f32(g))
        want = oracle.sigmoid_exact(g)
        if g >= -87.0:
            rel = abs(got - want) / want
            worst = max(worst, rel)
        elif g <= -89.0:
            assert got == 0.0 and want < 2.3e-39       # e^-g overflows binary32: the quotient is 1/Inf
        else:
            assert abs(got - want) <= 2.0 ** -148      # subnormal quotient
    assert worst <= 2.0 ** -21, worst
    assert float(oracle.sigmoid_f32(0.0)) == 0.5
    assert float(oracle.sigmoid_f32(30.0)) == 1.0      # 1 + e^-30 rounds to 1


def test_forward_definition_against_library_silu_in_binary64():
    gu, _ = _rand_case(5, 37, 53)
    g, u = gu[:, :53].double(), gu[:, 53:].double()
    want = (torch.nn.functional.silu(g) * u).numpy()
    got = oracle.swiglu_fwd_exact(_bits(gu))
    np.testing.assert_allclose(got, want, rtol=1e-14, atol=0)
    # silu(x) - silu(-x) = x  (because sigma(x) + sigma(-x) = 1): ties the sign conventions down
    x = torch.linspace(-20, 20, 64).to(torch.bfloat16)
    ones = torch.ones_like(x)
    p = oracle.swiglu_fwd_exact(_bits(torch.stack([x, ones], 0).reshape(1, -1)))
    m = oracle.swiglu_fwd_exact(_bits(torch.stack([-x, ones], 0).reshape(1, -1)))
    np.testing.assert_allclose(p - m, x.double().numpy().reshape(1, -1), rtol=0, atol=1e-14)


def test_layout_and_hand_computed_cases():
    # one row, I = 4: gate columns first, then up
    gu = _bf16([[0.0, 64.0, -200.0, 1.0, 3.0, 0.5, 7.0, 0.0]])
    h = oracle.swiglu_fwd(gu)
    assert h.shape == (1, 4)
    # g = 0 -> 0 ; g = 64 -> sigma rounds to 1, h = 64 * 0.5 ; g = -200 -> -0 ; u = 0 -> 0
    assert list(h[0]) == [0x0000, int(_bf16([32.0])[0]), 0x8000, 0x0000]
    # swapping the halves is a different function (planted-mistake check)
    swapped = np.concatenate([gu[:, 4:], gu[:, :4]], axis=1)
    assert list(oracle.swiglu_fwd(swapped)[0]) != list(h[0])
    # two rows: row-major, row m reads only row m of GU
    gu2 = np.concatenate([gu, _bf16([[64.0, 0.0, 0.0, 0.0, 2.0, 1.0, 1.0, 1.0]])], axis=0)
    h2 = oracle.swiglu_fwd(gu2)
    assert list(h2[0]) == list(h[0]) and list(h2[1]) == [int(_bf16([128.0])[0]), 0, 0, 0]
    # backward: g = 0: sigma = 1/2, d/dg = dh u / 2, d/du = 0 ; g = 64: d/dg = dh u, d/du = 64 dh
    dh = _bf16([[2.0, 2.0, 2.0, 2.0]])
    d = oracle.swiglu_bwd(dh, gu)
    assert d.shape == (1, 8)
    want_dg = [3.0, 1.0, None, None]
    want_du = [0.0, 128.0, None, 2.0 * 1.0 * float(oracle.sigmoid_f32(1.0))]
    for i in range(4):
        if want_dg[i] is not None:
            assert d[0, i] == _bf16([want_dg[i]])[0], i
        if want_du[i] is not None:
            assert d[0, 4 + i] == _bf16([want_du[i]])[0], i
    assert (d[0, 2] & 0x7FFF) == 0 and (d[0, 6] & 0x7FFF) == 0      # g = -200: both derivatives vanish


def test_forward_bits_are_the_rounded_definition():
    gu, _ = _rand_case(7, 64, 96, gstd=3.0)
    bits = oracle.swiglu_fwd(_bits(gu))
    got = _f32(bits).astype(np.float64)
    want = oracle.swiglu_fwd_exact(_bits(gu))
    # one rounding to BF16 of a binary32 value that is within a few binary32 ulps of the definition
    bound = _half_ulp_bf16(want) * (1 + 2.0 ** -9) + np.abs(want) * 2.0 ** -20
    assert (np.abs(got - want) <= bound).all()
    # an independent BF16 pipeline (library SiLU in binary32, product, cast) agrees except at rounding ties
    g, u = gu[:, :96].float(), gu[:, 96:].float()
    lib = _bits((torch.nn.functional.silu(g) * u).to(torch.bfloat16))
    diff = np.abs(bits.astype(np.int32) - lib.astype(np.int32))
    assert diff.max() <= 1 and (diff != 0).mean() < 5e-3


def test_forward_for_every_bf16_gate_value():
    g = FINITE
    for uval in (1.0, -3.0, 2.0 ** -100):
        u = np.full_like(g, _bf16([uval])[0])
        gu = np.concatenate([g[None, :], u[None, :]], axis=1)
        got = _f32(oracle.swiglu_fwd(gu)).astype(np.float64)
        want = oracle.swiglu_fwd_exact(gu)
        with np.errstate(over="ignore"):
            bound = _half_ulp_bf16(want) * (1 + 2.0 ** -9) + np.abs(want) * 2.0 ** -20
        # g <= -89: e^-g overflows binary32 and the result is +-0 where the definition is below 2^-121 |u|
        bound = bound + abs(uval) * 2.0 ** -121
        ok = np.abs(got - want) <= bound
        # products beyond the BF16 range round to Inf, as IEEE rounding prescribes
        over = np.abs(want) >= 2.0 ** 128 * (1 - 2.0 ** -9)
        assert (ok | (over & np.isinf(got))).all()


def test_backward_definition_by_finite_differences_and_autograd():
    gu, dh = _rand_case(9, 8, 16, dstd=1.0)
    exact = oracle.swiglu_bwd_exact(_bits(dh), _bits(gu))
    g = gu[:, :16].double().requires_grad_(True)
    u = gu[:, 16:].double().requires_grad_(True)
    (torch.nn.functional.silu(g) * u).backward(dh.double())
    np.testing.assert_allclose(exact[:, :16], g.grad.numpy(), rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(exact[:, 16:], u.grad.numpy(), rtol=1e-12, atol=1e-300)

    def f(gv, uv):
        return gv * oracle.sigmoid_exact(gv) * uv

    gd, ud, dd = gu[:, :16].double().numpy(), gu[:, 16:].double().numpy(), dh.double().numpy()
    eps = 1e-6
    for m in range(2):
        for i in range(16):
            dg = (f(gd[m, i] + eps, ud[m, i]) - f(gd[m, i] - eps, ud[m, i])) / (2 * eps) * dd[m, i]
            du = (f(gd[m, i], ud[m, i] + eps) - f(gd[m, i], ud[m, i] - eps)) / (2 * eps) * dd[m, i]
            assert abs(exact[m, i] - dg) <= 1e-6 * (abs(dg) + abs(dd[m, i] * ud[m, i]))
            assert abs(exact[m, 16 + i] - du) <= 1e-6 * (abs(du) + 1e-12)


def test_backward_bits_are_the_rounded_definition():
    gu, dh = _rand_case(11, 64, 96, gstd=3.0)
    bits = oracle.swiglu_bwd(_bits(dh), _bits(gu))
    got = _f32(bits).astype(np.float64)
    want = oracle.swiglu_bwd_exact(_bits(dh), _bits(gu))
    g, u, d = gu[:, :96].double().numpy(), gu[:, 96:].double().numpy(), dh.double().numpy()
    sg = 1.0 / (1.0 + np.exp(-g))
    # d/dg has a zero near g = -1.28 (1 + g (1 - sigma) cancels): the binary32 error is relative to the
    # terms before the cancellation
    cond = np.concatenate([np.abs(d * u) * sg * (1 + np.abs(g) * (1 - sg)), np.abs(d * g) * sg], axis=1)
    bound = _half_ulp_bf16(want) * (1 + 2.0 ** -9) + cond * 2.0 ** -19
    assert (np.abs(got - want) <= bound).all()
    assert (bits[:, :96] != bits[:, 96:]).any()


def test_extra_outputs_are_compositions():
    """absmax and FP8 bytes of the fused kernels are plain functions of the BF16 result."""
    gu, _ = _rand_case(13, 32, 48)
    h = oracle.swiglu_fwd(_bits(gu))
    a = oracle.amax_bf16(h)
    assert float(a) == float(np.abs(_f32(h)).max())
    s = oracle.scale(a, oracle.E4M3)
    q, qt = oracle.quantize(h, s, oracle.E4M3)
    assert q.max() == 0x7E or (q & 0x7F).max() == 0x7E       # the absmax lands on the largest code
    assert (qt.T == q).all()
