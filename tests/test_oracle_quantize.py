"""Pins for the oracle's absmax, scale and quantize(+transpose) (CPU only).

Section 3 ("Overview") of the paper fixes what must hold: the tensor's largest magnitude is mapped
onto the largest representable FP8 value and nothing is clipped.  The checks below are brute force
with a library (torch/numpy max, torch's float8 cast), invariants of that statement, and exact
special cases.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import synth

FMTS = [(oracle.E4M3, torch.float8_e4m3fn, 448.0, 0x7E), (oracle.E5M2, torch.float8_e5m2, 57344.0, 0x7B)]


def _bits(t):
    return synth.bf16_bits(t)


def _rand_bf16(shape, seed, std=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * std).to(torch.bfloat16)


def test_amax_matches_library_max():
    for seed, shape, std in [(1, (37, 53), 1.0), (2, (1, 1), 3.0), (3, (256, 512), 0.02), (4, (5, 7), 1e-30)]:
        x = _rand_bf16(shape, seed, std)
        want = x.float().abs().max().item()
        assert float(oracle.amax_bf16(_bits(x))) == want
    assert float(oracle.amax_bf16(np.zeros((4, 4), np.uint16))) == 0.0
    assert float(oracle.amax_bf16(np.array([0x8000, 0x0000], np.uint16))) == 0.0   # -0, +0
    # position independence and sign independence
    x = _rand_bf16((64, 64), 9)
    b = _bits(x).copy()
    b[17, 5] = 0xC2C8          # -100.0
    assert float(oracle.amax_bf16(b)) == 100.0
    # non-finite inputs: Inf dominates finite values, NaN dominates everything
    b[3, 3] = 0x7F80
    assert np.isinf(oracle.amax_bf16(b))
    b[60, 1] = 0xFFC1
    a = oracle.amax_bf16(b)
    assert np.isnan(a) and a.view(np.uint32) == 0x7FC00000


@pytest.mark.parametrize("fmt,tdtype,fmax,maxcode", FMTS)
def test_scale_rule(fmt, tdtype, fmax, maxcode):
    # all-zero tensor: the rule defines no scale; the neutral one is taken (-0.0 is zero too)
    assert float(oracle.scale(0.0, fmt)) == 1.0 and float(oracle.scale(np.float32(-0.0), fmt)) == 1.0
    # powers of two: FMAX * 2^j maps with an exact power-of-two scale
    for j in range(-20, 20):
        assert float(oracle.scale(fmax * 2.0 ** j, fmt)) == 2.0 ** (-j)
    assert float(oracle.scale(7.0, fmt)) == fmax / 7.0 == {448.0: 64.0, 57344.0: 8192.0}[fmax]
    # one binary32 division (numpy's float32 division is IEEE)
    rng = np.random.default_rng(11)
    for a in np.abs(rng.standard_normal(2000)).astype(np.float32) * np.float32(10.0) ** rng.integers(-8, 8, 2000).astype(np.float32):
        if a == 0:
            continue
        assert oracle.scale(a, fmt) == np.float32(fmax) / np.float32(a)
    # quotient overflow is clamped to the largest finite binary32
    assert float(oracle.scale(1e-40, fmt)) == float(np.finfo(np.float32).max)


@pytest.mark.parametrize("fmt,tdtype,fmax,maxcode", FMTS)
def test_amax_always_lands_on_fmax_code(fmt, tdtype, fmax, maxcode):
    """'mapped to the largest representable value' for every BF16 amax: q(fl32(a * fl32(FMAX/a)))
    is the FMAX code, for all positive finite BF16 a whose scale does not overflow."""
    bits = np.arange(0x0001, 0x7F80, dtype=np.uint16)
    a = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).float().numpy()
    s = np.float32(fmax) / a
    ok = np.isfinite(s)
    p = (a[ok] * s[ok]).astype(np.float32)
    codes = oracle.fp8_encode_array(np.ascontiguousarray(p), fmt)
    assert np.all(codes == maxcode)
    # and the oracle's own scale agrees on a sample
    for b in bits[ok][::501]:
        av = oracle.bf16_to_f32(int(b))
        assert oracle.scale(av, fmt) == np.float32(fmax) / np.float32(av)


@pytest.mark.parametrize("fmt,tdtype,fmax,maxcode", FMTS)
@pytest.mark.parametrize("shape,std,seed", [((64, 48), 1.0, 5), ((130, 257), 0.02, 6), ((1, 9), 1e-4, 7)])
def test_quantize_against_library_cast_and_invariants(fmt, tdtype, fmax, maxcode, shape, std, seed):
    x = _rand_bf16(shape, seed, std)
    xb = _bits(x)
    a = oracle.amax_bf16(xb)
    s = oracle.scale(a, fmt)
    q, qt = oracle.quantize(xb, s, fmt)
    # independent computation: binary32 multiply in torch, torch's RNE cast (in range by construction
    # except for an upward rounding of amax*s, which is clamped here the way saturation demands)
    p = x.float() * torch.tensor(float(s), dtype=torch.float32)
    p = torch.clamp(p, -fmax, fmax)
    want = p.to(tdtype).view(torch.uint8).numpy()
    assert np.array_equal(q, want)
    assert np.array_equal(qt, q.T)
    assert qt.flags["C_CONTIGUOUS"] and qt.shape == (shape[1], shape[0])
    # nothing clipped, the largest element sits exactly on the FMAX code, no special codes
    mag = q & 0x7F
    assert mag.max() == maxcode
    tab = oracle.decode_table(fmt)
    assert np.all(np.isfinite(tab[q]))
    # dequantisation error: half a unit in the last place of the FP8 grid (normal range)
    deq = tab[q] / float(s)
    xf = x.double().numpy()
    mbits = 3 if fmt == oracle.E4M3 else 2
    min_normal = 2.0 ** -6 if fmt == oracle.E4M3 else 2.0 ** -14
    normal = np.abs(xf * float(s)) >= min_normal
    rel = np.abs(deq - xf)[normal] / np.abs(xf)[normal]
    assert rel.max() <= 2.0 ** (-mbits - 1) * (1 + 2.0 ** -20)
    # no transposed copy requested
    q2, none = oracle.quantize(xb, s, fmt, transpose=False)
    assert none is None and np.array_equal(q2, q)


@pytest.mark.parametrize("fmt,tdtype,fmax,maxcode", FMTS)
def test_quantize_all_zero_and_given_scale(fmt, tdtype, fmax, maxcode):
    z = np.zeros((8, 16), np.uint16)
    z[2, 3] = 0x8000
    s = oracle.scale(oracle.amax_bf16(z), fmt)
    q, qt = oracle.quantize(z, s, fmt)
    assert float(s) == 1.0 and q[2, 3] == 0x80 and np.count_nonzero(q) == 1
    # every finite positive scale gives these same codes: the choice at absmax 0 cannot change a byte
    for other in (np.float32(np.finfo(np.float32).max), np.float32(2.0 ** -100)):
        assert np.array_equal(oracle.quantize(z, other, fmt)[0], q)
    # a scale that is too large saturates instead of overflowing to Inf/NaN codes
    x = _rand_bf16((16, 16), 12, 1.0)
    q, _ = oracle.quantize(_bits(x), np.float32(1e6), fmt)
    assert set(np.unique(q & 0x7F)) <= {0, maxcode} | set(range(maxcode + 1))
    assert (q & 0x7F).max() == maxcode and np.all(np.isfinite(oracle.decode_table(fmt)[q]))


def test_integer_inputs_quantize_losslessly():
    """Integers up to 7 with amax 7: scale is 64 (E4M3) / 8192 (E5M2 covers only {0,1,2,3,4,5,6,7}
    exactly up to its 2 mantissa bits, so restrict E5M2 to {0,1,2,3,4,6} and amax 7)."""
    vals4 = np.array([-7, -6, -5, -4, -3, -2, -1, 0, 1, 2, 3, 4, 5, 6, 7], dtype=np.float32)
    x = torch.from_numpy(np.tile(vals4, (3, 1))).to(torch.bfloat16)
    s = oracle.scale(oracle.amax_bf16(_bits(x)), oracle.E4M3)
    q, _ = oracle.quantize(_bits(x), s, oracle.E4M3)
    assert float(s) == 64.0
    assert np.array_equal(oracle.decode_table(oracle.E4M3)[q] / 64.0, x.double().numpy())
    vals5 = np.array([-7, -6, -4, -3, -2, -1, 0, 1, 2, 3, 4, 6, 7], dtype=np.float32)
    x = torch.from_numpy(np.tile(vals5, (2, 1))).to(torch.bfloat16)
    s = oracle.scale(oracle.amax_bf16(_bits(x)), oracle.E5M2)
    q, _ = oracle.quantize(_bits(x), s, oracle.E5M2)
    assert float(s) == 8192.0
    assert np.array_equal(oracle.decode_table(oracle.E5M2)[q] / 8192.0, x.double().numpy())


def test_config_inputs_have_the_stated_structure():
    cfg = synth.CONFIGS[3]
    x = synth.make_x(cfg, 0, M=512).float()
    col_std = x.std(dim=0)
    n_out = int((col_std > 10).sum())
    assert n_out == round(0.005 * cfg.linears[0].K) == 18
    assert abs(float(col_std[col_std < 10].mean()) - 1.0) < 0.05
    w = synth.make_w(synth.CONFIGS[1], 0).float()
    assert abs(float(w.std()) - 0.02) < 1e-3
    dy = synth.make_dy(synth.CONFIGS[1], 0).float()
    assert abs(float(dy.std()) - 1e-3) < 1e-4
    # same seed, same bytes
    assert torch.equal(synth.make_x(cfg, 0, M=64), synth.make_x(cfg, 0, M=64))
