"""Pins for the oracle's BF16 / FP8 encode and decode (CPU only).

None of these retypes the oracle's own formula: they use the landmark values of the format
specification (tests/golden/ocp_fp8_formats.txt), PyTorch's own CPU float8 casts as an independent
library implementation, and properties that any correct round-to-nearest-even saturating cast
must have (round trip, midpoints go to the even neighbour, monotone, saturation).
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle

FMTS = [(oracle.E4M3, torch.float8_e4m3fn, 448.0, 0x7E), (oracle.E5M2, torch.float8_e5m2, 57344.0, 0x7B)]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ocp_fp8_formats.txt")


def _torch_decode(tdtype):
    return torch.arange(256, dtype=torch.uint8).view(tdtype).to(torch.float64).numpy()


def test_golden_landmarks():
    n = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, code, val = line.split()
        fmt = {"e4m3": oracle.E4M3, "e5m2": oracle.E5M2}[name]
        got = oracle.fp8_decode(int(code, 16), fmt)
        want = float(val)
        if math.isnan(want):
            assert math.isnan(got), line
        else:
            assert got == want and math.copysign(1, got) == math.copysign(1, want), line
            if math.isfinite(want):
                assert oracle.fp8_encode(want, fmt) == int(code, 16), line
        n += 1
    assert n >= 30


@pytest.mark.parametrize("fmt,tdtype,fmax,maxcode", FMTS)
def test_decode_all_codes_vs_library(fmt, tdtype, fmax, maxcode):
    want = _torch_decode(tdtype)
    got = oracle.decode_table(fmt)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))
    assert got[maxcode] == fmax == oracle.fp8_max(fmt)
    finite = got[np.isfinite(got)]
    assert finite.max() == fmax and finite.min() == -fmax


@pytest.mark.parametrize("fmt,tdtype,fmax,maxcode", FMTS)
def test_round_trip_every_finite_code(fmt, tdtype, fmax, maxcode):
    tab = oracle.decode_table(fmt)
    for c in range(256):
        if math.isfinite(tab[c]):
            assert oracle.fp8_encode(tab[c], fmt) == c, hex(c)


@pytest.mark.parametrize("fmt,tdtype,fmax,maxcode", FMTS)
def test_midpoints_go_to_even_and_neighbours_to_nearest(fmt, tdtype, fmax, maxcode):
    tab = oracle.decode_table(fmt)
    pos = [c for c in range(0x80) if math.isfinite(tab[c])]
    assert pos == list(range(maxcode + 1))        # positive finite codes are ordered like their values
    for c in pos[:-1]:
        lo, hi = tab[c], tab[c + 1]
        mid = np.float32((lo + hi) / 2)
        assert float(mid) == (lo + hi) / 2          # midpoints are binary32 numbers
        even = c if c % 2 == 0 else c + 1
        below = np.nextafter(mid, np.float32(0))
        above = np.nextafter(mid, np.float32(np.inf))
        for sgn, sbit in ((1.0, 0), (-1.0, 0x80)):
            assert oracle.fp8_encode(sgn * float(mid), fmt) == even | sbit
            assert oracle.fp8_encode(sgn * float(below), fmt) == c | sbit
            assert oracle.fp8_encode(sgn * float(above), fmt) == (c + 1) | sbit


@pytest.mark.parametrize("fmt,tdtype,fmax,maxcode", FMTS)
def test_saturation_and_specials(fmt, tdtype, fmax, maxcode):
    big = [np.nextafter(np.float32(fmax), np.float32(np.inf)), fmax * 1.04, fmax * 1.08, 1e30,
           3.4028234e38, float("inf")]
    for v in big:
        assert oracle.fp8_encode(float(v), fmt) == maxcode
        assert oracle.fp8_encode(-float(v), fmt) == maxcode | 0x80
    assert oracle.fp8_encode(float("nan"), fmt) & 0x7F == 0x7F
    assert oracle.fp8_encode(0.0, fmt) == 0x00
    assert oracle.fp8_encode(-0.0, fmt) == 0x80
    tiny = oracle.decode_table(fmt)[1] / 4          # rounds to zero, sign kept
    assert oracle.fp8_encode(tiny, fmt) == 0x00
    assert oracle.fp8_encode(-tiny, fmt) == 0x80
    assert oracle.fp8_encode(1e-45, fmt) == 0x00


def _sweep_patterns():
    """binary32 patterns: every upper half with the lower halves where rounding decisions flip,
    plus seeded random patterns."""
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint32)
    grid = (hi[:, None] | lows[None, :]).ravel()
    rng = np.random.default_rng(7)
    rnd = rng.integers(0, 1 << 32, size=1 << 22, dtype=np.uint64).astype(np.uint32)
    return np.concatenate([grid, rnd])


@pytest.mark.parametrize("fmt,tdtype,fmax,maxcode", FMTS)
def test_encode_vs_library_cast_in_range(fmt, tdtype, fmax, maxcode):
    """PyTorch's CPU cast is an independent RNE implementation; it does not saturate, so only
    |p| <= FMAX is compared."""
    bits = _sweep_patterns()
    p = bits.view(np.float32)
    keep = np.abs(p) <= np.float32(fmax)            # drops NaN and out-of-range
    p = np.ascontiguousarray(p[keep])
    want = torch.from_numpy(p).to(tdtype).view(torch.uint8).numpy()
    got = oracle.fp8_encode_array(p, fmt)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, (p[bad[:5]], got[bad[:5]], want[bad[:5]])


@pytest.mark.parametrize("fmt,tdtype,fmax,maxcode", FMTS)
def test_encode_is_monotone_and_never_special(fmt, tdtype, fmax, maxcode):
    bits = _sweep_patterns()
    p = bits.view(np.float32)
    p = np.sort(p[~np.isnan(p)])
    codes = oracle.fp8_encode_array(np.ascontiguousarray(p), fmt)
    vals = oracle.decode_table(fmt)[codes]
    assert np.all(np.isfinite(vals))                # no Inf/NaN code from any non-NaN input
    assert np.all(np.diff(vals) >= 0)
    # nearest: the error never exceeds half the local spacing (for in-range inputs)
    inr = np.abs(p) <= fmax
    tab = np.sort(oracle.decode_table(fmt)[np.isfinite(oracle.decode_table(fmt))])
    err = np.abs(vals[inr] - p[inr].astype(np.float64))
    nearest = np.min(np.abs(tab[None, :] - p[inr][::997, None].astype(np.float64)), axis=1)
    assert np.array_equal(err[::997], nearest)


def test_bf16_decode_and_round():
    bits = np.arange(1 << 16, dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.bf16_to_f32(int(b)) for b in bits[::7]], dtype=np.float32)
    w = want[::7]
    ok = ~np.isnan(w)
    assert np.array_equal(got[ok], w[ok]) and np.all(np.isnan(got[~ok]))
    # binary64 -> BF16 against the library's round-to-nearest-even
    rng = np.random.default_rng(3)
    v = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-30, 30, 20000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895e38, 1e-40, -1e-45])])
    v32 = v.astype(np.float32)
    want = torch.from_numpy(v32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f64_to_bf16(float(x)) for x in v32], dtype=np.uint16)
    assert np.array_equal(got, want)
