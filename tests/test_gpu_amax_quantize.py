"""GPU parity: llmq_amax and llmq_quantize_fp8 against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import llmq, synth
from gpu_common import DEV, FMAX, f32_bits, np_f32_bits, gpu_amax, gpu_quantize, oracle_quantized

pytestmark = pytest.mark.gpu


def _randn_bf16(shape, seed, std=1.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * std).to(torch.bfloat16)


@pytest.mark.parametrize("n", [1, 7, 8, 9, 2047, 2048 * 8, 2048 * 8 + 5, 1_000_003, 256 * 512, 4096 * 3072 + 3])
@pytest.mark.parametrize("fmt", [0, 1])
def test_amax_and_scale_bit_exact(n, fmt):
    print("amax n=%d fmt=%d" % (n, fmt), flush=True)
    x = _randn_bf16((n,), 1000 + n % 97, std=0.37)
    a, s = gpu_amax(x.to(DEV), fmt)
    want_a = oracle.amax_bf16(synth.bf16_bits(x))
    want_s = oracle.scale(want_a, fmt)
    assert f32_bits(a) == np_f32_bits(want_a)
    assert f32_bits(s) == np_f32_bits(want_s)
    # without a scale output only the absmax is written
    a2, _ = gpu_amax(x.to(DEV), fmt, want_scale=False)
    assert f32_bits(a2) == np_f32_bits(want_a)


def test_amax_position_and_special_values():
    n = 300_001
    base = _randn_bf16((n,), 5, 0.01)
    for pos in [0, 1, 7, 8, n // 2, n - 9, n - 8, n - 1]:
        x = base.clone()
        x[pos] = -3.0
        a, s = gpu_amax(x.to(DEV), 0)
        assert a.item() == 3.0 and s.item() == np.float32(448.0) / np.float32(3.0), pos
    z = torch.zeros(4099, dtype=torch.bfloat16)
    z[17] = -0.0
    a, s = gpu_amax(z.to(DEV), 1)
    assert f32_bits(a) == 0 and s.item() == 1.0 == float(oracle.scale(0.0, 1))
    # subnormal BF16 values and a scale whose quotient overflows
    tiny = torch.tensor([1e-40, -3e-39, 0.0], dtype=torch.float32).to(torch.bfloat16)
    a, s = gpu_amax(tiny.to(DEV), 0)
    wa = oracle.amax_bf16(synth.bf16_bits(tiny))
    assert f32_bits(a) == np_f32_bits(wa) and f32_bits(s) == np_f32_bits(oracle.scale(wa, 0))
    assert s.item() == float(np.finfo(np.float32).max)
    # Inf and NaN propagate as documented
    x = base.clone()
    x[12345] = float("-inf")
    a, _ = gpu_amax(x.to(DEV), 0)
    assert f32_bits(a) == 0x7F800000
    x[777] = float("nan")
    a, _ = gpu_amax(x.to(DEV), 0)
    assert f32_bits(a) == 0x7FC00000 == np_f32_bits(oracle.amax_bf16(synth.bf16_bits(x)))


QSHAPES = [(256, 512), (1024, 512), (272, 400), (128, 64), (16, 8), (48, 1032), (100, 72), (33, 17), (1, 1), (5, 4096)]


@pytest.mark.parametrize("shape", QSHAPES)
@pytest.mark.parametrize("fmt", [0, 1])
def test_quantize_bit_exact(shape, fmt):
    print("quantize shape=%s fmt=%d" % (shape, fmt), flush=True)
    x = _randn_bf16(shape, 77 + shape[0] + shape[1], std=[1.0, 1e-3][fmt])
    wa, ws, wq, wqt = oracle_quantized(x, fmt)
    xd = x.to(DEV)
    a, s = gpu_amax(xd, fmt)
    q, qt = gpu_quantize(xd, s, fmt)
    assert f32_bits(s) == np_f32_bits(ws)
    assert np.array_equal(q.cpu().numpy(), wq)
    assert np.array_equal(qt.cpu().numpy(), wqt)
    q2, none = gpu_quantize(xd, s, fmt, transpose=False)
    assert none is None and torch.equal(q2, q)
    # determinism: same bytes on a second run
    q3, qt3 = gpu_quantize(xd, s, fmt)
    assert torch.equal(q3, q) and torch.equal(qt3, qt)


@pytest.mark.parametrize("fmt", [0, 1])
def test_quantize_every_bf16_value_under_many_scales(fmt):
    """All 65536 BF16 patterns as inputs, under scales that put products on, just below and just above
    rounding ties, far out of range (saturation) and deep in the subnormal range."""
    bits = np.arange(1 << 16, dtype=np.uint16)
    finite = (bits & 0x7F80) != 0x7F80                  # NaN/Inf inputs are unspecified
    xb = bits[finite]
    pad = (-len(xb)) % 128
    xb = np.concatenate([xb, np.zeros(pad, np.uint16)]).reshape(-1, 128)
    x = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16)
    xd = x.to(DEV)
    scales = [1.0, 1.0 + 2.0 ** -23, 1.0 - 2.0 ** -24, 1.0 + 2.0 ** -22, 0.999, 1.337, 3.0, 1.0 / 3.0,
              448.0 / 3.3, 57344.0 / 0.011, 1e6, 1e-6, 2.0 ** -9, 2.0 ** -16, 2.0 ** 20, 2.0 ** -30, 1e30, 1e-30,
              3.4028234e38]
    for sc in scales:
        print("sweep fmt=%d scale=%r" % (fmt, sc), flush=True)
        s = torch.tensor([sc], dtype=torch.float32, device=DEV)
        q, qt = gpu_quantize(xd, s, fmt)
        wq, wqt = oracle.quantize(xb, np.float32(sc), fmt)
        got = q.cpu().numpy()
        bad = np.argwhere(got != wq)
        assert bad.size == 0, (sc, hex(xb[tuple(bad[0])]), hex(got[tuple(bad[0])]), hex(wq[tuple(bad[0])]))
        assert np.array_equal(qt.cpu().numpy(), wqt)
        q_only, _ = gpu_quantize(xd, s, fmt, transpose=False)       # the kernel without a transposed copy
        assert np.array_equal(q_only.cpu().numpy(), wq)


def test_config_tensors_quantize_bit_exact_at_full_size():
    """Config 3 (7B-class) qkv activations with outlier channels and config 5's heavy-tailed
    activations, whole tensors, both outputs."""
    for cfg_i, li, which, fmt in [(3, 0, "x", 0), (5, 1, "x", 0), (2, 1, "dy", 1), (3, 1, "w", 0)]:
        cfg = synth.CONFIGS[cfg_i]
        print("full-size quantize config %d %s %s" % (cfg_i, cfg.linears[li].name, which), flush=True)
        t = {"x": synth.make_x, "w": synth.make_w, "dy": synth.make_dy}[which](cfg, li, device=DEV)
        a, s = gpu_amax(t, fmt)
        q, qt = gpu_quantize(t, s, fmt)
        wa, ws, wq, wqt = oracle_quantized(t, fmt)
        assert f32_bits(a) == np_f32_bits(wa) and f32_bits(s) == np_f32_bits(ws)
        assert np.array_equal(q.cpu().numpy(), wq)
        assert np.array_equal(qt.cpu().numpy(), wqt)
        assert (wq & 0x7F).max() == {0: 0x7E, 1: 0x7B}[fmt]
        q_only, _ = gpu_quantize(t, s, fmt, transpose=False)
        assert torch.equal(q_only, q)
        del t, q, qt, q_only
