"""GPU parity: SwiGLU with fused absmax / fused FP8 output (forward, recompute mode, backward) against
the oracle, bit for bit: BF16 results, absmax, scale and FP8 bytes."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import llmq, synth
from gpu_common import DEV, f32_bits, np_f32_bits, gpu_amax, gpu_quantize

pytestmark = pytest.mark.gpu

# (M, I): tuned patches (M % 4 == 0, I % 8 == 0; with q_t M % 16 == 0), partial column blocks, generic shapes,
# whole 128 x 256 tiles (their own kernel when q_t is written)
SHAPES = [(32, 256), (64, 264), (128, 512), (36, 40), (16, 8), (4, 8), (33, 17), (1, 1), (7, 24), (48, 1032), (260, 768),
          (128, 256), (384, 768)]


def _case(M, I, seed, gstd=2.0, ustd=1.5, dstd=1e-3):
    g = torch.Generator(device="cpu").manual_seed(seed)
    gu = torch.cat([torch.randn(M, I, generator=g) * gstd, torch.randn(M, I, generator=g) * ustd], dim=1).to(torch.bfloat16)
    dh = (torch.randn(M, I, generator=g) * dstd).to(torch.bfloat16)
    return gu, dh


def _ws(M, I):
    n = llmq.llmq_swiglu_workspace_bytes(M, I)
    assert n >= 4
    return torch.full((n,), 0xFF, device=DEV, dtype=torch.uint8)       # garbage on entry


def _bits_of(t):
    return synth.bf16_bits(t)


def gpu_swiglu_fwd(gu, fmt, want_scale=True):
    M, I = gu.shape[0], gu.shape[1] // 2
    h = torch.full((M, I), -7.0, device=DEV, dtype=torch.bfloat16)
    a = torch.full((1,), -1.0, device=DEV)
    s = torch.full((1,), -1.0, device=DEV) if want_scale else None
    llmq.llmq_swiglu_fwd(gu, h, fmt, a, s, _ws(M, I))
    return h, a, s


def gpu_swiglu_fp8(gu, d_scale, fmt, transpose=True, want_h=False):
    M, I = gu.shape[0], gu.shape[1] // 2
    q = torch.full((M, I), 0xAA, device=DEV, dtype=torch.uint8)
    qt = torch.full((I, M), 0xAA, device=DEV, dtype=torch.uint8) if transpose else None
    h = torch.full((M, I), -7.0, device=DEV, dtype=torch.bfloat16) if want_h else None
    llmq.llmq_swiglu_fwd_fp8(gu, d_scale, fmt, q, qt, h)
    return q, qt, h


def gpu_swiglu_bwd(dh, gu, fmt):
    M, I = dh.shape
    dgu = torch.full((M, 2 * I), -7.0, device=DEV, dtype=torch.bfloat16)
    a = torch.full((1,), -1.0, device=DEV)
    s = torch.full((1,), -1.0, device=DEV)
    llmq.llmq_swiglu_bwd(dh, gu, dgu, fmt, a, s, _ws(M, I))
    return dgu, a, s


def _assert_bits(got_t, want_bits, what):
    got = _bits_of(got_t).reshape(want_bits.shape)
    bad = np.argwhere(got != want_bits)
    assert bad.size == 0, "%s: %d mismatches, first at %s: got %#06x want %#06x" % (
        what, len(bad), bad[0], got[tuple(bad[0])], want_bits[tuple(bad[0])])


@pytest.mark.parametrize("shape", SHAPES)
def test_forward_result_absmax_and_scale_bit_exact(shape):
    M, I = shape
    print("swiglu fwd M=%d I=%d" % shape, flush=True)
    gu, _ = _case(M, I, 500 + M + I)
    want_h = oracle.swiglu_fwd(_bits_of(gu))
    want_a = oracle.amax_bf16(want_h)
    for fmt in (0, 1):
        h, a, s = gpu_swiglu_fwd(gu.to(DEV), fmt)
        _assert_bits(h, want_h, "h")
        assert f32_bits(a) == np_f32_bits(want_a)
        assert f32_bits(s) == np_f32_bits(oracle.scale(want_a, fmt))
    h2, a2, none = gpu_swiglu_fwd(gu.to(DEV), 0, want_scale=False)
    assert none is None and f32_bits(a2) == np_f32_bits(want_a) and torch.equal(h2, h)
    # the fused absmax is what the separate reduction gives for the tensor the kernel wrote
    a3, s3 = gpu_amax(h, 1)
    assert f32_bits(a3) == f32_bits(a) and f32_bits(s3) == f32_bits(s)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("fmt", [0, 1])
def test_recompute_mode_fp8_bytes_bit_exact(shape, fmt):
    M, I = shape
    print("swiglu fwd_fp8 M=%d I=%d fmt=%d" % (M, I, fmt), flush=True)
    gu, _ = _case(M, I, 900 + M + I)
    want_h = oracle.swiglu_fwd(_bits_of(gu))
    gud = gu.to(DEV)
    # the scale kept from the forward pass, then one that saturates and one deep in the subnormal range
    s_fwd = oracle.scale(oracle.amax_bf16(want_h), fmt)
    for sc in (s_fwd, np.float32(s_fwd * 8.0), np.float32(s_fwd * 2.0 ** -12)):
        wq, wqt = oracle.quantize(want_h, sc, fmt)
        d_s = torch.tensor([float(sc)], dtype=torch.float32, device=DEV)
        q, qt, h = gpu_swiglu_fp8(gud, d_s, fmt, transpose=True, want_h=True)
        assert np.array_equal(q.cpu().numpy(), wq)
        assert np.array_equal(qt.cpu().numpy(), wqt)
        _assert_bits(h, want_h, "h")
        q2, none, none2 = gpu_swiglu_fp8(gud, d_s, fmt, transpose=False, want_h=False)
        assert none is None and none2 is None and torch.equal(q2, q)
        q3, qt3, none3 = gpu_swiglu_fp8(gud, d_s, fmt, transpose=True, want_h=False)
        assert none3 is None and torch.equal(q3, q) and torch.equal(qt3, qt)
        q4, none4, h4 = gpu_swiglu_fp8(gud, d_s, fmt, transpose=False, want_h=True)
        assert none4 is None and torch.equal(q4, q) and torch.equal(h4, h)
    # same bytes as the unfused path on the GPU: SwiGLU -> absmax -> quantize
    h, a, s = gpu_swiglu_fwd(gud, fmt)
    uq, uqt = gpu_quantize(h, s, fmt)
    q, qt, _ = gpu_swiglu_fp8(gud, s, fmt)
    assert torch.equal(q, uq) and torch.equal(qt, uqt)


@pytest.mark.parametrize("shape", SHAPES)
def test_backward_result_absmax_and_scale_bit_exact(shape):
    M, I = shape
    print("swiglu bwd M=%d I=%d" % shape, flush=True)
    gu, dh = _case(M, I, 1300 + M + I)
    want = oracle.swiglu_bwd(_bits_of(dh), _bits_of(gu))
    want_a = oracle.amax_bf16(want)
    for fmt in (1, 0):
        dgu, a, s = gpu_swiglu_bwd(dh.to(DEV), gu.to(DEV), fmt)
        _assert_bits(dgu, want, "dGU")
        assert f32_bits(a) == np_f32_bits(want_a)
        assert f32_bits(s) == np_f32_bits(oracle.scale(want_a, fmt))


def test_every_bf16_gate_value():
    """All finite BF16 patterns as the gate (non-finite ones replaced by zero), against several up / dh
    values, through the tuned kernels: exercises the clamp, the overflow of e^-g, subnormal quotients
    and subnormal / overflowing results."""
    bits = np.arange(1 << 16, dtype=np.uint16)
    bits[(bits & 0x7F80) == 0x7F80] = 0
    g = bits.reshape(256, 256)
    for uval, dval in [(1.0, 1.0), (-3.0, 2.0 ** -20), (2.0 ** -100, 2.0 ** 60), (1.5e38, -1.0), (0.0, 3.0)]:
        print("gate sweep u=%r dh=%r" % (uval, dval), flush=True)
        ub = _bits_of(torch.tensor([uval], dtype=torch.float32).to(torch.bfloat16))[0]
        db = _bits_of(torch.tensor([dval], dtype=torch.float32).to(torch.bfloat16))[0]
        gub = np.concatenate([g, np.full_like(g, ub)], axis=1)
        dhb = np.full_like(g, db)
        gu = torch.from_numpy(gub.view(np.int16)).view(torch.bfloat16).to(DEV)
        dh = torch.from_numpy(dhb.view(np.int16)).view(torch.bfloat16).to(DEV)
        want_h = oracle.swiglu_fwd(gub)
        h, a, s = gpu_swiglu_fwd(gu, 0)
        _assert_bits(h, want_h, "h")
        wa = oracle.amax_bf16(want_h)
        assert f32_bits(a) == np_f32_bits(wa) and f32_bits(s) == np_f32_bits(oracle.scale(wa, 0))
        want_d = oracle.swiglu_bwd(dhb, gub)
        dgu, a, s = gpu_swiglu_bwd(dh, gu, 1)
        _assert_bits(dgu, want_d, "dGU")
        wa = oracle.amax_bf16(want_d)
        assert f32_bits(a) == np_f32_bits(wa) and f32_bits(s) == np_f32_bits(oracle.scale(wa, 1))


def test_scale_from_amax_matches_the_absmax_call():
    for v in [0.0, 1.0, 3.3, 1e-38, 2.0 ** -140, 448.0, 57344.0, 7e37, float("inf")]:
        a = torch.tensor([v], dtype=torch.float32, device=DEV)
        for fmt in (0, 1):
            s = torch.full((1,), -1.0, device=DEV)
            llmq.llmq_scale_from_amax(a, fmt, s)
            assert f32_bits(s) == np_f32_bits(oracle.scale(np.float32(v), fmt)), (v, fmt)


def test_fused_bytes_feed_the_down_projection():
    """Recompute mode end to end: the FP8 copies written straight into the linear workspace give the same
    down-projection output as quantizing the BF16 SwiGLU result inside the linear call."""
    M, I, N = 256, 512, 384
    gu, _ = _case(M, I, 4242)
    gud = gu.to(DEV)
    g = torch.Generator(device="cpu").manual_seed(7)
    W = (torch.randn(N, I, generator=g) * 0.02).to(torch.bfloat16).to(DEV)
    h, a_h, s_h = gpu_swiglu_fwd(gud, 0)
    a_w, s_w = gpu_amax(W, 0)
    ws_bytes = llmq.llmq_fp8_linear_workspace_bytes(M, N, I)
    off = llmq.llmq_fp8_linear_workspace_offsets(M, N, I)
    ws1 = torch.zeros(ws_bytes, dtype=torch.uint8, device=DEV)
    y1 = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    llmq.llmq_fp8_linear_fwd(h, W, M, N, I, s_h, s_w, y1, None, ws1)
    ws2 = torch.zeros(ws_bytes, dtype=torch.uint8, device=DEV)
    y2 = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    llmq.llmq_swiglu_fwd_fp8(gud, s_h, 0, ws2[off[0]:off[0] + M * I], ws2[off[1]:off[1] + M * I], None)
    llmq.llmq_fp8_linear_fwd(None, W, M, N, I, s_h, s_w, y2, None, ws2, flags=llmq.REUSE_X)
    assert torch.equal(ws1, ws2) and torch.equal(y1, y2)


def test_config_shapes_at_full_size():
    """The SwiGLU of config 2 (3B-class, every output) and config 5 (32B-class, forward and recompute mode)
    at the sizes the benchmark times, whole tensors against the oracle."""
    for cfg_i, do_bwd in [(2, True), (5, False)]:
        cfg = synth.CONFIGS[cfg_i]
        M, I = synth.swiglu_dims(cfg)
        print("full-size swiglu config %d M=%d I=%d" % (cfg_i, M, I), flush=True)
        gu = synth.make_gu(cfg, device=DEV)
        gub = _bits_of(gu)
        want_h = oracle.swiglu_fwd(gub)
        wa = oracle.amax_bf16(want_h)
        h, a, s = gpu_swiglu_fwd(gu, 0)
        assert np.array_equal(_bits_of(h), want_h)
        assert f32_bits(a) == np_f32_bits(wa) and f32_bits(s) == np_f32_bits(oracle.scale(wa, 0))
        del h
        print("  recompute mode", flush=True)
        q, qt, _ = gpu_swiglu_fp8(gu, s, 0)
        wq, wqt = oracle.quantize(want_h, oracle.scale(wa, 0), 0)
        assert np.array_equal(q.cpu().numpy(), wq) and np.array_equal(qt.cpu().numpy(), wqt)
        assert (wq & 0x7F).max() == 0x7E
        del q, qt, wq, wqt, want_h
        if do_bwd:
            print("  backward", flush=True)
            dh = synth.make_dh(cfg, device=DEV)
            want = oracle.swiglu_bwd(_bits_of(dh), gub)
            wa = oracle.amax_bf16(want)
            dgu, a, s = gpu_swiglu_bwd(dh, gu, 1)
            assert np.array_equal(_bits_of(dgu), want)
            assert f32_bits(a) == np_f32_bits(wa) and f32_bits(s) == np_f32_bits(oracle.scale(wa, 1))
            del dgu, dh, want
        del gu, gub
        torch.cuda.empty_cache()


def test_argument_errors_leave_outputs_alone():
    gu = torch.zeros((8, 16), dtype=torch.bfloat16, device=DEV)
    h = torch.full((8, 8), 5.0, dtype=torch.bfloat16, device=DEV)
    a = torch.full((1,), -1.0, device=DEV)
    small = torch.zeros(2, dtype=torch.uint8, device=DEV)
    with pytest.raises(llmq.LlmqError) as e:
        llmq.llmq_swiglu_fwd(gu, h, 0, a, None, small)
    assert e.value.status == -5
    with pytest.raises(llmq.LlmqError) as e:
        llmq.llmq_swiglu_fwd(gu, h, 9, a, None, _ws(8, 8))
    assert e.value.status == -4
    torch.cuda.synchronize()
    assert a.item() == -1.0 and (h == 5.0).all()
