"""GPU parity: RMSNorm + residual addition with fused absmax, and the recompute path that emits FP8
directly.  The residual sum and everything downstream of a GIVEN row statistic is bit-exact against the
oracle; the row statistic itself (a binary32 sum in the kernel's order) and the forward y computed from
it are compared within the tolerance derived from the arithmetic."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import llmq, synth
from gpu_common import DEV, f32_bits, np_f32_bits, gpu_amax, gpu_quantize

pytestmark = pytest.mark.gpu

EPS = 1e-6
RSTD_TOL = 2.0 ** -20            # binary32 sum of <= 8192 squares by lanes + butterfly, division, root, division
# forward shapes: single-pass kernel (C % 8 == 0, C <= 8192), rows not filling a workgroup, generic C
FWD_SHAPES = [(8, 64), (5, 264), (64, 3072), (16, 8192), (130, 5120), (33, 17), (1, 1), (6, 8200), (3, 100)]
APPLY_SHAPES = [(32, 256), (64, 264), (16, 8), (36, 40), (4, 8), (33, 17), (1, 1), (48, 1032), (256, 3584), (128, 256), (384, 768)]


def _bits_of(t):
    return synth.bf16_bits(t)


def _f32(bits16):
    return (bits16.astype(np.uint32) << 16).view(np.float32)


def _case(M, C, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    res = (torch.randn(M, C, generator=g) * 1.3).to(torch.bfloat16)
    x = (torch.randn(M, C, generator=g) * 0.4).to(torch.bfloat16)
    w = (1.0 + 0.2 * torch.randn(C, generator=g)).to(torch.bfloat16)
    return res, x, w


def _half_ulp_bf16(v):
    a = np.maximum(np.abs(v), 2.0 ** -126)
    return 0.5 * 2.0 ** (np.floor(np.log2(a)) - 7)


def gpu_rmsnorm_fwd(res, x, w, fmt, in_place=False):
    M, C = res.shape
    res_d = res.to(DEV).clone()
    x_d = x.to(DEV) if x is not None else None
    res_out = res_d if in_place else (torch.full((M, C), -7.0, device=DEV, dtype=torch.bfloat16) if x is not None else None)
    y = torch.full((M, C), -7.0, device=DEV, dtype=torch.bfloat16)
    rstd = torch.full((M,), -1.0, device=DEV)
    a = torch.full((1,), -1.0, device=DEV)
    s = torch.full((1,), -1.0, device=DEV)
    ws = torch.full((llmq.llmq_rmsnorm_workspace_bytes(M),), 0xFF, device=DEV, dtype=torch.uint8)
    llmq.llmq_rmsnorm_fwd(res_d, x_d, w.to(DEV), EPS, res_out, y, rstd, fmt, a, s, ws)
    return res_out, y, rstd, a, s


def gpu_apply(res_d, w_d, rstd_d, d_scale, fmt, transpose=True, want_y=False):
    M, C = res_d.shape
    q = torch.full((M, C), 0xAA, device=DEV, dtype=torch.uint8)
    qt = torch.full((C, M), 0xAA, device=DEV, dtype=torch.uint8) if transpose else None
    y = torch.full((M, C), -7.0, device=DEV, dtype=torch.bfloat16) if want_y else None
    llmq.llmq_rmsnorm_apply_fp8(res_d, w_d, rstd_d, d_scale, fmt, q, qt, y)
    return q, qt, y


def _check_forward(res, x, w, res_out, y, rstd, a, s, fmt, what):
    new_bits = oracle.residual_add(_bits_of(res), _bits_of(x)) if x is not None else _bits_of(res)
    if x is not None:
        assert np.array_equal(_bits_of(res_out), new_bits), what + ": residual sum"
    want_rstd = oracle.rms_rstd(new_bits, EPS)
    got_rstd = rstd.cpu().numpy().astype(np.float64)
    assert (np.abs(got_rstd - want_rstd) <= RSTD_TOL * want_rstd).all(), what + ": rstd"
    want_y = oracle.rmsnorm_exact(new_bits, _bits_of(w), EPS)
    got_y = _f32(_bits_of(y)).astype(np.float64)
    # one rounding to BF16 of (res' * rstd) * w with rstd within RSTD_TOL and two binary32 multiplications
    bound = _half_ulp_bf16(want_y) * (1 + 2.0 ** -8) + np.abs(want_y) * (RSTD_TOL + 2.0 ** -22)
    bad = np.argwhere(np.abs(got_y - want_y) > bound)
    assert bad.size == 0, "%s: y out of tolerance at %s: got %r want %r" % (what, bad[0], got_y[tuple(bad[0])], want_y[tuple(bad[0])])
    # the fused absmax is the maximum of the tensor the kernel wrote, and so is what the separate pass gives
    assert float(a.item()) == float(np.abs(got_y).max()), what + ": absmax"
    a2, s2 = gpu_amax(y, fmt)
    assert f32_bits(a2) == f32_bits(a) and f32_bits(s2) == f32_bits(s), what + ": absmax/scale vs llmq_amax"
    # and within one BF16 step of the oracle's own absmax
    want_a = float(oracle.amax_bf16(oracle.rmsnorm_apply(new_bits, _bits_of(w), want_rstd.astype(np.float32))))
    assert abs(a.item() - want_a) <= 2.0 ** -7 * want_a, what + ": absmax vs oracle"
    return new_bits


@pytest.mark.parametrize("shape", FWD_SHAPES)
def test_forward_with_residual_addition(shape):
    M, C = shape
    print("rmsnorm fwd M=%d C=%d" % shape, flush=True)
    res, x, w = _case(M, C, 2000 + M + C)
    for fmt in (0, 1):
        res_out, y, rstd, a, s = gpu_rmsnorm_fwd(res, x, w, fmt)
        _check_forward(res, x, w, res_out, y, rstd, a, s, fmt, "fmt %d" % fmt)
    # in place: the residual stream is updated where it lives; same results
    r2, y2, rstd2, a2, s2 = gpu_rmsnorm_fwd(res, x, w, 1, in_place=True)
    assert torch.equal(r2, res_out) and torch.equal(y2, y) and torch.equal(rstd2, rstd) and f32_bits(a2) == f32_bits(a)
    # without the addition the input is normalised as it is and res_out is not needed
    none, y3, rstd3, a3, s3 = gpu_rmsnorm_fwd(res, None, w, 0)
    assert none is None
    _check_forward(res, None, w, None, y3, rstd3, a3, s3, 0, "no addition")
    # run to run reproducible
    _, y4, rstd4, a4, _ = gpu_rmsnorm_fwd(res, None, w, 0)
    assert torch.equal(y4, y3) and torch.equal(rstd4, rstd3) and f32_bits(a4) == f32_bits(a3)


@pytest.mark.parametrize("shape", APPLY_SHAPES)
@pytest.mark.parametrize("fmt", [0, 1])
def test_recompute_path_bit_exact(shape, fmt):
    M, C = shape
    print("rmsnorm apply_fp8 M=%d C=%d fmt=%d" % (M, C, fmt), flush=True)
    res, _, w = _case(M, C, 3000 + M + C)
    rb, wb = _bits_of(res), _bits_of(w)
    rstd = oracle.rms_rstd(rb, EPS).astype(np.float32)            # the statistic kept from the forward pass
    want_y = oracle.rmsnorm_apply(rb, wb, rstd)
    s_fwd = oracle.scale(oracle.amax_bf16(want_y), fmt)
    res_d, w_d = res.to(DEV), w.to(DEV)
    rstd_d = torch.from_numpy(rstd).to(DEV)
    for sc in (s_fwd, np.float32(s_fwd * 8.0), np.float32(s_fwd * 2.0 ** -12)):
        wq, wqt = oracle.quantize(want_y, sc, fmt)
        d_s = torch.tensor([float(sc)], dtype=torch.float32, device=DEV)
        q, qt, y = gpu_apply(res_d, w_d, rstd_d, d_s, fmt, True, True)
        assert np.array_equal(q.cpu().numpy(), wq) and np.array_equal(qt.cpu().numpy(), wqt)
        assert np.array_equal(_bits_of(y), want_y)
        q2, none, none2 = gpu_apply(res_d, w_d, rstd_d, d_s, fmt, False, False)
        assert none is None and none2 is None and torch.equal(q2, q)
        q3, qt3, _ = gpu_apply(res_d, w_d, rstd_d, d_s, fmt, True, False)
        assert torch.equal(q3, q) and torch.equal(qt3, qt)
        q4, _, y4 = gpu_apply(res_d, w_d, rstd_d, d_s, fmt, False, True)
        assert torch.equal(q4, q) and torch.equal(y4, y)


@pytest.mark.parametrize("shape", [(64, 3072), (48, 264), (33, 17)])
def test_forward_and_recompute_agree_on_the_gpu(shape):
    """Recomputation must reproduce the forward pass: with the statistics the forward kernel stored, the
    recompute kernel gives the same y and the same FP8 bytes as quantizing the forward's y."""
    M, C = shape
    res, x, w = _case(M, C, 4000 + M + C)
    res_out, y, rstd, a, s = gpu_rmsnorm_fwd(res, x, w, 0)
    uq, uqt = gpu_quantize(y, s, 0)
    q, qt, y2 = gpu_apply(res_out, w.to(DEV), rstd, s, 0, True, True)
    assert torch.equal(y2, y) and torch.equal(q, uq) and torch.equal(qt, uqt)


def test_special_rows():
    """An all-zero row (rstd = eps^-1/2, y = 0), a row with one huge outlier, a tiny row (eps dominates)."""
    C = 512
    res = torch.zeros((8, C), dtype=torch.bfloat16)
    res[1, 7] = 3.0e4
    res[2] = 1.0e-20
    res[3] = 1.0
    res[4, ::2] = -2.0
    res[4, 1::2] = 2.0
    w = torch.ones(C, dtype=torch.bfloat16)
    _, y, rstd, a, s = gpu_rmsnorm_fwd(res, None, w, 0)
    _check_forward(res, None, w, None, y, rstd, a, s, 0, "special rows")
    assert (y[0] == 0).all() and abs(rstd[0].item() - EPS ** -0.5) <= 1e-3
    assert abs(rstd[3].item() - 1.0) < 1e-5 and (y[3].float() - 1.0).abs().max() < 2.0 ** -8
    assert abs(rstd[4].item() - 0.5) < 1e-6 and y[4, 0].item() == -1.0 and y[4, 1].item() == 1.0


def test_config_shapes_at_full_size():
    """Hidden sizes and token counts of config 3 (7B-class, outlier channels) and config 5 (32B-class,
    heavy tails): forward with addition, then the recompute path on the oracle's statistics, whole tensors."""
    for cfg_i in (3, 5):
        cfg = synth.CONFIGS[cfg_i]
        res, x, w = synth.make_norm_inputs(cfg, device=DEV)
        M, C = res.shape
        print("full-size rmsnorm config %d M=%d C=%d" % (cfg_i, M, C), flush=True)
        res_c, x_c, w_c = res.cpu(), x.cpu(), w.cpu()
        res_out, y, rstd, a, s = gpu_rmsnorm_fwd(res_c, x_c, w_c, 0)
        new_bits = _check_forward(res_c, x_c, w_c, res_out, y, rstd, a, s, 0, "config %d" % cfg_i)
        print("  recompute path", flush=True)
        rstd32 = oracle.rms_rstd(new_bits, EPS).astype(np.float32)
        want_y = oracle.rmsnorm_apply(new_bits, _bits_of(w_c), rstd32)
        sc = oracle.scale(oracle.amax_bf16(want_y), 0)
        wq, wqt = oracle.quantize(want_y, sc, 0)
        q, qt, _ = gpu_apply(res_out, w, torch.from_numpy(rstd32).to(DEV),
                             torch.tensor([float(sc)], dtype=torch.float32, device=DEV), 0, True, False)
        assert np.array_equal(q.cpu().numpy(), wq) and np.array_equal(qt.cpu().numpy(), wqt)
        del res, x, res_out, y, q, qt
        torch.cuda.empty_cache()


def test_argument_errors():
    res = torch.zeros((8, 16), dtype=torch.bfloat16, device=DEV)
    w = torch.ones(16, dtype=torch.bfloat16, device=DEV)
    y = torch.full((8, 16), 5.0, dtype=torch.bfloat16, device=DEV)
    rstd = torch.zeros(8, device=DEV)
    a = torch.full((1,), -1.0, device=DEV)
    ws = torch.zeros(llmq.llmq_rmsnorm_workspace_bytes(8), dtype=torch.uint8, device=DEV)
    with pytest.raises(llmq.LlmqError) as e:      # x without a place for the sum
        llmq.llmq_rmsnorm_fwd(res, res, w, EPS, None, y, rstd, 0, a, None, ws)
    assert e.value.status == -1
    with pytest.raises(llmq.LlmqError) as e:
        llmq.llmq_rmsnorm_fwd(res, None, w, -1.0, None, y, rstd, 0, a, None, ws)
    assert e.value.status == -2
    with pytest.raises(llmq.LlmqError) as e:
        llmq.llmq_rmsnorm_fwd(res, None, w, EPS, None, y, rstd, 0, a, None, ws[:1])
    assert e.value.status == -5
    torch.cuda.synchronize()
    assert a.item() == -1.0 and (y == 5.0).all()
